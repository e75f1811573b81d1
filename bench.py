#!/usr/bin/env python3
"""Benchmark of the pdelta hot path on one MI355X.

One timed "step" = the decode workload of the 4096 x 4096 fp16 layer: row and column mode at
batch 1 and batch 16 (four launches), each launch on a different (W_b, B, v) buffer set so that
it streams from HBM rather than from the 256 MB memory-side cache.  `value` is the effective
bandwidth of those K steps: algorithmic bytes (every weight, sign word, scale, X and Y once)
divided by the time between two events on the launching stream around the replay of a HIP
graph that holds exactly those K steps (a call through the Python binding costs host time of the
order of a decode kernel's run time).  The same process then times,
each with its own events, the other workloads of the path (prefill GEMM shapes, the 224-linear
decode stack, the offline pack of that stack, the in-place patch) and the CPU oracle on a
bounded sample; they are reported as extra objects on the same JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--skip group,variants,prefill,grad,stack,pack,patch,cpu]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_PEAK_TFLOPS = 2500.0      # MI355X dense bf16 / fp16
METRIC = "delta-linear decode GB/s + prefill TFLOP/s, % of MI355X HBM/MFMA roofline"


def decode_bytes(d_out: int, d_in: int, M: int, axis: str) -> int:
    """Algorithmic HBM bytes of one decode launch: W_b, packed signs, v, X in, Y out (fp16)."""
    v_len = d_out if axis == "row" else d_in
    return 2 * d_out * d_in + d_out * d_in // 8 + 2 * v_len + 2 * M * d_in + 2 * M * d_out


def gpu_sysfs_info() -> dict:
    """Clock levels and partition modes of the first amdgpu card, read from sysfs (no child process:
    nothing is executed, so this also works under a profiler).  Entries are null when not exposed."""
    import glob
    out = {"sclk_MHz": None, "mclk_MHz": None, "compute_partition": None, "memory_partition": None}

    def read(path):
        try:
            with open(path) as f:
                return f.read().strip()
        except OSError:
            return None

    def levels(text):
        # lines like "1: 2400Mhz *": all levels, and the one marked current
        if not text:
            return None
        all_levels, current = [], None
        for line in text.splitlines():
            digits = "".join(ch for ch in line.split(":")[-1] if ch.isdigit())
            if digits:
                all_levels.append(int(digits))
                if "*" in line:
                    current = int(digits)
        return {"levels": all_levels, "current_when_idle": current} if all_levels else None

    for dev in sorted(glob.glob("/sys/class/drm/card[0-9]*/device")):
        if read(os.path.join(dev, "vendor")) != "0x1002":
            continue
        out["sclk_MHz"] = levels(read(os.path.join(dev, "pp_dpm_sclk")))
        out["mclk_MHz"] = levels(read(os.path.join(dev, "pp_dpm_mclk")))
        out["compute_partition"] = read(os.path.join(dev, "current_compute_partition"))
        out["memory_partition"] = read(os.path.join(dev, "current_memory_partition"))
        break
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--skip", type=str, default="")
    ap.add_argument("--sets", type=int, default=24, help="rotating buffer sets for the decode layer")
    ap.add_argument("--repeats", type=int, default=7, help="timed replays of the K-step graph (median reported)")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a plain elementwise copy of 1 GiB (reads 1 GiB, writes 1 GiB) so that "
                         "a rocprofv3 --pmc run of this command has a kernel of known traffic in it")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        return 2
    skip = set(s for s in args.skip.split(",") if s)

    import numpy as np
    import torch
    from paper_2512_19720_amd import binding as pd
    from paper_2512_19720_amd import synth

    pd.lib()                                   # fail loudly if the HIP library is not built
    dev = "cuda:0"
    torch.cuda.set_device(0)
    f16 = torch.float16

    if args.calibrate:
        src = torch.ones(1 << 29, dtype=f16, device=dev)          # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.mul(src, 1.0, out=dst)                            # one read + one write per element
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    def timed(fn, iters: int) -> float:
        """Milliseconds for `iters` calls of fn between two events on the current stream."""
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)

    def make_layer(d_out, d_in, dtype, sigma_axis, seed):
        """W_b plus pack(dW, 0) -> (W_b, B, v_row, v_col); the delta itself is dropped."""
        L = synth.layer_device(d_out, d_in, dtype, sigma_axis, seed, dev)
        B, v_row, v_col = pd.pdelta_pack(L["dW"], torch.zeros_like(L["dW"]))
        return L["W_b"], B, v_row, v_col

    # ---------------- decode: d_out = d_in = 4096, fp16, row/col x batch 1/16 ------------------
    N = K = 4096
    sets = [make_layer(N, K, synth.F16, "row" if s % 2 == 0 else "col", synth.seed_for(1, s))
            for s in range(args.sets)]
    X1 = synth.x_device(1, K, synth.F16, synth.seed_for(1, 900), dev)
    X16 = synth.x_device(16, K, synth.F16, synth.seed_for(1, 901), dev)
    Y1 = torch.empty((1, N), dtype=f16, device=dev)
    Y16 = torch.empty((16, N), dtype=f16, device=dev)
    cases = [("row", 1), ("col", 1), ("row", 16), ("col", 16)]
    rot = [0]

    def decode_call(axis, M):
        W_b, B, v_row, v_col = sets[rot[0] % len(sets)]
        rot[0] += 1
        X, Y = (X1, Y1) if M == 1 else (X16, Y16)
        if axis == "row":
            pd.pdelta_linear_row(X, W_b, B, v_row, out=Y)
        else:
            pd.pdelta_linear_col(X, W_b, B, v_col, out=Y)

    def decode_step():
        for axis, M in cases:
            decode_call(axis, M)

    step_bytes = sum(decode_bytes(N, K, M, axis) for axis, M in cases)

    def graph_of(fn, iters):
        """The launches of `iters` calls of fn recorded into one HIP graph (the library records
        plain kernel nodes only).  The Python binding needs 5 us and more of host time per call,
        of the order of a decode kernel's 9 us, so launching from Python can end up timing the host."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()                                           # outside capture first
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(iters):
                fn()
        return g

    for _ in range(args.warmup):                           # W untimed steps, launched eagerly
        decode_step()
    torch.cuda.synchronize()
    rot[0] = 0
    ms_eager = timed(decode_step, args.steps)              # the same K steps launched from Python
    rot[0] = 0
    g_steps = graph_of(decode_step, args.steps)            # exactly K steps, rotating buffer sets
    timed(g_steps.replay, 1)
    # the timed region: `repeats` replays of the K-step graph, each between its own pair of events
    # (sync, K steps, sync); the median replay is the reported one, min and max show the spread
    t_wall0 = time.perf_counter()
    replays_ms = sorted(timed(g_steps.replay, 1) for _ in range(max(args.repeats, 1)))
    wall_s = time.perf_counter() - t_wall0
    ms_total = replays_ms[len(replays_ms) // 2]
    ms_per_step = ms_total / args.steps
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    per_case = {}
    for axis, M in cases:
        g_case = graph_of(lambda: decode_call(axis, M), 200)
        timed(g_case.replay, 1)
        ms = sorted(timed(g_case.replay, 1) for _ in range(5))[2] / 200      # >= 100 calls, median of 5
        b = decode_bytes(N, K, M, axis)
        per_case[f"{axis}_M{M}"] = {"us": round(ms * 1e3, 3), "GB/s": round(b / ms / 1e6, 1),
                                    "frac_hbm": round(b / ms / 1e6 / HBM_PEAK_GBS, 4)}
        del g_case
    g_hot = graph_of(lambda: pd.pdelta_linear_row(X1, sets[0][0], sets[0][1], sets[0][2], out=Y1), 200)
    timed(g_hot.replay, 1)
    per_case["row_M1_cache_hot_single_buffer"] = {"us": round(timed(g_hot.replay, 1) / 200 * 1e3, 3)}
    per_case["launched_from_python_ms_per_step"] = round(ms_eager / args.steps, 5)
    del g_hot, g_steps

    # HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, scaled by the
    # plain-copy calibration); taken from the committed summary when it exists.
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "decode_4096x4096_pmc_traffic.md")
    if os.path.exists(tpath):
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = int(float(line.split(":", 1)[1].split()[0]))
                traffic_source = ("counter figure, not measured in this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                                  "of this same command, committed as profiles/decode_4096x4096_pmc_traffic.md")
    launches = args.steps * len(cases)
    avg_launch_us = ms_total * 1e3 / launches
    roofline = {"bound": "hbm", "kernel": "linear_skinny_kernel / linear_skinny_staged_kernel (decode, 4096x4096 fp16)",
                "achieved": round(value, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(value / HBM_PEAK_GBS, 4),
                "bytes_per_launch": step_bytes // len(cases),
                "avg_launch_us": round(avg_launch_us, 3), "traffic": traffic, "traffic_source": traffic_source}

    # what the box is, and what plain kernels reach on it ("% of achievable" next to "% of peak")
    props = torch.cuda.get_device_properties(0)
    device_info = {"name": props.name, "arch": getattr(props, "gcnArchName", ""),
                   "compute_units": props.multi_processor_count,
                   "memory_GiB": round(props.total_memory / 2 ** 30, 1)}
    device_info.update(gpu_sysfs_info())
    sink = torch.zeros(64, dtype=torch.uint8, device=dev)
    big = torch.empty(1 << 32, dtype=torch.uint8, device=dev)            # 4 GiB, read-only stream
    big.view(torch.int32).fill_(0x01020304)
    timed(lambda: pd.pdelta_probe_read_stream(big, sink), 2)
    rms = sorted(timed(lambda: pd.pdelta_probe_read_stream(big, sink), 3) / 3 for _ in range(3))[1]
    # the same read-only kernel on pieces of the decode layer's size (35.7 MB per launch, 24 distinct
    # pieces): what a launch of that size can reach at best, ramp-up and drain included
    piece = step_bytes // len(cases) // 256 * 256
    pieces = [big[i * piece:(i + 1) * piece] for i in range(24)]
    prot = [0]

    def piece_read():
        pd.pdelta_probe_read_stream(pieces[prot[0] % 24], sink)
        prot[0] += 1

    g_piece = graph_of(piece_read, 200)
    timed(g_piece.replay, 1)
    pms = sorted(timed(g_piece.replay, 1) for _ in range(5))[2] / 200
    del g_piece, pieces
    csrc = big[:1 << 30].view(f16)                                       # 1 GiB
    cdst = torch.empty_like(csrc)
    timed(lambda: torch.mul(csrc, 1.0, out=cdst), 3)
    cms = timed(lambda: torch.mul(csrc, 1.0, out=cdst), 10) / 10
    ceiling = {"read_only_stream_4GiB": {"kind": "pdelta_probe_read_stream: 16-byte loads, every byte once, no writes",
                                         "GB/s": round((1 << 32) / rms / 1e6, 1),
                                         "frac_hbm": round((1 << 32) / rms / 1e6 / HBM_PEAK_GBS, 4)},
               "read_only_stream_per_launch_of_decode_layer_size": {
                   "bytes_per_launch": piece, "us": round(pms * 1e3, 3), "GB/s": round(piece / pms / 1e6, 1),
                   "frac_hbm": round(piece / pms / 1e6 / HBM_PEAK_GBS, 4),
                   "note": "the floor of any kernel launched once per 4096 x 4096 layer on this box"},
               "copy_1GiB": {"kind": "torch elementwise copy of 1 GiB (1 GiB read + 1 GiB written)",
                             "GB/s": round(2 * (1 << 30) / cms / 1e6, 1),
                             "frac_hbm": round(2 * (1 << 30) / cms / 1e6 / HBM_PEAK_GBS, 4)}}
    del csrc, cdst, big
    torch.cuda.empty_cache()
    mfma_ceiling = {"kind": "pdelta_probe_mfma: 256 workgroups, v_mfma_f32_32x32x16_f16 only"}
    for wps in (1, 2):
        for rnd in (False, True):
            fl = pd.pdelta_probe_mfma(wps, rnd, 2000, sink)
            mms = timed(lambda: pd.pdelta_probe_mfma(wps, rnd, 20000, sink), 2) / 2
            mfma_ceiling[f"{wps}_waves_per_simd_{'random' if rnd else 'constant'}_operands_TFLOP/s"] = round(
                fl * 10 / mms / 1e9, 1)

    out = {
        "metric": METRIC, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "config1: decode GEMV d_out=d_in=4096 fp16, row+col x M in {1,16}, "
                               f"{args.sets} rotating buffer sets ({args.sets * 35.7:.0f} MB), "
                               "the K steps replayed from one HIP graph",
                   "bytes_per_step": step_bytes},
        "roofline": roofline, "decode_cases": per_case, "wall_s_timed_region": round(wall_s, 4),
        "timed_replays": {"count": len(replays_ms), "ms_per_step_min": round(replays_ms[0] / args.steps, 5),
                          "ms_per_step_median": round(ms_per_step, 5),
                          "ms_per_step_max": round(replays_ms[-1] / args.steps, 5)},
        "device": device_info, "achieved_ceiling": ceiling, "mfma_ceiling": mfma_ceiling,
    }
    # ---------------- blockwise and scalar scales on the same decode layer ----------------------
    if "group" not in skip:
        res = {"workload": "decode GEMV 4096x4096 fp16, M = 1, scales per (row, block of 128 inputs) / one scalar per matrix; "
                           f"{args.sets} rotating buffer sets", "entry_point": "pdelta_linear_group"}
        for name, group, shared in (("group_128", 128, False), ("scalar", K, True)):
            n_groups = K // group
            vg = torch.full((1 if shared else N, n_groups), 1e-3, dtype=f16, device=dev)
            grot = [0]

            def group_call():
                W_b, B, _, _ = sets[grot[0] % len(sets)]
                grot[0] += 1
                pd.pdelta_linear_group(X1, W_b, B, vg, group, out=Y1)

            gg = graph_of(group_call, 200)
            timed(gg.replay, 1)
            ms = sorted(timed(gg.replay, 1) for _ in range(5))[2] / 200
            gb = 2 * N * K + N * K // 8 + 2 * vg.numel() + 2 * K + 2 * N
            res[name] = {"us": round(ms * 1e3, 3), "GB/s": round(gb / ms / 1e6, 1),
                         "frac_hbm": round(gb / ms / 1e6 / HBM_PEAK_GBS, 4)}
            del gg
        out["group_scales"] = res

    # ---------------- multi-variant decode: R requests share W_b, each has its own delta -------
    if "variants" not in skip:
        R, nsets = 16, 12                       # 12 x (32 MiB W_b + 16 x 2 MiB signs) = 768 MiB
        gen = torch.Generator(device=dev)
        gen.manual_seed(synth.seed_for(1, 950))
        XR = synth.x_device(R, K, synth.F16, synth.seed_for(1, 951), dev)
        YR = torch.empty((R, N), dtype=f16, device=dev)
        vsets = []
        for si in range(nsets):
            signs = [torch.randint(-2 ** 31, 2 ** 31 - 1, (N, K // 32), dtype=torch.int32, device=dev, generator=gen)
                     for _ in range(R)]
            vsets.append((sets[si][0], pd.VariantSet([(signs[r], sets[(si + r) % len(sets)][2]) for r in range(R)], pd.ROW)))
        vrot = [0]

        def variants_call():
            W_b, vs = vsets[vrot[0] % nsets]
            vrot[0] += 1
            pd.pdelta_linear_variants(XR, W_b, vs, out=YR)

        def separate_calls():
            W_b, vs = vsets[vrot[0] % nsets]
            vrot[0] += 1
            for r in range(R):
                pd.pdelta_linear_row(XR[r:r + 1], W_b, vs.tensors[r][0], vs.tensors[r][1], out=YR[r:r + 1])

        vbytes = 2 * N * K + R * (N * K // 8 + 2 * N + 2 * K + 2 * N)
        timed(variants_call, 20)
        msv = timed(variants_call, 120) / 120
        timed(separate_calls, 2)
        mss = timed(separate_calls, 12) / 12
        out["variants"] = {"workload": f"{R} requests x 1 token, one 4096x4096 fp16 base, {R} sign/scale sets, row mode; "
                                       f"{nsets} rotating buffer sets",
                           "entry_point": "pdelta_linear_variants", "bytes_per_call": vbytes,
                           "us": round(msv * 1e3, 2), "GB/s": round(vbytes / msv / 1e6, 1),
                           "frac_hbm": round(vbytes / msv / 1e6 / HBM_PEAK_GBS, 4),
                           "same_work_as_16_single_calls_us": round(mss * 1e3, 2)}
        # fewer requests on the same base: 2 + R / 8 bytes per weight
        fewer = {}
        for Rs in (4, 8):
            sub = [(W_b, pd.VariantSet(vs.tensors[:Rs], pd.ROW)) for W_b, vs in vsets]
            Xs_, Ys_ = XR[:Rs], YR[:Rs]

            def sub_call():
                W_b, vs = sub[vrot[0] % nsets]
                vrot[0] += 1
                pd.pdelta_linear_variants(Xs_, W_b, vs, out=Ys_)

            sb = 2 * N * K + Rs * (N * K // 8 + 2 * N + 2 * K + 2 * N)
            timed(sub_call, 20)
            mssub = timed(sub_call, 120) / 120
            fewer[f"R={Rs}"] = {"bytes_per_call": sb, "us": round(mssub * 1e3, 2), "GB/s": round(sb / mssub / 1e6, 1),
                                "frac_hbm": round(sb / mssub / 1e6 / HBM_PEAK_GBS, 4)}
            del sub
        out["variants"]["fewer_requests"] = fewer
        del vsets, XR, YR
    del sets
    torch.cuda.empty_cache()

    # ---------------- prefill: bf16, M = 2048, three MLP shapes, row scales --------------------
    if "prefill" not in skip:
        pre = {}
        group_prefill = None
        prefill_parts = None
        tot_flop, tot_ms = 0.0, 0.0
        M = 2048
        for d_out, d_in in synth.PREFILL_SHAPES:
            W_b, B, v_row, _ = make_layer(d_out, d_in, synth.BF16, "row", synth.seed_for(2, d_out % 1000))
            X = synth.x_device(M, d_in, synth.BF16, synth.seed_for(2, 7), dev)
            Y = torch.empty((M, d_out), dtype=torch.bfloat16, device=dev)
            fn = lambda: pd.pdelta_linear_row(X, W_b, B, v_row, out=Y)
            # The layer was just generated and packed: the first launches after that run at a
            # lower clock.  30 untimed calls (about 8 ms), then the median of five runs of 20.
            timed(fn, 30)
            runs = sorted(timed(fn, 20) / 20 for _ in range(5))
            ms = runs[2]
            flop = 2.0 * M * d_out * d_in
            pre[f"{d_out}x{d_in}"] = {"us": round(ms * 1e3, 1), "us_min": round(runs[0] * 1e3, 1),
                                      "us_max": round(runs[-1] * 1e3, 1),
                                      "TFLOP/s": round(flop / ms / 1e9, 1),
                                      "frac_mfma": round(flop / ms / 1e9 / MFMA_PEAK_TFLOPS, 4)}
            tot_flop += flop
            tot_ms += ms
            if (d_out, d_in) == synth.PREFILL_SHAPES[0]:
                # where the launch spends its time: the same kernel with parts of its loop compiled out
                # (pdelta_probe_prefill_parts; mask 15 is the product kernel)
                parts = {}
                for mask in pd.PREFILL_PARTS_BUILT:
                    fp = lambda: pd.pdelta_probe_prefill_parts(mask, X, W_b, B, v_row, Y)
                    timed(fp, 10)
                    msp = sorted(timed(fp, 20) / 20 for _ in range(3))[1]
                    kept = [name for name, bit in pd.PREFILL_PARTS.items() if mask & bit]
                    parts[str(mask)] = {"kept": kept or ["nothing (barriers and epilogue only)"], "us": round(msp * 1e3, 1)}
                prefill_parts = {"workload": f"{d_out}x{d_in}, bf16, M = {M}, row scales; linear_gemm_pipe_kernel "
                                             "with parts of its loop compiled out", "masks": parts}
            if (d_out, d_in) == synth.PREFILL_SHAPES[0] and "group" not in skip:
                # the same layer with one scale per (row, block of 128 inputs): reported, not in the aggregate
                vg = torch.full((d_out, d_in // 128), 1e-3, dtype=torch.float16, device=dev)
                fg = lambda: pd.pdelta_linear_group(X, W_b, B, vg, 128, out=Y)
                timed(fg, 30)
                msg = sorted(timed(fg, 20) / 20 for _ in range(5))[2]
                group_prefill = {"workload": f"{d_out}x{d_in}, bf16, M = {M}, scales per (row, block of 128 inputs)",
                                 "us": round(msg * 1e3, 1), "TFLOP/s": round(flop / msg / 1e9, 1),
                                 "frac_mfma": round(flop / msg / 1e9 / MFMA_PEAK_TFLOPS, 4)}
                del vg
            del W_b, B, v_row, X, Y
        agg = tot_flop / tot_ms / 1e9
        out["prefill"] = {"workload": "config2: bf16 X [2048, d_in], row scales, bf16 Y; per shape the median of 5 runs of 20 calls", "shapes": pre,
                          "TFLOP/s": round(agg, 1)}
        if group_prefill is not None:
            out["prefill"]["blockwise_scales"] = group_prefill
        out["prefill"]["parts"] = prefill_parts
        out["roofline_prefill"] = {"bound": "mfma", "kernel": "linear_gemm_pipe_kernel (prefill, bf16 in, fp16 MFMA)",
                                   "achieved": round(agg, 1), "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                                   "frac": round(agg / MFMA_PEAK_TFLOPS, 4), "traffic": None}
        torch.cuda.empty_cache()

    # ---------------- backward with respect to v: M = 2048 tokens, 4096 x 4096, bf16 -----------
    if "grad" not in skip:
        Mg, Ng, Kg = 2048, 4096, 4096
        Xg = synth.x_device(Mg, Kg, synth.BF16, synth.seed_for(2, 70), dev)
        dYg = synth.x_device(Mg, Ng, synth.BF16, synth.seed_for(2, 71), dev)
        Bg = torch.randint(-2 ** 31, 2 ** 31 - 1, (Ng, Kg // 32), dtype=torch.int32, device=dev)
        res = {"workload": "dL/dv from dY: 2048 tokens, 4096 x 4096 layer, bf16 X and dY, fp32 gradient"}
        for name, axis in (("row", pd.ROW), ("col", pd.COL)):
            ws = torch.empty(pd.pdelta_grad_v_workspace_bytes(Mg, Ng, Kg, axis), dtype=torch.uint8, device=dev)
            outg = torch.empty(Ng if axis == pd.ROW else Kg, dtype=torch.float32, device=dev)
            fn = lambda: pd.pdelta_grad_v(Xg, dYg, Bg, axis, out=outg, workspace=ws)
            timed(fn, 3)
            ms = timed(fn, 20) / 20
            flop = 2.0 * Mg * Ng * Kg
            res[name] = {"us": round(ms * 1e3, 1), "TFLOP/s": round(flop / ms / 1e9, 1),
                         "frac_mfma": round(flop / ms / 1e9 / MFMA_PEAK_TFLOPS, 4)}
        out["grad_v"] = res
        del Xg, dYg, Bg
        torch.cuda.empty_cache()

    # ---------------- stack: 224 linears of a 7B-shaped model, batch 1 -------------------------
    layers = None
    if "stack" not in skip or "pack" not in skip or "patch" not in skip:
        shapes = synth.stack_shapes()
        layers = []
        for li, (name, d_out, d_in, axis) in enumerate(shapes):
            W_b, B, v_row, v_col = make_layer(d_out, d_in, synth.F16, axis, synth.seed_for(3, li))
            layers.append((d_out, d_in, axis, W_b, B, v_row if axis == "row" else v_col))
        Xs = {4096: synth.x_device(1, 4096, synth.F16, synth.seed_for(3, 900), dev),
              11008: synth.x_device(1, 11008, synth.F16, synth.seed_for(3, 901), dev)}
        Ys = [torch.empty((1, l[0]), dtype=f16, device=dev) for l in layers]
        torch.cuda.synchronize()

    if "stack" not in skip:
        def stack_pass():
            for (d_out, d_in, axis, W_b, B, v), Y in zip(layers, Ys):
                if axis == "row":
                    pd.pdelta_linear_row(Xs[d_in], W_b, B, v, out=Y)
                else:
                    pd.pdelta_linear_col(Xs[d_in], W_b, B, v, out=Y)

        stack_bytes = sum(decode_bytes(l[0], l[1], 1, l[2]) for l in layers)
        timed(stack_pass, 2)
        ms = timed(stack_pass, 10) / 10
        res = {"workload": "config3: 224 linears (32 x q,k,v,o,gate,up,down), fp16, M=1, row/col by block",
               "bytes_per_token": stack_bytes, "ms_per_token": round(ms, 4),
               "tokens/s": round(1e3 / ms, 1), "GB/s": round(stack_bytes / ms / 1e6, 1),
               "frac_hbm": round(stack_bytes / ms / 1e6 / HBM_PEAK_GBS, 4)}
        # same launches replayed from a HIP graph (no host launch gaps)
        try:
            g = torch.cuda.CUDAGraph()
            s = torch.cuda.Stream()
            s.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(s):
                stack_pass()
            torch.cuda.current_stream().wait_stream(s)
            with torch.cuda.graph(g):
                stack_pass()
            timed(g.replay, 2)
            msg = timed(g.replay, 10) / 10
            res["graph"] = {"ms_per_token": round(msg, 4), "tokens/s": round(1e3 / msg, 1),
                            "frac_hbm": round(stack_bytes / msg / 1e6 / HBM_PEAK_GBS, 4)}
        except Exception as exc:  # graph capture is an extra; the stream figure stands on its own
            res["graph"] = {"error": str(exc)[:200]}
        # the same per-layer launches, but recorded on 8 forked streams so that the graph knows the
        # layers are independent (they are here: each has its own X and Y) and may overlap them
        try:
            branches = [torch.cuda.Stream() for _ in range(8)]

            def stack_pass_forked():
                main = torch.cuda.current_stream()
                for b in branches:
                    b.wait_stream(main)
                for li, ((d_out, d_in, axis, W_b, B, v), Y) in enumerate(zip(layers, Ys)):
                    with torch.cuda.stream(branches[li % len(branches)]):
                        if axis == "row":
                            pd.pdelta_linear_row(Xs[d_in], W_b, B, v, out=Y)
                        else:
                            pd.pdelta_linear_col(Xs[d_in], W_b, B, v, out=Y)
                for b in branches:
                    main.wait_stream(b)

            stack_pass_forked()
            torch.cuda.synchronize()
            gp = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gp):
                stack_pass_forked()
            timed(gp.replay, 2)
            msp = timed(gp.replay, 10) / 10
            res["graph_8_branches"] = {"ms_per_token": round(msp, 4), "tokens/s": round(1e3 / msp, 1),
                                       "frac_hbm": round(stack_bytes / msp / 1e6 / HBM_PEAK_GBS, 4)}
            del gp
        except Exception as exc:
            res["graph_8_branches"] = {"error": str(exc)[:200]}
        # the same 224 layers through the batched entry point: one launch instead of 224
        ROW_COL = {"row": pd.ROW, "col": pd.COL}
        plan = pd.pdelta_linear_batch_plan(
            [(Xs[d_in], W_b, B, v, ROW_COL[axis], Y) for (d_out, d_in, axis, W_b, B, v), Y in zip(layers, Ys)])
        timed(lambda: pd.pdelta_linear_batch(plan), 2)
        msb = timed(lambda: pd.pdelta_linear_batch(plan), 10) / 10
        res["batched"] = {"entry_point": "pdelta_linear_batch", "ms_per_token": round(msb, 4),
                          "tokens/s": round(1e3 / msb, 1),
                          "frac_hbm": round(stack_bytes / msb / 1e6 / HBM_PEAK_GBS, 4)}
        del plan
        out["stack"] = res

    # ---------------- pack: offline pass over the same 224 shapes ------------------------------
    if "pack" not in skip:
        # W_f = round(W_b + dW) per layer with 5 % exact zeros in dW; 13 GB more of HBM
        Wfs = []
        for li, (d_out, d_in, axis, W_b, _, _) in enumerate(layers):
            L = synth.layer_device(d_out, d_in, synth.F16, "row", synth.seed_for(4, li), dev, zero_frac=0.05)
            Wfs.append((W_b.float() + L["dW"].float()).to(f16))
            del L
        outs = [(torch.empty((l[0], l[1] // 32), dtype=torch.int32, device=dev),
                 torch.empty(l[0], dtype=f16, device=dev), torch.empty(l[1], dtype=f16, device=dev))
                for l in layers]
        ws = torch.empty(pd.pdelta_pack_workspace_bytes(11008, 11008), dtype=torch.uint8, device=dev)

        def pack_pass():
            for l, Wf, o in zip(layers, Wfs, outs):
                pd.pdelta_pack(Wf, l[3], out=o, workspace=ws)

        pack_bytes = sum(4 * l[0] * l[1] + l[0] * l[1] // 8 + 2 * (l[0] + l[1]) for l in layers)
        timed(pack_pass, 1)
        ms = timed(pack_pass, 5) / 5
        out["pack"] = {"workload": "config4: pdelta_pack over the 224 layers, fp16, 5% zero deltas, v_row + v_col",
                       "bytes": pack_bytes, "ms": round(ms, 3), "GB/s": round(pack_bytes / ms / 1e6, 1),
                       "frac_hbm": round(pack_bytes / ms / 1e6 / HBM_PEAK_GBS, 4)}
        # the same 224 layers through the model-wide entry point: two launches instead of 448
        pplan = pd.pdelta_pack_batch_plan([(Wf, l[3]) for l, Wf in zip(layers, Wfs)], out=outs)
        timed(lambda: pd.pdelta_pack_batch(pplan), 1)
        msb = timed(lambda: pd.pdelta_pack_batch(pplan), 5) / 5
        out["pack"]["batched"] = {"entry_point": "pdelta_pack_batch", "ms": round(msb, 3),
                                  "GB/s": round(pack_bytes / msb / 1e6, 1),
                                  "frac_hbm": round(pack_bytes / msb / 1e6 / HBM_PEAK_GBS, 4)}
        del Wfs, outs, pplan
        torch.cuda.empty_cache()

    # ---------------- patch: merge the delta into all 224 layers, in place ---------------------
    if "patch" not in skip:
        # The merge runs in place on the resident base weights (the hot-swap of a fine-tune); a
        # second pass with negated scales takes it out again.  Out-of-place into one reused
        # buffer would let the 256 MB memory-side cache absorb the writes and overstate the rate.
        ROW_COL = {"row": pd.ROW, "col": pd.COL}
        negs = [-l[5] for l in layers]

        def patch_pass(scales):
            for (d_out, d_in, axis, W_b, B, v), s in zip(layers, scales):
                pd.pdelta_patch(W_b, B, s, ROW_COL[axis], out=W_b)

        def swap_pass_layerwise():
            patch_pass([l[5] for l in layers])
            patch_pass(negs)

        patch_bytes = sum(4 * l[0] * l[1] + l[0] * l[1] // 8 for l in layers)
        timed(swap_pass_layerwise, 1)
        ms = timed(swap_pass_layerwise, 3) / 6
        out["patch"] = {"workload": "pdelta_patch in place over the 224 layers (read W_b + signs, write W_b), fp16; "
                                    "merge and un-merge passes alternate",
                        "bytes": patch_bytes, "ms": round(ms, 3), "GB/s": round(patch_bytes / ms / 1e6, 1),
                        "frac_hbm": round(patch_bytes / ms / 1e6 / HBM_PEAK_GBS, 4)}
        # the same through the model-wide entry point: one launch per model swap
        swap_in = pd.pdelta_patch_batch_plan([(W_b, B, v, ROW_COL[axis], W_b) for (_, _, axis, W_b, B, v) in layers])
        swap_out = pd.pdelta_patch_batch_plan([(l[3], l[4], n, ROW_COL[l[2]], l[3]) for l, n in zip(layers, negs)])

        def swap_pass():
            pd.pdelta_patch_batch(swap_in)
            pd.pdelta_patch_batch(swap_out)

        timed(swap_pass, 1)
        msb = timed(swap_pass, 3) / 6
        out["patch"]["batched"] = {"entry_point": "pdelta_patch_batch", "ms_per_model_swap": round(msb, 3),
                                   "GB/s": round(patch_bytes / msb / 1e6, 1),
                                   "frac_hbm": round(patch_bytes / msb / 1e6 / HBM_PEAK_GBS, 4)}
        # Hot-swap from host memory: the packed delta of the whole model (signs + scales, one
        # contiguous pinned buffer) goes to the GPU in ONE copy and is merged by one launch - the
        # paper's loader (packed deltas transferred in a single operation, then applied on the
        # base).  The host leg is PCIe-bound and is reported separately; it is never `value`.
        try:
            pieces, offs, total = [], [], 0
            for (_, _, axis, W_b, B, v) in layers:
                for t in (B, v):
                    nbytes = t.numel() * t.element_size()
                    offs.append((total, nbytes))
                    total += (nbytes + 255) & ~255
            flat_dev = torch.empty(total, dtype=torch.uint8, device=dev)
            flat_host = torch.empty(total, dtype=torch.uint8, pin_memory=True)
            views = []
            k = 0
            for (_, _, axis, W_b, B, v) in layers:
                vb = flat_dev[offs[k][0]: offs[k][0] + offs[k][1]].view(torch.int32).view(B.shape)
                vv = flat_dev[offs[k + 1][0]: offs[k + 1][0] + offs[k + 1][1]].view(f16).view(v.shape)
                vb.copy_(B)
                vv.copy_(v)
                views.append((W_b, vb, vv, ROW_COL[axis], W_b))
                k += 2
            flat_host.copy_(flat_dev)
            torch.cuda.synchronize()
            from_host = pd.pdelta_patch_batch_plan(views)

            def swap_from_host():
                flat_dev.copy_(flat_host, non_blocking=True)
                pd.pdelta_patch_batch(from_host)

            swap_from_host()
            pd.pdelta_patch_batch(swap_out)
            msh = 0.0
            for _ in range(3):
                msh += timed(swap_from_host, 1)
                pd.pdelta_patch_batch(swap_out)             # untimed: back to the base weights
            msh /= 3
            out["patch"]["swap_from_pinned_host"] = {
                "delta_bytes": total, "ms": round(msh, 3),
                "note": "one host-to-device copy of the packed delta (PCIe) + one pdelta_patch_batch launch"}
            del flat_dev, flat_host, views, from_host
        except Exception as exc:
            out["patch"]["swap_from_pinned_host"] = {"error": str(exc)[:200]}
        del swap_in, swap_out, negs
    layers = None
    torch.cuda.empty_cache()

    # ---------------- CPU oracle on bounded samples of the workloads ---------------------------
    if "cpu" not in skip:
        import ctypes
        import platform
        from oracle import pdelta_oracle as orc
        all_threads = orc.threads()

        def set_threads(n):
            ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))

        cpu_model = platform.processor() or ""
        try:
            for line in open("/proc/cpuinfo"):
                if line.startswith("model name"):
                    cpu_model = line.split(":", 1)[1].strip()
                    break
        except OSError:
            pass
        L = synth.layer_host(N, K, 16, synth.F16, "row", synth.seed_for(1, 0))
        Bo, vr, vc = orc.pack(L["dW"], np.zeros_like(L["dW"]))

        def decode_pass():
            for axis, M in cases:
                orc.linear(L["X"][:M], L["W_b"], Bo, vr if axis == "row" else vc,
                           orc.ROW if axis == "row" else orc.COL)

        reps = 0
        t0 = time.perf_counter()
        while reps < 2 or (time.perf_counter() - t0 < 10.0 and reps < 16):     # about 10 s of CPU work
            decode_pass()
            reps += 1
        dt = time.perf_counter() - t0
        set_threads(1)
        t0 = time.perf_counter()
        decode_pass()
        dt1 = time.perf_counter() - t0
        set_threads(all_threads)
        cpu = {"value": round(reps * step_bytes / dt / 1e9, 4), "unit": "GB/s", "cores": all_threads, "kind": "oracle",
               "sample": f"{reps} passes of the same 4-launch decode step on one buffer set "
                         f"(fp64, dense W_hat rebuilt per call), {dt:.1f} s",
               "one_thread": {"value": round(step_bytes / dt1 / 1e9, 4), "unit": "GB/s", "cores": 1,
                              "sample": f"1 pass of the decode step, {dt1:.1f} s"},
               "cpu_model": cpu_model, "nproc": os.cpu_count()}
        # configs 2-4: one layer or shape of each kind, scaled to the whole workload (stated per entry)
        other = {}
        Lp = synth.layer_host(4096, 4096, 32, synth.BF16, "row", synth.seed_for(2, 1))
        Bp, vp, _ = orc.pack(Lp["dW"], np.zeros_like(Lp["dW"]), orc.BF16, want_col=False)
        t0 = time.perf_counter()
        orc.linear(Lp["X"], Lp["W_b"], Bp, vp, orc.ROW, orc.BF16)
        dtp = time.perf_counter() - t0
        flop_sample = 2.0 * 32 * 4096 * 4096
        flop_cfg2 = sum(2.0 * 2048 * o * i for o, i in synth.PREFILL_SHAPES)
        other["config2_prefill"] = {"GFLOP/s": round(flop_sample / dtp / 1e9, 2), "cores": all_threads,
                                    "sample": f"32 tokens x one 4096 x 4096 bf16 layer, {dtp:.2f} s",
                                    "whole_workload_s_scaled": round(dtp * flop_cfg2 / flop_sample, 1)}
        t3 = 0.0
        for d_out, d_in, count in ((4096, 4096, 128), (11008, 4096, 64), (4096, 11008, 32)):
            Ls = L if (d_out, d_in) == (4096, 4096) else synth.layer_host(d_out, d_in, 1, synth.F16, "row", synth.seed_for(3, d_out))
            Bs, vs, _ = (Bo, vr, None) if Ls is L else orc.pack(Ls["dW"], np.zeros_like(Ls["dW"]), want_col=False)
            t0 = time.perf_counter()
            orc.linear(Ls["X"][:1], Ls["W_b"], Bs, vs, orc.ROW)
            t3 += (time.perf_counter() - t0) * count
        other["config3_stack"] = {"tokens/s": round(1.0 / t3, 4), "cores": all_threads,
                                  "sample": "one layer of each of the three shapes, M = 1, scaled by their counts "
                                            f"(128 / 64 / 32): {t3:.1f} s per token"}
        Lw = synth.layer_host(4096, 4096, 1, synth.F16, "row", synth.seed_for(4, 0), zero_frac=0.05, with_wf=True)
        t0 = time.perf_counter()
        orc.pack(Lw["W_f"], Lw["W_b"])
        dtk = time.perf_counter() - t0
        pack_sample_bytes = 4 * 4096 * 4096 + 4096 * 4096 // 8 + 4 * 4096
        total_weights = sum(o * i for _, o, i, _ in synth.stack_shapes())
        other["config4_pack"] = {"GB/s": round(pack_sample_bytes / dtk / 1e9, 3), "cores": 1,
                                 "sample": f"one 4096 x 4096 fp16 pair (the oracle's pack loops are serial), {dtk:.2f} s",
                                 "whole_workload_s_scaled": round(dtk * total_weights / (4096 * 4096), 1)}
        cpu["other_configs"] = other
        out["cpu_baseline"] = cpu

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
