"""GPU parity at the benchmark's full size: the 224-layer, 7B-shaped stack through the three
model-wide entry points exactly as bench.py launches them (one descriptor array of 224 records
per call), checked layer by layer against the CPU oracle on sampled rows and columns.

  pdelta_pack_batch    W_f = round(W_b + dW), 5 % exact zeros in dW, fp16: packed words and v_row
                       on sampled rows (the oracle packs those rows), v_col on sampled blocks of
                       32 columns (the oracle packs all rows of those columns)
  pdelta_linear_batch  one token per layer, fp16 in and out, even blocks row mode / odd blocks
                       column mode: sampled outputs, one fp64 dot product each by the oracle
  pdelta_patch_batch   in-place merge of the whole stack: sampled rows bit for bit

Sampled rows always include the first and last rows of a layer and rows on both sides of the
16-row workgroup boundary; the first and the last layer of the stack are sampled like every
other layer.  Oracle inputs never come from the GPU: signs and row scales are packed by the
oracle from the same synthetic rows, and the column-mode layers use a scale vector drawn on the
host (the GPU's own v_col is checked separately, on the sampled column blocks).
"""
import numpy as np
import pytest
import torch

from oracle import pdelta_oracle as orc
from paper_2512_19720_amd import binding as pd
from paper_2512_19720_amd import synth
from parity_util import DEV, check_y, f16_dev, words_host

pytestmark = pytest.mark.gpu

ROWS_PER_LAYER = 16
COL_BLOCKS_PER_LAYER = 3


def sample_rows(rng, d_out):
    fixed = [0, 1, 15, 16, d_out - 17, d_out - 16, d_out - 1]
    extra = rng.integers(0, d_out, ROWS_PER_LAYER - len(fixed))
    return np.unique(np.concatenate([fixed, extra]))


@pytest.fixture(scope="module")
def stack():
    """The stack of bench.py's offline-pack and decode workloads, resident on the GPU, plus the
    host copies of the sampled rows and column blocks taken BEFORE anything is merged."""
    shapes = synth.stack_shapes()
    assert len(shapes) == 224
    rng = np.random.default_rng(synth.seed_for(3, 4242))
    layers = []
    for li, (name, d_out, d_in, axis) in enumerate(shapes):
        L = synth.layer_device(d_out, d_in, synth.F16, "row" if axis == "row" else "col", synth.seed_for(4, li), DEV,
                               zero_frac=0.05, with_wf=True)
        rows = sample_rows(rng, d_out)
        blocks = np.unique(np.concatenate([[0, d_in // 32 - 1], rng.integers(0, d_in // 32, COL_BLOCKS_PER_LAYER - 2)]))
        rows_t = torch.from_numpy(rows).to(DEV)
        rec = {"name": name, "d_out": d_out, "d_in": d_in, "axis": orc.ROW if axis == "row" else orc.COL,
               "W_b": L["W_b"], "W_f": L["W_f"], "rows": rows, "blocks": blocks,
               "Wb_rows": synth.torch_to_bits(L["W_b"][rows_t]), "Wf_rows": synth.torch_to_bits(L["W_f"][rows_t]),
               "Wb_cols": [synth.torch_to_bits(L["W_b"][:, 32 * b:32 * b + 32].contiguous()) for b in blocks],
               "Wf_cols": [synth.torch_to_bits(L["W_f"][:, 32 * b:32 * b + 32].contiguous()) for b in blocks]}
        # column-mode layers: a scale vector drawn on the host, shaped like mean|dW| of the recipe
        if rec["axis"] == orc.COL:
            sig = np.exp(rng.normal(synth.SIGMA_LOG_MEAN, synth.SIGMA_LOG_STD, d_in)) * np.sqrt(2.0 / np.pi)
            rec["v_col_host"] = sig.astype(np.float16).view(np.uint16)
        layers.append(rec)
        del L
    torch.cuda.synchronize()
    yield layers
    layers.clear()
    torch.cuda.empty_cache()


@pytest.fixture(scope="module")
def packed(stack):
    """pdelta_pack_batch over all 224 (W_f, W_b) pairs: one call, as bench.py times it."""
    plan = pd.pdelta_pack_batch_plan([(r["W_f"], r["W_b"]) for r in stack])
    assert len(plan) == 224
    outs = pd.pdelta_pack_batch(plan)
    torch.cuda.synchronize()
    return outs


def test_pack_batch_of_the_whole_stack(stack, packed):
    zero_seen = 0
    for li, (r, (B, v_row, v_col)) in enumerate(zip(stack, packed)):
        what = f"layer {li} {r['name']} {r['d_out']}x{r['d_in']}"
        rows_t = torch.from_numpy(r["rows"]).to(DEV)
        Bo, vo, _ = orc.pack(r["Wf_rows"], r["Wb_rows"], orc.F16, want_col=False)
        assert np.array_equal(words_host(B[rows_t]), Bo), f"{what}: packed words of the sampled rows"
        assert np.array_equal(synth.torch_to_bits(v_row[rows_t]), vo), f"{what}: v_row of the sampled rows"
        zero_seen += int((r["Wf_rows"] == r["Wb_rows"]).sum())
        got_vc = synth.torch_to_bits(v_col)
        for b, wf, wb in zip(r["blocks"], r["Wf_cols"], r["Wb_cols"]):
            Bc, _, vc = orc.pack(wf, wb, orc.F16, want_row=False)
            assert np.array_equal(got_vc[32 * b:32 * b + 32], vc), f"{what}: v_col of columns {32 * b}.."
            assert np.array_equal(words_host(B[:, b]), Bc[:, 0]), f"{what}: sign word column {b}"
    assert zero_seen > 1000                                    # the sign(0) convention is exercised


def test_linear_batch_of_the_whole_stack_one_token(stack, packed):
    Xs = {4096: synth.x_device(1, 4096, synth.F16, synth.seed_for(3, 900), DEV),
          11008: synth.x_device(1, 11008, synth.F16, synth.seed_for(3, 901), DEV)}
    Xh = {k: synth.torch_to_bits(v) for k, v in Xs.items()}
    items = []
    for r, (B, v_row, v_col) in zip(stack, packed):
        v = v_row if r["axis"] == orc.ROW else f16_dev(r["v_col_host"])
        items.append((Xs[r["d_in"]], r["W_b"], B, v, r["axis"]))
    plan = pd.pdelta_linear_batch_plan(items, out_dtype=torch.float16)
    assert len(plan) == 224 and plan.host[223].first_block == sum((r["d_out"] + 15) // 16 for r in stack[:223])
    for Y in plan.Y:
        Y.fill_(float("nan"))
    Ys = pd.pdelta_linear_batch(plan)
    torch.cuda.synchronize()
    for li, (r, Y) in enumerate(zip(stack, Ys)):
        what = f"layer {li} {r['name']} axis={r['axis']}"
        assert torch.isfinite(Y).all(), f"{what}: an output was not written"
        Bo, vo, _ = orc.pack(r["Wf_rows"], r["Wb_rows"], orc.F16, want_col=False)
        v = vo if r["axis"] == orc.ROW else r["v_col_host"]
        n = len(r["rows"])
        ref = orc.linear_at(Xh[r["d_in"]], r["Wb_rows"], Bo, v, r["axis"], np.zeros(n, dtype=np.int64), np.arange(n), orc.F16)
        got = Y[0, torch.from_numpy(r["rows"]).to(DEV)].reshape(1, -1)
        # the tolerance is relative to RMS(Y) of the layer: take it from the sampled outputs
        check_y(got, ref.reshape(1, -1), what)
    # the single-layer entry points give the same bits on a few layers of each shape and axis
    # (4096 x 4096 and 11008 x 4096 layers: there both kernels use 8 waves, hence one summation order)
    for li in (0, 4, 7, 11, 220):
        r, (X, W_b, B, v, axis) = stack[li], items[li]
        fn = pd.pdelta_linear_row if axis == orc.ROW else pd.pdelta_linear_col
        single = fn(X, W_b, B, v)
        torch.cuda.synchronize()
        assert torch.equal(single.view(torch.int16), Ys[li].view(torch.int16)), f"layer {li}"


def test_patch_batch_of_the_whole_stack_in_place(stack, packed):
    # runs last in this module: it overwrites the resident base weights, as the hot-swap does
    items = []
    for r, (B, v_row, v_col) in zip(stack, packed):
        v = v_row if r["axis"] == orc.ROW else f16_dev(r["v_col_host"])
        items.append((r["W_b"], B, v, r["axis"], r["W_b"]))
    plan = pd.pdelta_patch_batch_plan(items)
    assert len(plan) == 224
    pd.pdelta_patch_batch(plan)
    torch.cuda.synchronize()
    for li, r in enumerate(stack):
        Bo, vo, _ = orc.pack(r["Wf_rows"], r["Wb_rows"], orc.F16, want_col=False)
        rows_t = torch.from_numpy(r["rows"]).to(DEV)
        got = synth.torch_to_bits(r["W_b"][rows_t])
        if r["axis"] == orc.ROW:
            want = orc.patch_round(r["Wb_rows"], Bo, vo, orc.ROW, orc.F16)
        else:
            want = orc.patch_round(r["Wb_rows"], Bo, r["v_col_host"], orc.COL, orc.F16)
        assert np.array_equal(got, want), f"layer {li} {r['name']}: merged rows differ from the oracle"
