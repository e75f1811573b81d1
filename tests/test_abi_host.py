"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function
the header declares, and turns every invalid argument into its error code before any HIP call."""
import ctypes
import os
import re

import pytest

from paper_2512_19720_amd import binding as pd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
A = 0x10000          # a fake, 16-byte aligned, non-null device address (never dereferenced)


def declared_functions():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if header.endswith(".h"):
            text = open(os.path.join(ROOT, "include", header)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(pdelta_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_function():
    names = declared_functions()
    assert {"pdelta_pack", "pdelta_linear_row", "pdelta_linear_col", "pdelta_patch",
            "pdelta_pack_workspace_bytes", "pdelta_status_string", "pdelta_linear_batch_plan",
            "pdelta_linear_batch", "pdelta_patch_batch", "pdelta_pack_batch_plan",
            "pdelta_pack_batch", "pdelta_linear_variants", "pdelta_grad_v",
            "pdelta_grad_v_workspace_bytes"} <= set(names)
    L = pd.lib()
    for n in names:
        assert hasattr(L, n), n


def test_probe_argument_errors():
    L = pd.lib()
    assert L.pdelta_probe_read_stream(None, 1024, A, None) == pd.EINVAL
    assert L.pdelta_probe_read_stream(A, 0, A + 4096, None) == pd.EINVAL
    assert L.pdelta_probe_read_stream(A, 1000, A + 4096, None) == pd.ESHAPE
    assert L.pdelta_probe_read_stream(A + 8, 1024, A + 4096, None) == pd.EALIGN
    assert L.pdelta_probe_mfma(3, 0, 10, A, None) == pd.EINVAL
    assert L.pdelta_probe_mfma(2, 2, 10, A, None) == pd.EINVAL
    assert L.pdelta_probe_mfma(2, 1, 0, A, None) == pd.EINVAL
    assert L.pdelta_probe_mfma(2, 1, 10, None, None) == pd.EINVAL
    # prefill parts: mask range, pdelta_linear_row's checks, more than 128 tokens (nothing is launched)
    W, B, V, Y = A + (1 << 20), A + (2 << 20), A + (3 << 20), A + (4 << 20)
    assert L.pdelta_probe_prefill_parts(16, A, W, B, V, Y, 256, 128, 64, pd.BF16, None) == pd.EINVAL
    assert L.pdelta_probe_prefill_parts(-1, A, W, B, V, Y, 256, 128, 64, pd.BF16, None) == pd.EINVAL
    assert L.pdelta_probe_prefill_parts(15, None, W, B, V, Y, 256, 128, 64, pd.BF16, None) == pd.EINVAL
    assert L.pdelta_probe_prefill_parts(15, A, W, B, V, Y, 256, 128, 48, pd.BF16, None) == pd.ESHAPE
    assert L.pdelta_probe_prefill_parts(15, A, W, B, V, Y, 128, 128, 64, pd.BF16, None) == pd.ESHAPE
    assert L.pdelta_probe_prefill_parts(15, A + 2, W, B, V, Y, 256, 128, 64, pd.BF16, None) == pd.EALIGN
    assert L.pdelta_probe_prefill_parts(15, A, W, B, V, Y, 256, 128, 64, 7, None) == pd.EDTYPE


def test_status_strings():
    L = pd.lib()
    for code in range(0, -7, -1):
        s = L.pdelta_status_string(code).decode()
        assert s.startswith("PDELTA_")
    assert "unknown" in L.pdelta_status_string(5).decode()


def test_workspace_bytes():
    assert pd.pdelta_pack_workspace_bytes(4096, 11008) == 8 * (11 * 4096 + 64 * 11008)
    assert pd.pdelta_pack_workspace_bytes(65, 32) == 8 * (1 * 65 + 2 * 32)
    assert pd.pdelta_pack_workspace_bytes(0, 32) == 0
    assert pd.pdelta_pack_workspace_bytes(32, -1) == 0


def call_linear(fn="pdelta_linear_row", X=A, W=A + 0x1000000, B=A + 0x2000000, v=A + 0x3000000,
                Y=A + 0x4000000, M=4, d_out=64, d_in=128, xdt=pd.F16, ydt=pd.F16):
    return getattr(pd.lib(), fn)(X, W, B, v, Y, M, d_out, d_in, xdt, ydt, None)


@pytest.mark.parametrize("fn", ["pdelta_linear_row", "pdelta_linear_col"])
def test_linear_argument_errors(fn):
    for null in ("X", "W", "B", "v", "Y"):
        assert call_linear(fn, **{null: None}) == pd.EINVAL
    assert call_linear(fn, M=-1) == pd.EINVAL
    assert call_linear(fn, d_out=0) == pd.EINVAL
    assert call_linear(fn, d_in=0) == pd.EINVAL
    assert call_linear(fn, d_in=100) == pd.ESHAPE
    assert call_linear(fn, d_in=48) == pd.ESHAPE
    assert call_linear(fn, d_out=(1 << 22) + 1) == pd.ESHAPE
    assert call_linear(fn, xdt=pd.F32) == pd.EDTYPE
    assert call_linear(fn, xdt=7) == pd.EDTYPE
    assert call_linear(fn, ydt=3) == pd.EDTYPE
    for name in ("X", "W", "B", "v", "Y"):
        assert call_linear(fn, **{name: A + 0x5000000 + 8}) == pd.EALIGN
    # Y overlapping an input
    assert call_linear(fn, Y=A + 0x1000000) == pd.EINVAL
    assert call_linear(fn, Y=A + 16) == pd.EINVAL                      # inside X
    # an empty batch is a no-op, decided on the host
    assert call_linear(fn, M=0) == pd.OK
    assert call_linear(fn, M=0, X=None, Y=None) == pd.OK
    assert call_linear(fn, M=0, d_in=33) == pd.ESHAPE                  # still validated


def fake_layers(n=3, **edit):
    arr = (pd.Layer * n)()
    for k in range(n):
        base = A + k * 0x10000000
        arr[k] = pd.Layer(base, base + 0x1000000, base + 0x2000000, base + 0x3000000, base + 0x4000000,
                          64 + 16 * k + 1, 128 * (k + 1), k % 2, -1)
    for name, value in edit.items():
        setattr(arr[1], name, value)
    return arr


def test_batch_plan_and_argument_errors():
    L = pd.lib()
    arr = fake_layers()
    assert L.pdelta_linear_batch_plan(arr, 3) == pd.OK
    # first_block = running sum of ceil(d_out / 16): 65 -> 5 blocks, 81 -> 6 blocks
    assert [arr[k].first_block for k in range(3)] == [0, 5, 11]
    assert L.pdelta_linear_batch_plan(None, 0) == pd.OK
    assert L.pdelta_linear_batch_plan(None, 2) == pd.EINVAL
    assert L.pdelta_linear_batch_plan(arr, -1) == pd.EINVAL
    assert L.pdelta_linear_batch_plan(fake_layers(axis=2), 3) == pd.EINVAL
    assert L.pdelta_linear_batch_plan(fake_layers(d_in=100), 3) == pd.ESHAPE
    assert L.pdelta_linear_batch_plan(fake_layers(d_out=0), 3) == pd.EINVAL

    dev = A + 0x70000000

    def run(a, n=3, M=2, xdt=pd.F16, ydt=pd.F16, d=dev):
        return L.pdelta_linear_batch(a, d, n, M, xdt, ydt, None)

    assert run(arr, M=0) == pd.OK                                      # empty batch: host-side no-op
    assert run(arr, n=0) == pd.OK
    assert run(None, n=0, d=None) == pd.OK
    assert run(arr, n=-1) == pd.EINVAL
    assert run(arr, M=-1) == pd.EINVAL
    assert run(None) == pd.EINVAL
    assert run(arr, d=None) == pd.EINVAL
    assert run(arr, d=dev + 8) == pd.EALIGN
    assert run(arr, xdt=pd.F32) == pd.EDTYPE
    assert run(arr, ydt=9) == pd.EDTYPE
    assert run(fake_layers(), M=0) == pd.EINVAL                        # never planned
    for name in ("X", "W_b", "B_packed", "v", "Y"):
        bad = fake_layers(**{name: None})
        assert L.pdelta_linear_batch_plan(bad, 3) == pd.OK             # the plan looks at shapes only
        assert run(bad) == pd.EINVAL
        bad = fake_layers(**{name: A + 0x60000008})
        L.pdelta_linear_batch_plan(bad, 3)
        assert run(bad) == pd.EALIGN
    edited = fake_layers()
    L.pdelta_linear_batch_plan(edited, 3)
    edited[1].d_out = 300                                              # shape edited after planning
    assert run(edited, M=0) == pd.EINVAL
    alias = fake_layers()
    alias[1].Y = alias[1].W_b
    L.pdelta_linear_batch_plan(alias, 3)
    assert run(alias) == pd.EINVAL


def test_patch_batch_argument_errors():
    L = pd.lib()
    dev = A + 0x70000000

    def run(a, n=3, dt=pd.F16, d=dev):
        return L.pdelta_patch_batch(a, d, n, dt, None)

    arr = fake_layers()
    assert run(arr) == pd.EINVAL                                       # never planned
    L.pdelta_linear_batch_plan(arr, 3)
    assert run(arr, n=0) == pd.OK
    assert run(arr, n=-1) == pd.EINVAL
    assert run(None) == pd.EINVAL
    assert run(arr, d=None) == pd.EINVAL
    assert run(arr, d=dev + 4) == pd.EALIGN
    assert run(arr, dt=pd.F32) == pd.EDTYPE
    for name in ("W_b", "B_packed", "v", "Y"):
        bad = fake_layers(**{name: None})
        L.pdelta_linear_batch_plan(bad, 3)
        assert run(bad) == pd.EINVAL
        bad = fake_layers(**{name: A + 0x60000008})
        L.pdelta_linear_batch_plan(bad, 3)
        assert run(bad) == pd.EALIGN
    ok = fake_layers(X=None)                                           # X is not used by the merge
    L.pdelta_linear_batch_plan(ok, 3)
    inplace = fake_layers()
    inplace[1].Y = inplace[1].W_b                                      # in place is allowed
    L.pdelta_linear_batch_plan(inplace, 3)
    overlap = fake_layers()
    overlap[1].Y = overlap[1].W_b + 64                                 # partial overlap is not
    L.pdelta_linear_batch_plan(overlap, 3)
    assert run(overlap) == pd.EINVAL
    # valid descriptors would launch: not exercised without a GPU
    del ok, inplace


def fake_jobs(n=3, **edit):
    arr = (pd.PackJob * n)()
    for k in range(n):
        base = A + k * 0x10000000
        d_out, d_in = 100 + 500 * k, 1024 * (k + 1) + 32
        arr[k] = pd.PackJob(base, base + 0x1000000, base + 0x2000000, base + 0x3000000, base + 0x3100000,
                            base + 0x4000000, pd.pdelta_pack_workspace_bytes(d_out, d_in), d_out, d_in, -1, -1, -1, 0)
    for name, value in edit.items():
        setattr(arr[1], name, value)
    return arr


def test_pack_batch_plan_and_argument_errors():
    L = pd.lib()
    arr = fake_jobs()
    assert L.pdelta_pack_batch_plan(arr, 3) == pd.OK
    # job 0: 100 x 1056 -> 64-row tiles (2 blocks): 2 row tiles x 2 column tiles; 2 + 17 finalize blocks
    # job 1: 600 x 2080 -> 128-row tiles (4 blocks): 5 x 3 tiles; 10 + 33 finalize blocks
    assert [arr[k].tile_blocks for k in range(3)] == [2, 4, 4]
    assert [arr[k].first_tile for k in range(3)] == [0, 4, 19]
    assert [arr[k].first_fin_block for k in range(3)] == [0, 19, 62]
    assert L.pdelta_pack_batch_plan(None, 0) == pd.OK
    assert L.pdelta_pack_batch_plan(None, 1) == pd.EINVAL
    assert L.pdelta_pack_batch_plan(fake_jobs(d_in=100), 3) == pd.ESHAPE
    assert L.pdelta_pack_batch_plan(fake_jobs(d_out=-4), 3) == pd.EINVAL
    dev = A + 0x70000000

    def run(a, n=3, dt=pd.F16, d=dev):
        return L.pdelta_pack_batch(a, d, n, dt, None)

    assert run(arr, n=0) == pd.OK
    assert run(arr, n=-2) == pd.EINVAL
    assert run(None) == pd.EINVAL
    assert run(arr, d=None) == pd.EINVAL
    assert run(arr, d=dev + 8) == pd.EALIGN
    assert run(arr, dt=pd.F32) == pd.EDTYPE
    assert run(fake_jobs()) == pd.EINVAL                               # never planned
    for name in ("W_f", "W_b", "B_packed"):
        bad = fake_jobs(**{name: None})
        L.pdelta_pack_batch_plan(bad, 3)
        assert run(bad) == pd.EINVAL
    bad = fake_jobs(workspace=None)
    L.pdelta_pack_batch_plan(bad, 3)
    assert run(bad) == pd.EWORKSPACE
    bad = fake_jobs(workspace_bytes=64)
    L.pdelta_pack_batch_plan(bad, 3)
    assert run(bad) == pd.EWORKSPACE
    bad = fake_jobs(v_col=A + 0x60000002)
    L.pdelta_pack_batch_plan(bad, 3)
    assert run(bad) == pd.EALIGN
    edited = fake_jobs()
    L.pdelta_pack_batch_plan(edited, 3)
    edited[0].d_out = 4096                                             # shape edited after planning
    edited[0].workspace_bytes = 1 << 30
    assert run(edited) == pd.EINVAL


def test_linear_variants_argument_errors():
    L = pd.lib()

    def variants(n=3, **edit):
        arr = (pd.Variant * n)()
        for r in range(n):
            arr[r] = pd.Variant(A + 0x2000000 + r * 0x100000, A + 0x3000000 + r * 0x10000)
        for name, value in edit.items():
            setattr(arr[1], name, value)
        return arr

    def run(arr, X=A, W=A + 0x1000000, dev=A + 0x5000000, R=3, axis=pd.ROW, Y=A + 0x4000000, d_out=64,
            d_in=128, xdt=pd.F16, ydt=pd.F16):
        return L.pdelta_linear_variants(X, W, arr, dev, R, axis, Y, d_out, d_in, xdt, ydt, None)

    ok = variants()
    assert run(ok, R=0) == pd.OK
    assert run(None, R=0, dev=None, X=None, Y=None) == pd.OK
    assert run(ok, R=0, d_in=100) == pd.ESHAPE                        # still validated
    assert run(ok, R=-1) == pd.EINVAL
    assert run(None) == pd.EINVAL
    assert run(ok, dev=None) == pd.EINVAL
    assert run(ok, dev=A + 0x5000008) == pd.EALIGN
    assert run(ok, axis=5) == pd.EINVAL
    assert run(ok, X=None) == pd.EINVAL
    assert run(ok, Y=None) == pd.EINVAL
    assert run(ok, d_in=48) == pd.ESHAPE
    assert run(ok, xdt=pd.F32) == pd.EDTYPE
    assert run(variants(B_packed=None)) == pd.EINVAL
    assert run(variants(v=None)) == pd.EINVAL
    assert run(variants(v=A + 0x3000002)) == pd.EALIGN
    assert run(variants(B_packed=A + 0x4000000)) == pd.EINVAL         # Y overlaps a variant's signs
    # one axis per request: every record must name ROW or COL; R = 0 stays a no-op
    assert run(ok, R=0, axis=pd.PER_REQUEST) == pd.OK
    assert run(variants(axis=2), axis=pd.PER_REQUEST) == pd.EINVAL
    assert run(variants(axis=-1), axis=pd.PER_REQUEST) == pd.EINVAL
    assert run(variants(axis=7), axis=pd.ROW, R=0) == pd.OK            # ignored when the call names the axis
    # a column-mode record's v has d_in entries: Y placed inside that (longer) range is an overlap
    assert run(variants(axis=pd.COL), axis=pd.PER_REQUEST, Y=A + 0x3010000 + 128, d_out=64, d_in=128) == pd.EINVAL


def test_group_scale_entry_points_argument_errors():
    L = pd.lib()
    W, Bp, v, X, Y, ws = A, A + (1 << 32), A + (2 << 32), A + (3 << 32), A + (4 << 32), A + (5 << 32)

    def lin(X=X, W=W, B=Bp, v=v, group=32, shared=0, Y=Y, M=4, d_out=64, d_in=128, xdt=pd.F16, ydt=pd.F16):
        return L.pdelta_linear_group(X, W, B, v, group, shared, Y, M, d_out, d_in, xdt, ydt, None)

    for null in ("X", "W", "B", "v", "Y"):
        assert lin(**{null: None}) == pd.EINVAL
    assert lin(M=-1) == pd.EINVAL and lin(group=0) == pd.EINVAL and lin(shared=2) == pd.EINVAL
    for bad_group in (16, 48, 96, 256):                                # too small, not a power of two, does not divide
        assert lin(group=bad_group) == pd.ESHAPE
    assert lin(d_in=100, group=100) == pd.ESHAPE                        # d_in itself must be a multiple of 32
    assert lin(xdt=pd.F32) == pd.EDTYPE and lin(ydt=9) == pd.EDTYPE
    assert lin(v=v + 2) == pd.EALIGN
    assert lin(M=0) == pd.OK and lin(M=0, X=None, Y=None) == pd.OK
    assert lin(M=0, d_in=96, group=96) == pd.OK                         # the whole row is always a valid group
    assert lin(Y=v) == pd.EINVAL                                        # Y on top of the scales
    # v has d_out * d_in / group = 256 entries here (512 bytes): a Y that starts inside them overlaps
    assert lin(Y=v + 64, M=0) == pd.OK                                  # an empty batch writes nothing
    assert lin(Y=v + 496) == pd.EINVAL

    def patch(W=W, B=Bp, v=v, group=64, shared=0, out=Y, d_out=64, d_in=128, dt=pd.F16):
        return L.pdelta_patch_group(W, B, v, group, shared, out, d_out, d_in, dt, None)

    for null in ("W", "B", "v", "out"):
        assert patch(**{null: None}) == pd.EINVAL
    assert patch(group=24) == pd.ESHAPE and patch(shared=-1) == pd.EINVAL and patch(dt=pd.F32) == pd.EDTYPE
    assert patch(out=W + 64) == pd.EINVAL and patch(out=Bp) == pd.EINVAL and patch(out=Y + 4) == pd.EALIGN

    def pack(Wf=X, Wb=W, d_out=64, d_in=128, dt=pd.F16, group=32, shared=0, B=Bp, v=v, ws=ws, wsb=1 << 20):
        return L.pdelta_pack_group(Wf, Wb, d_out, d_in, dt, group, shared, B, v, ws, wsb, None)

    for null in ("Wf", "Wb", "B", "v"):
        assert pack(**{null: None}) == pd.EINVAL
    assert pack(group=12) == pd.ESHAPE and pack(dt=5) == pd.EDTYPE and pack(B=Bp + 8) == pd.EALIGN
    assert L.pdelta_pack_group_workspace_bytes(64, 128, 32, 0) == 0
    assert L.pdelta_pack_group_workspace_bytes(64, 128, 32, 1) == 8 * 64 * 4
    assert L.pdelta_pack_group_workspace_bytes(64, 128, 128, 1) == 8 * 64
    assert L.pdelta_pack_group_workspace_bytes(64, 128, 48, 1) == 0       # invalid group
    assert pack(shared=1, ws=None) == pd.EWORKSPACE and pack(shared=1, wsb=8 * 64 * 4 - 1) == pd.EWORKSPACE
    assert pack(shared=1, ws=ws + 8) == pd.EALIGN
    assert pack(v=X + 64) == pd.EINVAL and pack(B=W) == pd.EINVAL and pack(shared=1, ws=Bp) == pd.EINVAL


def test_grad_v_workspace_and_argument_errors():
    L = pd.lib()
    # row: one fp32 partial per (256-token tile, output); col: the same per input, rounded up
    # to 256 bytes, plus the transposed sign bits
    assert pd.pdelta_grad_v_workspace_bytes(2048, 4096, 11008, pd.ROW) == 8 * 4096 * 4
    assert pd.pdelta_grad_v_workspace_bytes(300, 64, 96, pd.COL) == 2 * 96 * 4 + 96 * 64 // 8
    assert pd.pdelta_grad_v_workspace_bytes(0, 64, 96, pd.ROW) == 64 * 4
    assert pd.pdelta_grad_v_workspace_bytes(5, 0, 96, pd.ROW) == 0
    assert pd.pdelta_grad_v_workspace_bytes(5, 64, 96, 3) == 0

    def run(X=A, dY=A + 0x1000000, B=A + 0x2000000, axis=pd.ROW, g=A + 0x3000000, M=4, d_out=64, d_in=128,
            dt=pd.F16, ws=A + 0x4000000, wsb=1 << 20):
        return L.pdelta_grad_v(X, dY, B, axis, g, M, d_out, d_in, dt, ws, wsb, None)

    for null in ("X", "dY", "B", "g"):
        assert run(**{null: None}) == pd.EINVAL
    assert run(axis=2) == pd.EINVAL
    assert run(M=-1) == pd.EINVAL
    assert run(d_in=100) == pd.ESHAPE
    assert run(axis=pd.COL, d_out=48) == pd.ESHAPE                    # column mode transposes 32-bit words
    assert run(dt=pd.F32) == pd.EDTYPE
    assert run(ws=None) == pd.EWORKSPACE
    assert run(wsb=64 * 4 - 1) == pd.EWORKSPACE
    for name in ("X", "dY", "B", "g", "ws"):
        assert run(**{name: A + 0x5000008}) == pd.EALIGN
    assert run(g=A + 16) == pd.EINVAL                                 # inside X
    assert run(g=A + 0x4000000) == pd.EINVAL                          # inside the workspace


def call_pack(Wf=A, Wb=A + 0x1000000, d_out=64, d_in=128, dt=pd.F16, B=A + 0x2000000,
              vr=A + 0x3000000, vc=A + 0x3100000, ws=A + 0x4000000, wsb=1 << 20):
    return pd.lib().pdelta_pack(Wf, Wb, d_out, d_in, dt, B, vr, vc, ws, wsb, None)


def test_pack_argument_errors():
    for null in ("Wf", "Wb", "B"):
        assert call_pack(**{null: None}) == pd.EINVAL
    assert call_pack(d_out=-3) == pd.EINVAL
    assert call_pack(d_in=65) == pd.ESHAPE
    assert call_pack(d_in=(1 << 22) + 32) == pd.ESHAPE
    assert call_pack(dt=pd.F32) == pd.EDTYPE
    assert call_pack(ws=None) == pd.EWORKSPACE
    assert call_pack(wsb=8 * (64 + 128) - 1) == pd.EWORKSPACE
    assert call_pack(ws=A + 0x4000000 + 4) == pd.EALIGN
    assert call_pack(Wf=A + 2) == pd.EALIGN
    assert call_pack(vr=A + 0x3000000 + 2) == pd.EALIGN
    assert call_pack(B=A + 32) == pd.EINVAL                             # B_packed inside W_f
    # every output and the scratch must be disjoint from the inputs and from each other
    assert call_pack(vr=A + 64) == pd.EINVAL                            # v_row inside W_f
    assert call_pack(vc=A + 0x1000000 + 64) == pd.EINVAL                # v_col inside W_b
    assert call_pack(ws=A) == pd.EINVAL                                 # workspace on top of W_f
    assert call_pack(ws=A + 0x1000000, wsb=1 << 12) == pd.EINVAL        # workspace on top of W_b
    assert call_pack(vr=A + 0x2000000) == pd.EINVAL                     # v_row on top of B_packed
    assert call_pack(vc=A + 0x3000000 + 64) == pd.EINVAL                # v_col inside v_row
    assert call_pack(ws=A + 0x3100000 - 4096) == pd.EINVAL              # workspace reaches into v_col
    assert call_pack(ws=A + 0x2000000) == pd.EINVAL                     # workspace on top of B_packed


def call_patch(W=A, B=A + 0x1000000, v=A + 0x2000000, axis=pd.ROW, out=A + 0x3000000, d_out=64,
               d_in=128, dt=pd.F16):
    return pd.lib().pdelta_patch(W, B, v, axis, out, d_out, d_in, dt, None)


def test_patch_argument_errors():
    for null in ("W", "B", "v", "out"):
        assert call_patch(**{null: None}) == pd.EINVAL
    assert call_patch(axis=2) == pd.EINVAL
    assert call_patch(axis=-1) == pd.EINVAL
    assert call_patch(d_in=16) == pd.ESHAPE
    assert call_patch(dt=pd.F32) == pd.EDTYPE
    assert call_patch(out=A + 0x3000000 + 6) == pd.EALIGN
    assert call_patch(out=A + 64) == pd.EINVAL                          # partial overlap with W_b
    assert call_patch(out=A + 0x1000000) == pd.EINVAL                   # W_out on top of B_packed


def test_binding_refuses_cpu_tensors():
    import torch
    W = torch.zeros((32, 32), dtype=torch.float16)
    with pytest.raises(ValueError):
        pd.pdelta_patch(W, torch.zeros((32, 1), dtype=torch.int32), torch.zeros(32, dtype=torch.float16), pd.ROW)


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(pd, "_lib", None)
    monkeypatch.setattr(pd, "_LIB_PATH", "/nonexistent/libpdelta.so")
    with pytest.raises(RuntimeError, match="no CPU or PyTorch fallback"):
        pd.lib()


def test_header_is_plain_c_and_struct_layouts_match_the_binding(tmp_path):
    """include/pdelta.h must compile as C (it is the boundary), and the ctypes mirrors of its
    structs must agree with the C compiler on size and field offsets."""
    import subprocess
    src = tmp_path / "layout.c"
    src.write_text(r'''
#include <stdio.h>
#include <stddef.h>
#include "pdelta.h"
int main(void) {
    printf("pdelta_layer %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu\n", sizeof(pdelta_layer),
           offsetof(pdelta_layer, X), offsetof(pdelta_layer, W_b), offsetof(pdelta_layer, B_packed),
           offsetof(pdelta_layer, v), offsetof(pdelta_layer, Y), offsetof(pdelta_layer, d_out),
           offsetof(pdelta_layer, d_in), offsetof(pdelta_layer, axis), offsetof(pdelta_layer, first_block));
    printf("pdelta_variant %zu %zu %zu %zu %zu\n", sizeof(pdelta_variant), offsetof(pdelta_variant, B_packed),
           offsetof(pdelta_variant, v), offsetof(pdelta_variant, axis), offsetof(pdelta_variant, reserved));
    printf("pdelta_pack_job %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu\n", sizeof(pdelta_pack_job),
           offsetof(pdelta_pack_job, W_f), offsetof(pdelta_pack_job, W_b), offsetof(pdelta_pack_job, B_packed),
           offsetof(pdelta_pack_job, v_row), offsetof(pdelta_pack_job, v_col), offsetof(pdelta_pack_job, workspace),
           offsetof(pdelta_pack_job, workspace_bytes), offsetof(pdelta_pack_job, d_out), offsetof(pdelta_pack_job, d_in),
           offsetof(pdelta_pack_job, first_tile), offsetof(pdelta_pack_job, first_fin_block),
           offsetof(pdelta_pack_job, tile_blocks));
    printf("enums %d %d %d %d %d %d %d\n", PDELTA_F16, PDELTA_BF16, PDELTA_F32, PDELTA_ROW, PDELTA_COL, PDELTA_EHIP,
           PDELTA_PER_REQUEST);
    return 0;
}
''')
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe)], check=True)
    lines = dict(l.split(" ", 1) for l in subprocess.run([str(exe)], check=True, capture_output=True,
                                                       text=True).stdout.strip().splitlines())

    def layout(struct, fields):
        return [ctypes.sizeof(struct)] + [getattr(struct, f).offset for f in fields]

    assert list(map(int, lines["pdelta_layer"].split())) == layout(
        pd.Layer, ["X", "W_b", "B_packed", "v", "Y", "d_out", "d_in", "axis", "first_block"])
    assert list(map(int, lines["pdelta_variant"].split())) == layout(pd.Variant, ["B_packed", "v", "axis", "reserved"])
    assert list(map(int, lines["pdelta_pack_job"].split())) == layout(
        pd.PackJob, ["W_f", "W_b", "B_packed", "v_row", "v_col", "workspace", "workspace_bytes", "d_out", "d_in",
                     "first_tile", "first_fin_block", "tile_blocks"])
    assert list(map(int, lines["enums"].split())) == [pd.F16, pd.BF16, pd.F32, pd.ROW, pd.COL, pd.EHIP, pd.PER_REQUEST]
