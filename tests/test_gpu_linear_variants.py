"""GPU parity of pdelta_linear_variants (R requests sharing W_b, each with its own delta) against
the CPU oracle, under the tolerance rule of parity_util.py, and against R single-token calls of
pdelta_linear_row / pdelta_linear_col."""
import numpy as np
import pytest
import torch

from oracle import pdelta_oracle as orc
from paper_2512_19720_amd import binding as pd
from paper_2512_19720_amd import synth
from parity_util import DEV, check_y, f16_dev, gpu_linear, to_dev, words_dev

pytestmark = pytest.mark.gpu


def make_variants(d_out, d_in, R, dtype, axis, seed):
    """Shared base + R independent deltas: host bits, oracle packs, device tensors."""
    base = synth.layer_host(d_out, d_in, max(R, 1), dtype, "row" if axis == orc.ROW else "col", seed)
    Bs, vs = [], []
    for r in range(R):
        Lr = synth.layer_host(d_out, d_in, 1, dtype, "row" if axis == orc.ROW else "col", seed + 1000 + r)
        B, v_row, v_col = orc.pack(Lr["dW"], np.zeros_like(Lr["dW"]), dtype)
        Bs.append(B)
        vs.append(v_row if axis == orc.ROW else v_col)
    X = base["X"][:R]
    dev = {"X": to_dev(X, dtype), "W_b": to_dev(base["W_b"], dtype),
           "variants": [(words_dev(B), f16_dev(v)) for B, v in zip(Bs, vs)]}
    return X, base["W_b"], Bs, vs, dev


@pytest.mark.parametrize("R", [1, 3, 8, 9, 16])
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
@pytest.mark.parametrize("axis", [orc.ROW, orc.COL])
@pytest.mark.parametrize("kernel", [1, 2])
def test_fused_kernel_matches_oracle(R, dtype, axis, kernel, monkeypatch):
    monkeypatch.setenv("PDELTA_TUNE", f"var_kernel={kernel}")          # 1: slab kernel, 2: stride kernel
    for d_out, d_in in ((64, 256), (100, 1152), (7, 128)):
        X, W_b, Bs, vs, d = make_variants(d_out, d_in, R, dtype, axis, synth.seed_for(1, 3000 + 17 * R + d_out))
        ref = orc.linear_variants(X, W_b, Bs, vs, axis, dtype)
        vset = pd.VariantSet(d["variants"], axis)
        for yd in (torch.float32, torch.float16 if dtype == synth.F16 else torch.bfloat16):
            Y = torch.full((R, d_out), float("nan"), dtype=yd, device=DEV)     # every entry must be written
            pd.pdelta_linear_variants(d["X"], d["W_b"], vset, out=Y)
            torch.cuda.synchronize()
            check_y(Y, ref, f"variants R={R} {d_out}x{d_in} dt={dtype} axis={axis} y={yd}")


@pytest.mark.parametrize("axis", [orc.ROW, orc.COL])
def test_decode_layer_4096_sixteen_variants(axis):
    R = 16
    X, W_b, Bs, vs, d = make_variants(4096, 4096, R, synth.F16, axis, synth.seed_for(1, 4000 + axis))
    ref = orc.linear_variants(X, W_b, Bs, vs, axis, synth.F16)
    vset = pd.VariantSet(d["variants"], axis)
    Y = pd.pdelta_linear_variants(d["X"], d["W_b"], vset, out_dtype=torch.float32)
    torch.cuda.synchronize()
    check_y(Y, ref, f"4096x4096 R=16 axis={axis}")
    # against sixteen single-token calls of the ordinary entry points (different summation order:
    # close, not bit-equal)
    for r in (0, 7, 8, 15):
        B_r, v_r = d["variants"][r]
        single = gpu_linear(axis, d["X"][r:r + 1].contiguous(), d["W_b"], B_r, v_r, torch.float32)
        assert torch.allclose(single[0], Y[r], rtol=2e-3, atol=2e-3 * float(Y[r].abs().mean()))


@pytest.mark.parametrize("R,d_in,kernel", [(7, 11008, 0), (16, 11008, 0), (20, 384, 2), (33, 256, 1), (5, 128, 2),
                                           (12, 1152, 2), (16, 2176, 2)])
def test_chunks_of_sixteen_and_both_kernels(R, d_in, kernel, monkeypatch):
    # kernel 0: chosen by size (d_in = 11008: only six whole sign slabs fit in LDS, so 7 and more
    # requests go to the stride kernel); 1: slab kernel; 2: stride kernel forced, also on inputs of
    # 1 to 17 strides with a ragged last one (d_in = 128 ... 2176) and more than 16 requests
    monkeypatch.setenv("PDELTA_TUNE", f"var_kernel={kernel}")
    d_out = 40
    for axis in (orc.ROW, orc.COL):
        X, W_b, Bs, vs, d = make_variants(d_out, d_in, R, synth.F16, axis, synth.seed_for(1, 6000 + R))
        ref = orc.linear_variants(X, W_b, Bs, vs, axis, synth.F16)
        Y = pd.pdelta_linear_variants(d["X"], d["W_b"], pd.VariantSet(d["variants"], axis), out_dtype=torch.float32)
        torch.cuda.synchronize()
        check_y(Y, ref, f"chunked R={R} d_in={d_in} kernel={kernel} axis={axis}")


@pytest.mark.parametrize("R,d_in", [(17, 160), (4, 160), (20, 96)])
def test_request_by_request_fallback(R, d_in):
    # d_in not a multiple of 128: the requests run one after the other
    d_out = 48
    X, W_b, Bs, vs, d = make_variants(d_out, d_in, R, synth.F16, orc.COL, synth.seed_for(1, 5000 + R))
    ref = orc.linear_variants(X, W_b, Bs, vs, orc.COL, synth.F16)
    Y = pd.pdelta_linear_variants(d["X"], d["W_b"], pd.VariantSet(d["variants"], orc.COL), out_dtype=torch.float32)
    torch.cuda.synchronize()
    check_y(Y, ref, f"fallback R={R} d_in={d_in}")


def make_mixed(d_out, d_in, axes, dtype, seed):
    """Shared base + one delta per request, request r in mode axes[r]."""
    R = len(axes)
    base = synth.layer_host(d_out, d_in, R, dtype, "row", seed)
    Bs, vs = [], []
    for r, axis in enumerate(axes):
        Lr = synth.layer_host(d_out, d_in, 1, dtype, "row" if axis == orc.ROW else "col", seed + 2000 + r)
        B, v_row, v_col = orc.pack(Lr["dW"], np.zeros_like(Lr["dW"]), dtype)
        Bs.append(B)
        vs.append(v_row if axis == orc.ROW else v_col)
    dev = {"X": to_dev(base["X"], dtype), "W_b": to_dev(base["W_b"], dtype),
           "variants": [(words_dev(B), f16_dev(v)) for B, v in zip(Bs, vs)]}
    return base["X"], base["W_b"], Bs, vs, dev


@pytest.mark.parametrize("R", [3, 16, 21])
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_one_axis_per_request(R, dtype, monkeypatch):
    rng = np.random.default_rng(40 + R)
    axes = [int(a) for a in rng.integers(0, 2, R)]
    axes[0], axes[1] = orc.ROW, orc.COL                                # both modes are present
    for d_out, d_in, tune in ((100, 1152, ""), (64, 4096, ""), (40, 384, "var_kernel=2"), (100, 1152, "var_kernel=2"),
                              (48, 160, "")):
        monkeypatch.setenv("PDELTA_TUNE", tune)                        # fused (slab / stride kernel) and fallback paths
        X, W_b, Bs, vs, d = make_mixed(d_out, d_in, axes, dtype, synth.seed_for(1, 7000 + R + d_out))
        ref = orc.linear_variants(X, W_b, Bs, vs, axes, dtype)
        vset = pd.VariantSet(d["variants"], axes)
        assert vset.axis == pd.PER_REQUEST
        for yd in (torch.float32, torch.float16 if dtype == synth.F16 else torch.bfloat16):
            Y = torch.full((R, d_out), float("nan"), dtype=yd, device=DEV)
            pd.pdelta_linear_variants(d["X"], d["W_b"], vset, out=Y)
            torch.cuda.synchronize()
            check_y(Y, ref, f"mixed axes R={R} {d_out}x{d_in} dt={dtype} y={yd} tune={tune!r}")


def test_per_request_axes_that_all_agree_use_the_single_mode_kernels():
    for axis in (orc.ROW, orc.COL):
        X, W_b, Bs, vs, d = make_variants(64, 512, 5, synth.F16, axis, 91)
        one = pd.pdelta_linear_variants(d["X"], d["W_b"], pd.VariantSet(d["variants"], axis), out_dtype=torch.float32)
        per = pd.pdelta_linear_variants(d["X"], d["W_b"], pd.VariantSet(d["variants"], [axis] * 5), out_dtype=torch.float32)
        torch.cuda.synchronize()
        assert torch.equal(one, per)


def test_identical_variants_equal_the_ordinary_layer():
    X, W_b, Bs, vs, d = make_variants(128, 512, 6, synth.F16, orc.ROW, 77)
    vset = pd.VariantSet([d["variants"][2]] * 6, orc.ROW)
    Y = pd.pdelta_linear_variants(d["X"], d["W_b"], vset, out_dtype=torch.float32)
    torch.cuda.synchronize()
    check_y(Y, orc.linear(X, W_b, Bs[2], vs[2], orc.ROW), "identical variants")


def test_no_requests_is_a_no_op():
    W = torch.zeros((32, 128), dtype=torch.float16, device=DEV)
    X = torch.zeros((0, 128), dtype=torch.float16, device=DEV)
    Y = pd.pdelta_linear_variants(X, W, pd.VariantSet([], pd.ROW))
    assert Y.shape == (0, 32)
