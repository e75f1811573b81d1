"""GPU parity of the blockwise ("per-group") and scalar scale entry points pdelta_pack_group,
pdelta_linear_group and pdelta_patch_group against the CPU oracle: packed words, scales and merged
weights bit for bit, Y under the tolerance rule of parity_util.py.  Shapes cover every dispatch
branch (staged / plain decode kernels, small-tile and big-tile prefill kernels), ragged d_out,
d_in that is not a multiple of 128, groups inside one 32-input word up to the whole row, rows
that share their scales, and the single scalar."""
import numpy as np
import pytest
import torch

from oracle import pdelta_oracle as orc
from paper_2512_19720_amd import binding as pd
from paper_2512_19720_amd import synth
from parity_util import DEV, check_y, to_dev, words_dev, words_host

pytestmark = pytest.mark.gpu

TORCH16 = {synth.F16: torch.float16, synth.BF16: torch.bfloat16}


def group_case(d_out, d_in, M, dtype, group, shared, seed):
    L = synth.layer_host(d_out, d_in, M, dtype, "row", seed, zero_frac=0.05, with_wf=True)
    B, v = orc.pack_group(L["W_f"], L["W_b"], group, shared_rows=shared, w_dtype=dtype)
    L.update(B=B, v=v)
    return L


def v_dev(v_bits):
    return synth.bits_to_torch(v_bits, synth.F16, DEV)


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
@pytest.mark.parametrize("d_out,d_in,group", [(64, 512, 32), (37, 1024, 64), (100, 1152, 128), (9, 2048, 256),
                                               (130, 4096, 512), (16, 4096, 1024), (33, 2048, 2048),
                                               (70, 1056, 1056), (5, 96, 96), (257, 160, 32), (12, 11008, 11008)])
@pytest.mark.parametrize("shared", [False, True])
def test_pack_group_bit_for_bit(dtype, d_out, d_in, group, shared):
    L = group_case(d_out, d_in, 1, dtype, group, shared, synth.seed_for(4, 500 + d_out + group))
    B, v = pd.pdelta_pack_group(to_dev(L["W_f"], dtype), to_dev(L["W_b"], dtype), group, shared_rows=shared)
    torch.cuda.synchronize()
    assert np.array_equal(words_host(B), L["B"]), "packed words"
    assert v.shape == L["v"].shape
    assert np.array_equal(synth.torch_to_bits(v), L["v"]), "block scales"
    if not shared and group == d_in:                           # the row-mode case: equal to pdelta_pack's v_row
        _, v_row, _ = pd.pdelta_pack(to_dev(L["W_f"], dtype), to_dev(L["W_b"], dtype))
        torch.cuda.synchronize()
        assert torch.equal(v_row, v[:, 0])


def test_pack_group_scalar_of_a_full_size_layer():
    L = synth.layer_device(4096, 11008, synth.F16, "row", synth.seed_for(4, 77), DEV, zero_frac=0.05, with_wf=True)
    B, alpha = pd.pdelta_pack_group(L["W_f"], L["W_b"], 11008, shared_rows=True)
    Bg, vg = pd.pdelta_pack_group(L["W_f"], L["W_b"], 128)
    torch.cuda.synchronize()
    wf, wb = synth.torch_to_bits(L["W_f"]), synth.torch_to_bits(L["W_b"])
    Bo, ao = orc.pack_group(wf, wb, 11008, shared_rows=True)
    assert np.array_equal(words_host(B), Bo) and np.array_equal(synth.torch_to_bits(alpha), ao)
    rows = np.array([0, 1, 2047, 4095])
    Bo, vo = orc.pack_group(wf[rows], wb[rows], 128)
    assert np.array_equal(words_host(Bg)[rows], Bo) and np.array_equal(synth.torch_to_bits(vg)[rows], vo)


LINEAR_CASES = [  # (M, d_out, d_in, group)
    (1, 64, 512, 32), (4, 100, 1152, 128), (16, 37, 4096, 64), (16, 48, 11008, 256),     # staged decode kernel
    (3, 33, 160, 32), (17, 64, 512, 64), (40, 100, 1056, 1056), (64, 16, 256, 256),      # plain decode kernel
    (65, 128, 256, 64), (130, 257, 1024, 128), (300, 384, 512, 512), (200, 100, 96, 32), # prefill kernels
]


@pytest.mark.parametrize("M,d_out,d_in,group", LINEAR_CASES)
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
@pytest.mark.parametrize("shared", [False, True])
def test_linear_group_matches_oracle(M, d_out, d_in, group, dtype, shared):
    L = group_case(d_out, d_in, M, dtype, group, shared, synth.seed_for(1, 8000 + M + d_out + group))
    ref = orc.linear_group(L["X"], L["W_b"], L["B"], L["v"], group, dtype)
    X, W_b, B, v = to_dev(L["X"], dtype), to_dev(L["W_b"], dtype), words_dev(L["B"]), v_dev(L["v"])
    for yd in (torch.float32, TORCH16[dtype]):
        Y = torch.full((M, d_out), float("nan"), dtype=yd, device=DEV)       # every entry must be written
        pd.pdelta_linear_group(X, W_b, B, v, group, out=Y)
        torch.cuda.synchronize()
        check_y(Y, ref, f"group linear M={M} {d_out}x{d_in} g={group} shared={shared} dt={dtype} y={yd}")


@pytest.mark.parametrize("M,d_out,d_in,group", [c for c in LINEAR_CASES if c[0] > 128])
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
@pytest.mark.parametrize("kernel", ["pipelined", "two_per_cu"])
def test_linear_group_big_tile_kernels_forced(M, d_out, d_in, group, dtype, kernel, monkeypatch):
    """The two 256 x 128 tile kernels on shapes that the dispatch would give to the small-tile kernel."""
    monkeypatch.setenv("PDELTA_TUNE", "gemm_small=0,gemm_pipe=" + ("1" if kernel == "pipelined" else "0"))
    L = group_case(d_out, d_in, M, dtype, group, False, synth.seed_for(1, 8300 + M + d_out + group))
    ref = orc.linear_group(L["X"], L["W_b"], L["B"], L["v"], group, dtype)
    X, W_b, B, v = to_dev(L["X"], dtype), to_dev(L["W_b"], dtype), words_dev(L["B"]), v_dev(L["v"])
    for yd in (torch.float32, TORCH16[dtype]):
        Y = torch.full((M, d_out), float("nan"), dtype=yd, device=DEV)
        pd.pdelta_linear_group(X, W_b, B, v, group, out=Y)
        torch.cuda.synchronize()
        check_y(Y, ref, f"group linear ({kernel}) M={M} {d_out}x{d_in} g={group} dt={dtype} y={yd}")


@pytest.mark.parametrize("M", [1, 16, 2048])
def test_linear_group_on_a_benchmark_layer(M):
    """4096 x 4096 with groups of 128 inputs (the usual block size of group-wise formats) and the
    scalar case, at decode and prefill batch sizes: sampled outputs, one fp64 dot product each."""
    dtype = synth.F16 if M <= 16 else synth.BF16
    d_out = d_in = 4096
    L = synth.layer_device(d_out, d_in, dtype, "row", synth.seed_for(1, 8500 + M), DEV)
    X = synth.x_device(M, d_in, dtype, synth.seed_for(1, 8600 + M), DEV)
    rng = np.random.default_rng(M)
    m_idx = rng.integers(0, M, 300)
    o_idx = np.concatenate([rng.integers(0, d_out, 296), [0, 15, 16, d_out - 1]])
    rows = np.unique(o_idx)
    wb_rows, dw_rows = synth.torch_to_bits(L["W_b"][rows]), synth.torch_to_bits(L["dW"][rows])
    Xh = synth.torch_to_bits(X)
    zero = torch.zeros_like(L["dW"])
    for group, shared in ((128, False), (4096, True)):
        B, v = pd.pdelta_pack_group(L["dW"], zero, group, shared_rows=shared)
        torch.cuda.synchronize()
        if shared:                                             # the scalar needs the whole matrix
            Bo_all, vo = orc.pack_group(synth.torch_to_bits(L["dW"]), np.zeros((d_out, d_in), np.uint16), group,
                                        shared_rows=True, w_dtype=dtype)
            Bo = Bo_all[rows]
            assert np.array_equal(synth.torch_to_bits(v), vo)
        else:
            Bo, vo = orc.pack_group(dw_rows, np.zeros_like(dw_rows), group, w_dtype=dtype)
            assert np.array_equal(synth.torch_to_bits(v)[rows], vo)
        assert np.array_equal(words_host(B)[rows], Bo)
        ref = orc.linear_group_at(Xh, wb_rows, Bo, vo, group, m_idx, np.searchsorted(rows, o_idx), dtype)
        Y = pd.pdelta_linear_group(X, L["W_b"], B, v, group, out_dtype=torch.float32)
        torch.cuda.synchronize()
        got = Y[torch.from_numpy(m_idx).to(DEV), torch.from_numpy(o_idx).to(DEV)].reshape(1, -1)
        check_y(got, ref.reshape(1, -1), f"4096x4096 M={M} group={group} shared={shared}")


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
@pytest.mark.parametrize("d_out,d_in,group", [(64, 512, 32), (37, 1024, 128), (9, 2112, 64), (130, 4096, 4096),
                                               (17, 96, 96)])
@pytest.mark.parametrize("shared", [False, True])
def test_patch_group_bit_for_bit(dtype, d_out, d_in, group, shared):
    L = group_case(d_out, d_in, 1, dtype, group, shared, synth.seed_for(0, 600 + d_out + group))
    want = orc.patch_group_round(L["W_b"], L["B"], L["v"], group, dtype)
    W_b, B, v = to_dev(L["W_b"], dtype), words_dev(L["B"]), v_dev(L["v"])
    out = pd.pdelta_patch_group(W_b, B, v, group)
    torch.cuda.synchronize()
    assert np.array_equal(synth.torch_to_bits(out), want)
    assert np.array_equal(synth.torch_to_bits(W_b), L["W_b"])           # input untouched
    pd.pdelta_patch_group(W_b, B, v, group, out=W_b)                       # in place
    torch.cuda.synchronize()
    assert np.array_equal(synth.torch_to_bits(W_b), want)


def test_group_of_the_whole_row_is_row_mode_and_a_constant_is_the_scalar():
    L = group_case(96, 512, 8, synth.F16, 512, False, 31)
    X, W_b, B = to_dev(L["X"], synth.F16), to_dev(L["W_b"], synth.F16), words_dev(L["B"])
    v = v_dev(L["v"])
    Yg = pd.pdelta_linear_group(X, W_b, B, v, 512, out_dtype=torch.float32)
    Yr = pd.pdelta_linear_row(X, W_b, B, v[:, 0].contiguous(), out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert torch.allclose(Yg, Yr, rtol=0, atol=2e-4)
    assert torch.equal(pd.pdelta_patch_group(W_b, B, v, 512), pd.pdelta_patch(W_b, B, v[:, 0].contiguous(), pd.ROW))
    c = torch.full((1, 1), 0.0017, dtype=torch.float16, device=DEV)
    Ys = pd.pdelta_linear_group(X, W_b, B, c, 512, out_dtype=torch.float32)
    Yc = pd.pdelta_linear_group(X, W_b, B, c.expand(96, 16).contiguous(), 32, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert torch.allclose(Ys, Yc, rtol=0, atol=2e-4)
    check_y(Ys, orc.linear(L["X"], L["W_b"], L["B"], np.full(96, np.float16(0.0017)), orc.ROW), "scalar vs row oracle")


def test_empty_batch_is_a_no_op():
    L = group_case(32, 128, 1, synth.F16, 32, False, 3)
    Y = pd.pdelta_linear_group(to_dev(L["X"], synth.F16)[:0].contiguous(), to_dev(L["W_b"], synth.F16),
                               words_dev(L["B"]), v_dev(L["v"]), 32)
    assert Y.shape == (0, 32)
