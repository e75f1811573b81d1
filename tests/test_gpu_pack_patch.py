"""GPU parity of pdelta_pack and pdelta_patch against the CPU oracle: bit for bit."""
import numpy as np
import pytest
import torch

from oracle import pdelta_oracle as orc
from paper_2512_19720_amd import binding as pd
from paper_2512_19720_amd import synth
from parity_util import DEV, f16_dev, to_dev, words_dev, words_host

pytestmark = pytest.mark.gpu


def gpu_pack(Wf_bits, Wb_bits, dtype, want_row=True, want_col=True):
    B, v_row, v_col = pd.pdelta_pack(to_dev(Wf_bits, dtype), to_dev(Wb_bits, dtype), want_row, want_col)
    torch.cuda.synchronize()
    return (words_host(B),
            synth.torch_to_bits(v_row) if v_row is not None else None,
            synth.torch_to_bits(v_col) if v_col is not None else None)


def assert_pack_equal(got, want, what):
    for g, w, name in zip(got, want, ("B_packed", "v_row", "v_col")):
        if w is None:
            assert g is None
            continue
        bad = int((g != w).sum())
        assert bad == 0, f"{what}: {name} differs in {bad} of {w.size} entries"


# shapes: one tile, ragged rows (d_out % 32 != 0), ragged columns (d_in % 1024 != 0, % 512 != 0),
# several tiles each way, minimum size
PACK_SHAPES = [(256, 512), (32, 32), (1, 32), (33, 96), (100, 1056), (70, 2048 + 160), (515, 1024)]


@pytest.mark.parametrize("shape", PACK_SHAPES)
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_pack_matches_oracle(shape, dtype):
    L = synth.layer_host(shape[0], shape[1], 1, dtype, "row", synth.seed_for(4, shape[0] + shape[1]),
                         zero_frac=0.05, with_wf=True)
    want = orc.pack(L["W_f"], L["W_b"], dtype)
    assert_pack_equal(gpu_pack(L["W_f"], L["W_b"], dtype), want, f"pack {shape} dtype {dtype}")


def test_pack_sign_of_zero_signed_zeros_and_subnormals():
    rng = np.random.default_rng(1)
    pool = np.array([0x0000, 0x8000, 0x0001, 0x8001, 0x0002, 0x03FF, 0x83FF, 0x0400, 0x8400,
                     0x3C00, 0xBC00, 0x7BFF, 0xFBFF, 0x2000], np.uint16)
    W_f = pool[rng.integers(0, pool.size, (64, 128))]
    W_b = pool[rng.integers(0, pool.size, (64, 128))]
    W_f[:, :16] = W_b[:, :16]                                     # exact ties -> +1
    want = orc.pack(W_f, W_b, orc.F16)
    assert_pack_equal(gpu_pack(W_f, W_b, synth.F16), want, "special values")
    U = orc.unpack(want[0], 128)
    assert np.all(U[:, :16] == 1.0)


def test_pack_without_scales_or_with_one_of_them():
    L = synth.layer_host(40, 160, 1, synth.F16, "col", 77, with_wf=True)
    want = orc.pack(L["W_f"], L["W_b"])
    got = gpu_pack(L["W_f"], L["W_b"], synth.F16, want_row=False, want_col=False)
    assert np.array_equal(got[0], want[0]) and got[1] is None and got[2] is None
    got = gpu_pack(L["W_f"], L["W_b"], synth.F16, want_row=True, want_col=False)
    assert np.array_equal(got[1], want[1]) and got[2] is None
    got = gpu_pack(L["W_f"], L["W_b"], synth.F16, want_row=False, want_col=True)
    assert np.array_equal(got[2], want[2]) and got[1] is None


def test_pack_is_reproducible_and_ignores_workspace_contents():
    L = synth.layer_host(300, 2048, 1, synth.F16, "row", 5, with_wf=True)
    Wf, Wb = to_dev(L["W_f"], synth.F16), to_dev(L["W_b"], synth.F16)
    ws = torch.full((pd.pdelta_pack_workspace_bytes(300, 2048),), 0xAB, dtype=torch.uint8, device=DEV)
    first = pd.pdelta_pack(Wf, Wb, workspace=ws)
    torch.cuda.synchronize()
    for _ in range(3):
        again = pd.pdelta_pack(Wf, Wb, workspace=ws)          # workspace now holds old sums
        torch.cuda.synchronize()
        for a, b in zip(first, again):
            assert torch.equal(a, b)
    want = orc.pack(L["W_f"], L["W_b"])
    assert np.array_equal(words_host(first[0]), want[0])
    assert np.array_equal(synth.torch_to_bits(first[1]), want[1])


def test_pack_large_magnitudes_stay_exact():
    # |dW| up to ~1e5 and 4096 of them per row: sums near 2^28, still exact in both schemes
    rng = np.random.default_rng(2)
    W_f = np.clip(rng.standard_normal((48, 4096)) * 3e4, -65000, 65000).astype(np.float16)
    W_b = np.clip(rng.standard_normal((48, 4096)) * 3e4, -65000, 65000).astype(np.float16)
    want = orc.pack(W_f, W_b)
    assert_pack_equal(gpu_pack(W_f.view(np.uint16), W_b.view(np.uint16), synth.F16), want, "large")


@pytest.mark.parametrize("shape", [(4096, 11008), (11008, 4096), (4096, 4096)])
def test_pack_full_size_layers_of_the_offline_workload(shape):
    L = synth.layer_device(shape[0], shape[1], synth.F16, "row", synth.seed_for(4, shape[0]), DEV,
                           zero_frac=0.05, with_wf=True)
    B, v_row, v_col = pd.pdelta_pack(L["W_f"], L["W_b"])
    torch.cuda.synchronize()
    want = orc.pack(synth.torch_to_bits(L["W_f"]), synth.torch_to_bits(L["W_b"]))
    assert_pack_equal((words_host(B), synth.torch_to_bits(v_row), synth.torch_to_bits(v_col)), want,
                      f"full {shape}")
    assert (L["W_f"] == L["W_b"]).float().mean().item() > 0.04     # the sign(0) case is exercised


# ---- patch ------------------------------------------------------------------------------------

@pytest.mark.parametrize("shape", [(256, 512), (1, 32), (37, 96), (9, 2048 + 64), (130, 4096)])
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
@pytest.mark.parametrize("axis", [orc.ROW, orc.COL])
def test_patch_matches_oracle_bit_for_bit(shape, dtype, axis):
    L = synth.layer_host(shape[0], shape[1], 1, dtype, "row" if axis == orc.ROW else "col",
                         synth.seed_for(0, 7 * shape[0] + shape[1]))
    B, v_row, v_col = orc.pack(L["dW"], np.zeros_like(L["dW"]), dtype)
    v = v_row if axis == orc.ROW else v_col
    want = orc.patch_round(L["W_b"], B, v, axis, dtype)
    W_b = to_dev(L["W_b"], dtype)
    out = pd.pdelta_patch(W_b, words_dev(B), f16_dev(v), axis)
    torch.cuda.synchronize()
    assert np.array_equal(synth.torch_to_bits(out), want)
    assert np.array_equal(synth.torch_to_bits(W_b), L["W_b"])      # input untouched
    pd.pdelta_patch(W_b, words_dev(B), f16_dev(v), axis, out=W_b)  # in place
    torch.cuda.synchronize()
    assert np.array_equal(synth.torch_to_bits(W_b), want)


def test_patch_rounding_cases_large_scales_and_negative_scales():
    # scales comparable to the weights, negative scales, subnormal weights: the single rounding
    # of the exact sum must still match
    rng = np.random.default_rng(3)
    d_out, d_in = 64, 256
    W_b = (rng.standard_normal((d_out, d_in)) * 10.0 ** rng.uniform(-7, 2, (d_out, d_in))).astype(np.float16)
    v = (rng.standard_normal(d_in) * 10.0 ** rng.uniform(-6, 1, d_in)).astype(np.float16)
    B = rng.integers(0, 2 ** 32, (d_out, d_in // 32), dtype=np.uint32)
    want = orc.patch_round(W_b, B, v, orc.COL)
    out = pd.pdelta_patch(to_dev(W_b.view(np.uint16), synth.F16), words_dev(B), f16_dev(v.view(np.uint16)), pd.COL)
    torch.cuda.synchronize()
    assert np.array_equal(synth.torch_to_bits(out), want)


def test_unpack_through_patch_and_zero_scale():
    rng = np.random.default_rng(4)
    d_out, d_in = 50, 320
    B = rng.integers(0, 2 ** 32, (d_out, d_in // 32), dtype=np.uint32)
    zeros = torch.zeros((d_out, d_in), dtype=torch.float16, device=DEV)
    ones = torch.ones(d_out, dtype=torch.float16, device=DEV)
    out = pd.pdelta_patch(zeros, words_dev(B), ones, pd.ROW)
    torch.cuda.synchronize()
    assert np.array_equal(out.double().cpu().numpy(), orc.unpack(B, d_in))       # exactly +-1
    W = to_dev(synth.layer_host(d_out, d_in, 1, synth.F16, "row", 9)["W_b"], synth.F16)
    out = pd.pdelta_patch(W, words_dev(B), torch.zeros(d_in, dtype=torch.float16, device=DEV), pd.COL)
    torch.cuda.synchronize()
    assert torch.equal(out, W)                                                   # v = 0: untouched


def test_pack_then_patch_restores_an_exactly_representable_fine_tune():
    rng = np.random.default_rng(6)
    d_out, d_in = 96, 512
    W_b = (rng.integers(-32, 32, (d_out, d_in)) / 64.0).astype(np.float16)
    v_r = (rng.integers(1, 8, d_out) / 1024.0).astype(np.float16)
    Bd = np.where(rng.random((d_out, d_in)) < 0.5, -1.0, 1.0)
    W_f = (W_b.astype(np.float64) + v_r.astype(np.float64)[:, None] * Bd).astype(np.float16)
    Wf_d, Wb_d = to_dev(W_f.view(np.uint16), synth.F16), to_dev(W_b.view(np.uint16), synth.F16)
    B, v_row, _ = pd.pdelta_pack(Wf_d, Wb_d)
    out = pd.pdelta_patch(Wb_d, B, v_row, pd.ROW)
    torch.cuda.synchronize()
    assert torch.equal(v_row.cpu(), torch.from_numpy(v_r))
    assert torch.equal(out, Wf_d)
