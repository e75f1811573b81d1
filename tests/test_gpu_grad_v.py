"""GPU parity of pdelta_grad_v (gradient of a loss with respect to the scale vector) against
the CPU oracle.

Tolerance: every product X * (+-1) and every MFMA product is exact; the sums over d_in (or
d_out) and over the tokens are accumulated in fp32.  The result is compared with the fp64
oracle by relative Frobenius error <= 1e-4 and max |err| <= 1e-3 * RMS(grad_oracle): two orders
of magnitude above the fp32 accumulation error of these sizes, far below any wrong index.
"""
import numpy as np
import pytest
import torch

from oracle import pdelta_oracle as orc
from paper_2512_19720_amd import binding as pd
from paper_2512_19720_amd import synth
from parity_util import DEV, to_dev, words_dev

pytestmark = pytest.mark.gpu


def check_grad(got: torch.Tensor, ref: np.ndarray, what: str):
    g = got.double().cpu().numpy()
    assert g.shape == ref.shape and np.isfinite(g).all(), what
    rms = float(np.sqrt(np.mean(ref ** 2)))
    frob = float(np.linalg.norm(g - ref)) / max(float(np.linalg.norm(ref)), 1e-300)
    assert frob <= 1e-4, f"{what}: relative Frobenius error {frob:.3e}"
    assert float(np.abs(g - ref).max()) <= 1e-3 * rms, f"{what}: max error {np.abs(g - ref).max():.3e} rms {rms:.3e}"


def make(M, d_out, d_in, dtype, seed):
    rng = np.random.default_rng(seed)
    conv = (lambda a: a.astype(np.float16).view(np.uint16)) if dtype == synth.F16 else synth.f32_to_bf16_bits
    X = conv(rng.standard_normal((M, d_in)).astype(np.float32))
    dY = conv((rng.standard_normal((M, d_out)) * 0.1).astype(np.float32))
    B = rng.integers(0, 2 ** 32, (d_out, d_in // 32), dtype=np.uint32)
    return X, dY, B


# ragged token counts and outputs around the 256 x 128 x 64 tile, d_in % 64 == 32, one token
SHAPES = [(1, 32, 32), (5, 64, 96), (300, 160, 224), (257, 128, 64), (1000, 96, 1056), (64, 416, 512)]


@pytest.mark.parametrize("M,d_out,d_in", SHAPES)
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
@pytest.mark.parametrize("axis", [orc.ROW, orc.COL])
@pytest.mark.parametrize("kernel", ["pipelined", "two_per_cu"])
def test_grad_v_matches_oracle(M, d_out, d_in, dtype, axis, kernel, monkeypatch):
    monkeypatch.setenv("PDELTA_TUNE", "grad_pipe=1" if kernel == "pipelined" else "grad_pipe=0")
    X, dY, B = make(M, d_out, d_in, dtype, synth.seed_for(2, 7000 + M + d_out))
    ref = orc.grad_v(X, dY, B, axis, dtype)
    ws = torch.full((pd.pdelta_grad_v_workspace_bytes(M, d_out, d_in, axis),), 0xCD, dtype=torch.uint8, device=DEV)
    out = torch.full((d_out if axis == orc.ROW else d_in,), float("nan"), dtype=torch.float32, device=DEV)
    pd.pdelta_grad_v(to_dev(X, dtype), to_dev(dY, dtype), words_dev(B), axis, out=out, workspace=ws)
    torch.cuda.synchronize()
    check_grad(out, ref, f"grad_v M={M} {d_out}x{d_in} dt={dtype} axis={axis}")
    again = pd.pdelta_grad_v(to_dev(X, dtype), to_dev(dY, dtype), words_dev(B), axis, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(again, out)                                    # fixed summation order


@pytest.mark.parametrize("axis", [orc.ROW, orc.COL])
@pytest.mark.parametrize("kernel", ["default", "two_per_cu"])
def test_grad_v_training_shape_sampled(axis, kernel, monkeypatch):
    """M = 2048 tokens on a 4096 x 4096 layer (the benchmark's shape): the oracle evaluates a
    sample of the entries, each from the rows / columns it needs."""
    if kernel == "two_per_cu":
        monkeypatch.setenv("PDELTA_TUNE", "grad_pipe=0")
    M, d_out, d_in = 2048, 4096, 4096
    X, dY, B = make(M, d_out, d_in, synth.BF16, synth.seed_for(2, 7900 + axis))
    got = pd.pdelta_grad_v(to_dev(X, synth.BF16), to_dev(dY, synth.BF16), words_dev(B), axis)
    torch.cuda.synchronize()
    idx = np.unique(np.concatenate([[0, 1, 127, 128, 4095], np.random.default_rng(5).integers(0, 4096, 40)]))
    if axis == orc.ROW:       # entry o needs row o of B and column o of dY
        ref = orc.grad_v(X, np.ascontiguousarray(dY[:, idx]), np.ascontiguousarray(B[idx]), orc.ROW, synth.BF16)
    else:                     # entry i needs bit i of every row: take whole 32-column words
        words = np.unique(idx // 32)
        cols = (words[:, None] * 32 + np.arange(32)[None, :]).reshape(-1)
        full = orc.grad_v(np.ascontiguousarray(X[:, cols]), dY, np.ascontiguousarray(B[:, words]), orc.COL, synth.BF16)
        ref = full[np.searchsorted(cols, idx)]
    check_grad(got[torch.from_numpy(idx).to(DEV)], ref, f"sampled training shape axis={axis}")


def test_grad_v_of_no_tokens_is_zero():
    B = words_dev(np.zeros((64, 4), dtype=np.uint32))
    X = torch.zeros((0, 128), dtype=torch.float16, device=DEV)
    dY = torch.zeros((0, 64), dtype=torch.float16, device=DEV)
    for axis, n in ((pd.ROW, 64), (pd.COL, 128)):
        out = torch.full((n,), 3.0, dtype=torch.float32, device=DEV)
        pd.pdelta_grad_v(X, dY, B, axis, out=out)
        torch.cuda.synchronize()
        assert torch.count_nonzero(out) == 0
