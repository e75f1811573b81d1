"""Helpers of the GPU parity tests: move seeded inputs to the device, run the oracle on the
same bits, and apply the comparison rules.

Tolerance for Y (stated once, used everywhere):
  * relative Frobenius error  ||Y_gpu - Y_ref||_F / ||Y_ref||_F <= 1e-3
  * max |Y_gpu - Y_ref| <= 1e-2 * RMS(Y_oracle)
  where Y_ref is the fp64 oracle itself, unrounded.  fp32 and fp16 outputs must meet exactly
  these.  A bf16 output cannot (rounding to 8 significant bits alone costs ~1.6e-3 relative,
  and half an ulp at |y| in [4, 8) is already above 1e-2 * RMS for the benchmark's layers), so
  for bf16 outputs each bound is widened by what the final rounding may add at most, half a
  bf16 ulp per entry: per entry 1e-2 * RMS + ulp/2, and 1e-3 + ||ulp/2||_F / ||Y_ref||_F for
  the Frobenius ratio.  Every bf16 case is also run with fp32 output, which carries the
  unwidened check.
Packed words, fp16 scales and patched weights are compared bit for bit.
"""
import numpy as np
import torch

from oracle import pdelta_oracle as orc
from paper_2512_19720_amd import binding as pd
from paper_2512_19720_amd import synth

DEV = "cuda:0"
REL_FROB = 1e-3
MAX_ABS_OVER_RMS = 1e-2


def to_dev(bits: np.ndarray, dtype: int) -> torch.Tensor:
    return synth.bits_to_torch(bits, dtype, DEV)


def words_dev(B: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(B).view(np.int32).copy()).to(DEV)


def words_host(B: torch.Tensor) -> np.ndarray:
    return B.cpu().numpy().view(np.uint32)


def f16_dev(bits: np.ndarray) -> torch.Tensor:
    return synth.bits_to_torch(bits, synth.F16, DEV)


def y_to_f64(Y: torch.Tensor) -> np.ndarray:
    return Y.detach().to(torch.float64).cpu().numpy()


def bf16_ulp(x: np.ndarray) -> np.ndarray:
    e = np.floor(np.log2(np.maximum(np.abs(x), 2.0 ** -126)))
    return 2.0 ** (e - 7)


def check_y(Y_gpu: torch.Tensor, Y_ref64: np.ndarray, what: str = ""):
    got = y_to_f64(Y_gpu)
    assert got.shape == Y_ref64.shape, what
    assert np.isfinite(got).all(), what
    rms = float(np.sqrt(np.mean(Y_ref64 ** 2)))
    ref = Y_ref64
    ref_norm = max(float(np.linalg.norm(ref)), 1e-300)
    bound = np.full(ref.shape, MAX_ABS_OVER_RMS * rms)
    frob_bound = REL_FROB
    if Y_gpu.dtype == torch.bfloat16:
        half_ulp = 0.5 * bf16_ulp(ref)
        bound = bound + half_ulp
        frob_bound += float(np.linalg.norm(half_ulp)) / ref_norm
    err = np.abs(got - ref)
    frob = float(np.linalg.norm(got - ref)) / ref_norm
    assert frob <= frob_bound, f"{what}: relative Frobenius error {frob:.3e} > {frob_bound:.3e}"
    worst = float((err / bound).max())
    assert worst <= 1.0, f"{what}: max |err| is {worst:.3f} x the bound (rms {rms:.3e})"
    return frob, float(err.max() / rms)


def gpu_linear(axis, X, W_b, B, v, y_dtype=None):
    fn = pd.pdelta_linear_row if axis == orc.ROW else pd.pdelta_linear_col
    Y = fn(X, W_b, B, v, out_dtype=y_dtype)
    torch.cuda.synchronize()
    return Y


def make_case(d_out, d_in, M, dtype, sigma_axis, seed):
    """Host bits + device tensors + oracle pack of one synthetic layer (delta given directly,
    so the pack inputs are W_f := dW, W_b := 0)."""
    L = synth.layer_host(d_out, d_in, M, dtype, sigma_axis, seed)
    zero = np.zeros_like(L["dW"])
    B, v_row, v_col = orc.pack(L["dW"], zero, dtype)
    L.update(B=B, v_row=v_row, v_col=v_col)
    L["d"] = {"X": to_dev(L["X"], dtype), "W_b": to_dev(L["W_b"], dtype), "dW": to_dev(L["dW"], dtype),
              "B": words_dev(B), "v_row": f16_dev(v_row), "v_col": f16_dev(v_col)}
    return L
