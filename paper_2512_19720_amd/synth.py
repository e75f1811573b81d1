"""Seeded synthetic inputs shaped like the paper's workloads (LLM linear projections).

This module only draws random tensors and converts number formats.  It contains none of the
method's arithmetic (no sign, no packing, no scale, no patched weight): both the GPU library
and the CPU oracle are fed from here and each does all of the method's work on its own.

Recipe (one linear layer, d_out x d_in):
  W_b      ~ N(0, 0.02^2)                                   base weights
  sigma    = exp(N(ln 1e-3, 0.5^2))   one per output row ("row") or per input column ("col")
  Delta W  = sigma (broadcast along the other axis) * N(0, 1), optionally with a Bernoulli
             fraction of entries set to exactly 0
  W_f      = round_to_storage(W_b + Delta W)                only where a fine-tuned matrix is
             needed as such (the offline pack workload)
  X        ~ N(0, 1), [M, d_in]
all rounded to the 16-bit storage format (fp16 or bf16).  The fine-tuned/base pairs the paper
compresses are Llama-3.1-8B-like projections; no trained weights exist here, so these stand in.

Seeds: ``seed_for(config, tensor_index)`` = 251219720 + 1000 * config + tensor_index.
"""
from __future__ import annotations

import numpy as np

F16, BF16 = 0, 1

BASE_SEED = 251219720
W_STD = 0.02
SIGMA_LOG_MEAN = float(np.log(1e-3))
SIGMA_LOG_STD = 0.5

# The 7B-Llama-shaped stack: per transformer block q, k, v, o, gate, up, down as (d_out, d_in).
STACK_BLOCK = (("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
               ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008))
STACK_BLOCKS = 32
PREFILL_SHAPES = ((11008, 4096), (4096, 11008), (14336, 4096))


def seed_for(config: int, tensor_index: int = 0) -> int:
    return BASE_SEED + 1000 * config + tensor_index


# ---- number-format helpers (host) ----------------------------------------------------------

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bfloat16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage_bits(a: np.ndarray, dtype: int) -> np.ndarray:
    """fp32/fp64 values -> uint16 bit patterns of the 16-bit storage format."""
    if dtype == BF16:
        return f32_to_bf16_bits(np.asarray(a, dtype=np.float32))
    return np.asarray(a, dtype=np.float32).astype(np.float16).view(np.uint16)


def from_storage_bits(b: np.ndarray, dtype: int) -> np.ndarray:
    """uint16 bit patterns -> fp32 values (exact)."""
    if dtype == BF16:
        return bf16_bits_to_f32(b)
    return np.ascontiguousarray(b, dtype=np.uint16).view(np.float16).astype(np.float32)


# ---- host generator (numpy, PCG64) ----------------------------------------------------------

def layer_host(d_out: int, d_in: int, M: int, dtype: int, sigma_axis: str, seed: int,
               zero_frac: float = 0.0, with_wf: bool = False) -> dict:
    """One layer's inputs as uint16 bit patterns: W_b, dW [d_out,d_in], X [M,d_in] (+ W_f)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    W_b = (rng.standard_normal((d_out, d_in), dtype=np.float32) * np.float32(W_STD))
    n_sigma = d_out if sigma_axis == "row" else d_in
    sigma = np.exp(rng.normal(SIGMA_LOG_MEAN, SIGMA_LOG_STD, n_sigma)).astype(np.float32)
    dW = rng.standard_normal((d_out, d_in), dtype=np.float32)
    dW *= sigma[:, None] if sigma_axis == "row" else sigma[None, :]
    if zero_frac > 0.0:
        dW[rng.random((d_out, d_in), dtype=np.float32) < zero_frac] = 0.0
    X = rng.standard_normal((M, d_in), dtype=np.float32)
    out = {"W_b": to_storage_bits(W_b, dtype), "dW": to_storage_bits(dW, dtype),
           "X": to_storage_bits(X, dtype), "dtype": dtype, "sigma_axis": sigma_axis}
    if with_wf:
        wb = from_storage_bits(out["W_b"], dtype)
        dw = from_storage_bits(out["dW"], dtype)
        out["W_f"] = to_storage_bits(wb + dw, dtype)
    return out


# ---- device generator (torch, for the multi-GB stacks) --------------------------------------

def torch_dtype(dtype: int):
    import torch
    return torch.bfloat16 if dtype == BF16 else torch.float16


def bits_to_torch(bits: np.ndarray, dtype: int, device):
    """uint16 bit patterns (host) -> torch tensor of the storage dtype on `device`."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16).copy())
    return t.view(torch_dtype(dtype)).to(device)


def torch_to_bits(t) -> np.ndarray:
    """torch fp16/bf16 tensor (any device) -> uint16 bit patterns on the host."""
    import torch
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def layer_device(d_out: int, d_in: int, dtype: int, sigma_axis: str, seed: int, device,
                 zero_frac: float = 0.0, with_wf: bool = False) -> dict:
    """One layer's W_b and dW (and W_f) as torch tensors drawn on `device`."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    td = torch_dtype(dtype)
    W_b = (torch.randn((d_out, d_in), generator=g, device=device, dtype=torch.float32) * W_STD).to(td)
    n_sigma = d_out if sigma_axis == "row" else d_in
    sigma = torch.exp(torch.randn(n_sigma, generator=g, device=device, dtype=torch.float32)
                      * SIGMA_LOG_STD + SIGMA_LOG_MEAN)
    dW = torch.randn((d_out, d_in), generator=g, device=device, dtype=torch.float32)
    dW *= sigma[:, None] if sigma_axis == "row" else sigma[None, :]
    if zero_frac > 0.0:
        keep = torch.rand((d_out, d_in), generator=g, device=device) >= zero_frac
        dW *= keep
    out = {"W_b": W_b, "dW": dW.to(td), "dtype": dtype, "sigma_axis": sigma_axis}
    if with_wf:
        out["W_f"] = (W_b.float() + out["dW"].float()).to(td)
    return out


def x_device(M: int, d_in: int, dtype: int, seed: int, device):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return torch.randn((M, d_in), generator=g, device=device, dtype=torch.float32).to(torch_dtype(dtype))


def stack_shapes(blocks: int = STACK_BLOCKS):
    """[(name, d_out, d_in, sigma_axis)] for the 7 x `blocks` linears; even blocks carry
    row-structured deltas, odd blocks column-structured ones."""
    out = []
    for b in range(blocks):
        axis = "row" if b % 2 == 0 else "col"
        for name, d_out, d_in in STACK_BLOCK:
            out.append((f"blk{b}.{name}", d_out, d_in, axis))
    return out
