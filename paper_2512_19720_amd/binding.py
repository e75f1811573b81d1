"""Thin Python binding of the pdelta C ABI (``include/pdelta.h``).

Argument marshalling only: torch supplies device memory and the current stream, every step of
the path runs in the HIP kernels of ``libpdelta.so``.  There is no fallback of any kind: if the
library has not been built, or a call is rejected, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

F16, BF16, F32 = 0, 1, 2
ROW, COL = 0, 1

OK, EINVAL, ESHAPE, EALIGN, EDTYPE, EWORKSPACE, EHIP = 0, -1, -2, -3, -4, -5, -6

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libpdelta.so")
_lib = None


class PdeltaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib().pdelta_status_string(status).decode()} ({status})")


def lib() -> ctypes.CDLL:
    """The loaded C library.  Raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2512_19720_amd.build` "
                "(hipcc, gfx950).  The pdelta path has no CPU or PyTorch fallback.")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
        L.pdelta_pack_workspace_bytes.restype = sz
        L.pdelta_pack_workspace_bytes.argtypes = [i64, i64]
        L.pdelta_pack.restype = i32
        L.pdelta_pack.argtypes = [vp, vp, i64, i64, i32, vp, vp, vp, vp, sz, vp]
        for name in ("pdelta_linear_row", "pdelta_linear_col"):
            f = getattr(L, name)
            f.restype = i32
            f.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, i32, vp]
        L.pdelta_patch.restype = i32
        L.pdelta_patch.argtypes = [vp, vp, vp, i32, vp, i64, i64, i32, vp]
        L.pdelta_status_string.restype = ctypes.c_char_p
        L.pdelta_status_string.argtypes = [i32]
        _lib = L
    return _lib


def dtype_code(t: torch.dtype) -> int:
    if t == torch.float16:
        return F16
    if t == torch.bfloat16:
        return BF16
    if t == torch.float32:
        return F32
    raise TypeError(f"unsupported dtype {t}")


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, name: str) -> int:
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous tensor on the GPU")
    return t.data_ptr()


def _check(rc: int, where: str):
    if rc != OK:
        raise PdeltaError(rc, where)


def pdelta_pack_workspace_bytes(d_out: int, d_in: int) -> int:
    return int(lib().pdelta_pack_workspace_bytes(d_out, d_in))


def pdelta_pack(W_f: torch.Tensor, W_b: torch.Tensor, want_row: bool = True, want_col: bool = True,
                out=None, workspace: torch.Tensor | None = None):
    """(B_packed int32 [d_out, d_in/32], v_row fp16 [d_out] | None, v_col fp16 [d_in] | None)."""
    d_out, d_in = W_b.shape
    if W_f.shape != W_b.shape or W_f.dtype != W_b.dtype:
        raise ValueError("W_f and W_b must agree in shape and dtype")
    dev = W_b.device
    if out is None:
        B = torch.empty((d_out, d_in // 32), dtype=torch.int32, device=dev)
        v_row = torch.empty(d_out, dtype=torch.float16, device=dev) if want_row else None
        v_col = torch.empty(d_in, dtype=torch.float16, device=dev) if want_col else None
    else:
        B, v_row, v_col = out
    if workspace is None:
        workspace = torch.empty(pdelta_pack_workspace_bytes(d_out, d_in), dtype=torch.uint8, device=dev)
    rc = lib().pdelta_pack(_dev(W_f, "W_f"), _dev(W_b, "W_b"), d_out, d_in, dtype_code(W_b.dtype),
                           _dev(B, "B_packed"),
                           _dev(v_row, "v_row") if v_row is not None else None,
                           _dev(v_col, "v_col") if v_col is not None else None,
                           _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                           _stream())
    _check(rc, "pdelta_pack")
    return B, v_row, v_col


def _linear(fn_name: str, X, W_b, B_packed, v, out, out_dtype):
    M, d_in = X.shape
    d_out = W_b.shape[0]
    if W_b.shape[1] != d_in or X.dtype != W_b.dtype:
        raise ValueError("X and W_b must agree in d_in and dtype")
    if out is None:
        out = torch.empty((M, d_out), dtype=out_dtype or X.dtype, device=X.device)
    rc = getattr(lib(), fn_name)(_dev(X, "X"), _dev(W_b, "W_b"), _dev(B_packed, "B_packed"),
                                 _dev(v, "v"), _dev(out, "Y"), M, d_out, d_in,
                                 dtype_code(X.dtype), dtype_code(out.dtype), _stream())
    _check(rc, fn_name)
    return out


def pdelta_linear_row(X, W_b, B_packed, v_row, out=None, out_dtype=None):
    """Y = X W_b^T + v_row (.) (X B^T), v_row fp16 [d_out]."""
    return _linear("pdelta_linear_row", X, W_b, B_packed, v_row, out, out_dtype)


def pdelta_linear_col(X, W_b, B_packed, v_col, out=None, out_dtype=None):
    """Y = X W_b^T + (X (.) v_col) B^T, v_col fp16 [d_in]."""
    return _linear("pdelta_linear_col", X, W_b, B_packed, v_col, out, out_dtype)


def pdelta_patch(W_b, B_packed, v, axis: int, out=None):
    """W_out = round(W_b + v (.) B); pass out=W_b to merge in place."""
    d_out, d_in = W_b.shape
    if out is None:
        out = torch.empty_like(W_b)
    rc = lib().pdelta_patch(_dev(W_b, "W_b"), _dev(B_packed, "B_packed"), _dev(v, "v"), axis,
                            _dev(out, "W_out"), d_out, d_in, dtype_code(W_b.dtype), _stream())
    _check(rc, "pdelta_patch")
    return out
