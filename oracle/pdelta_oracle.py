"""ctypes front end of the CPU oracle (``pdelta_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  The product package never imports this module and this
module never imports the product package.

All arrays are numpy, on the host.  16-bit floating inputs travel as their raw bit patterns
(``uint16``); ``np.float16`` arrays are accepted and viewed, bf16 must already be ``uint16``.
Linear and patch results come back as ``float64`` so that the caller decides about rounding.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

F16, BF16 = 0, 1
ROW, COL = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pdelta_oracle.c")
_LIB = os.path.join(_HERE, "libpdelta_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math: fp64 semantics stay IEEE)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def use_library(path: str) -> None:
    """Load the oracle from `path` instead of building pdelta_oracle.c.  Only the mutation test
    calls this (through the pytest option --oracle-lib of its child run): it points the pins at
    deliberately broken copies of the oracle to show that they notice.  Must come before the
    first call into the oracle."""
    global _lib_override
    if _lib is not None:
        raise RuntimeError("the oracle library is already loaded")
    _lib_override = path


_lib_override = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_lib_override or build())
        i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        lib.pdelta_ref_decode.restype = ctypes.c_double
        lib.pdelta_ref_decode.argtypes = [ctypes.c_uint16, i32]
        lib.pdelta_ref_rne_f16.restype = ctypes.c_uint16
        lib.pdelta_ref_rne_f16.argtypes = [ctypes.c_double]
        lib.pdelta_ref_rne_bf16.restype = ctypes.c_uint16
        lib.pdelta_ref_rne_bf16.argtypes = [ctypes.c_double]
        lib.pdelta_ref_decode_array.argtypes = [vp, i64, i32, vp]
        lib.pdelta_ref_decode_array.restype = None
        lib.pdelta_ref_rne_array.argtypes = [vp, i64, i32, vp]
        lib.pdelta_ref_rne_array.restype = None
        lib.pdelta_pack_ref.argtypes = [vp, vp, i64, i64, i32, vp, vp, vp]
        lib.pdelta_unpack_ref.argtypes = [vp, i64, i64, vp]
        lib.pdelta_patch_ref.argtypes = [vp, vp, vp, i32, i64, i64, i32, vp]
        lib.pdelta_patch_round_ref.argtypes = [vp, vp, vp, i32, i64, i64, i32, vp]
        lib.pdelta_linear_ref.argtypes = [vp, vp, vp, vp, i32, i64, i64, i64, i32, vp]
        lib.pdelta_linear_ref_at.argtypes = [vp, vp, vp, vp, i32, i64, i64, i64, i32, i64, vp, vp, vp]
        lib.pdelta_grad_v_ref.argtypes = [vp, vp, vp, i32, i64, i64, i64, i32, vp]
        lib.pdelta_pack_group_ref.argtypes = [vp, vp, i64, i64, i32, i64, i64, vp, vp]
        lib.pdelta_patch_group_ref.argtypes = [vp, vp, vp, i64, i64, i64, i64, i32, vp]
        lib.pdelta_patch_group_round_ref.argtypes = [vp, vp, vp, i64, i64, i64, i64, i32, vp]
        lib.pdelta_linear_group_ref.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, i32, vp]
        lib.pdelta_linear_group_ref_at.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, i32, i64, vp, vp, vp]
        lib.pdelta_ref_threads.restype = i32
        _lib = lib
    return _lib


def _bits16(a) -> np.ndarray:
    a = np.asarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError(f"16-bit patterns expected (float16 or uint16), got {a.dtype}")
    return np.ascontiguousarray(a)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"{what}: oracle rejected the arguments (rc={rc})")


def words_per_row(d_in: int) -> int:
    return (d_in + 31) // 32


def decode(bits, dtype: int = F16) -> np.ndarray:
    """Exact fp64 value of each 16-bit pattern."""
    lib = _load()
    b = _bits16(bits)
    out = np.empty(b.shape, dtype=np.float64)
    lib.pdelta_ref_decode_array(_ptr(b), b.size, dtype, _ptr(out))
    return out


def rne(x, dtype: int = F16) -> np.ndarray:
    """Round fp64 values to nearest-even in the 16-bit format; returns the bit patterns."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty(x.shape, dtype=np.uint16)
    lib.pdelta_ref_rne_array(_ptr(x), x.size, dtype, _ptr(out))
    return out


def pack(W_f, W_b, w_dtype: int = F16, want_row: bool = True, want_col: bool = True):
    """(B_packed uint32 [d_out, ceil(d_in/32)], v_row fp16 bits [d_out], v_col fp16 bits [d_in])."""
    lib = _load()
    wf, wb = _bits16(W_f), _bits16(W_b)
    if wf.ndim != 2 or wf.shape != wb.shape:
        raise ValueError("W_f and W_b must be 2-D and of equal shape")
    d_out, d_in = wf.shape
    B = np.empty((d_out, words_per_row(d_in)), dtype=np.uint32)
    v_row = np.empty(d_out, dtype=np.uint16) if want_row else None
    v_col = np.empty(d_in, dtype=np.uint16) if want_col else None
    rc = lib.pdelta_pack_ref(_ptr(wf), _ptr(wb), d_out, d_in, w_dtype, _ptr(B),
                             _ptr(v_row) if want_row else None,
                             _ptr(v_col) if want_col else None)
    _check(rc, "pack")
    return B, v_row, v_col


def unpack(B_packed, d_in: int) -> np.ndarray:
    lib = _load()
    B = np.ascontiguousarray(B_packed, dtype=np.uint32)
    d_out = B.shape[0]
    if B.shape[1] != words_per_row(d_in):
        raise ValueError("B_packed has the wrong number of words per row")
    out = np.empty((d_out, d_in), dtype=np.float64)
    _check(lib.pdelta_unpack_ref(_ptr(B), d_out, d_in, _ptr(out)), "unpack")
    return out


def _patch_args(W_b, B_packed, v, axis):
    wb = _bits16(W_b)
    d_out, d_in = wb.shape
    B = np.ascontiguousarray(B_packed, dtype=np.uint32)
    vv = _bits16(v)
    if B.shape != (d_out, words_per_row(d_in)):
        raise ValueError("B_packed shape does not match W_b")
    if vv.shape != ((d_out,) if axis == ROW else (d_in,)):
        raise ValueError("v has the wrong length for this axis")
    return wb, B, vv, d_out, d_in


def patch(W_b, B_packed, v, axis: int, w_dtype: int = F16) -> np.ndarray:
    """Exact fp64 W_hat = v (.) B + W_b."""
    lib = _load()
    wb, B, vv, d_out, d_in = _patch_args(W_b, B_packed, v, axis)
    out = np.empty((d_out, d_in), dtype=np.float64)
    _check(lib.pdelta_patch_ref(_ptr(wb), _ptr(B), _ptr(vv), axis, d_out, d_in, w_dtype,
                                _ptr(out)), "patch")
    return out


def patch_round(W_b, B_packed, v, axis: int, w_dtype: int = F16) -> np.ndarray:
    """W_hat rounded once (RNE) to the weight dtype; returns bit patterns."""
    lib = _load()
    wb, B, vv, d_out, d_in = _patch_args(W_b, B_packed, v, axis)
    out = np.empty((d_out, d_in), dtype=np.uint16)
    _check(lib.pdelta_patch_round_ref(_ptr(wb), _ptr(B), _ptr(vv), axis, d_out, d_in, w_dtype,
                                      _ptr(out)), "patch_round")
    return out


def linear(X, W_b, B_packed, v, axis: int, x_dtype: int = F16) -> np.ndarray:
    """fp64 Y [M, d_out] = X W_hat^T with W_hat rebuilt densely."""
    lib = _load()
    wb, B, vv, d_out, d_in = _patch_args(W_b, B_packed, v, axis)
    x = _bits16(X)
    if x.ndim != 2 or x.shape[1] != d_in:
        raise ValueError("X must be [M, d_in]")
    M = x.shape[0]
    out = np.empty((M, d_out), dtype=np.float64)
    _check(lib.pdelta_linear_ref(_ptr(x), _ptr(wb), _ptr(B), _ptr(vv), axis, M, d_out, d_in,
                                 x_dtype, _ptr(out)), "linear")
    return out


def linear_at(X, W_b, B_packed, v, axis: int, m_idx, o_idx, x_dtype: int = F16) -> np.ndarray:
    """fp64 Y[m_idx[s], o_idx[s]] for each s, one dot product per sample."""
    lib = _load()
    wb, B, vv, d_out, d_in = _patch_args(W_b, B_packed, v, axis)
    x = _bits16(X)
    if x.ndim != 2 or x.shape[1] != d_in:
        raise ValueError("X must be [M, d_in]")
    mi = np.ascontiguousarray(m_idx, dtype=np.int64)
    oi = np.ascontiguousarray(o_idx, dtype=np.int64)
    if mi.shape != oi.shape or mi.ndim != 1:
        raise ValueError("m_idx and o_idx must be 1-D and of equal length")
    out = np.empty(mi.shape, dtype=np.float64)
    _check(lib.pdelta_linear_ref_at(_ptr(x), _ptr(wb), _ptr(B), _ptr(vv), axis, x.shape[0],
                                    d_out, d_in, x_dtype, mi.size, _ptr(mi), _ptr(oi),
                                    _ptr(out)), "linear_at")
    return out


def grad_v(X, dY, B_packed, axis: int, dtype: int = F16) -> np.ndarray:
    """dL/dv (fp64) for upstream gradient dY: [d_out] in row mode, [d_in] in column mode."""
    X, dY = _bits16(X), _bits16(dY)
    B = np.ascontiguousarray(B_packed, dtype=np.uint32)
    M, d_in = X.shape
    d_out = dY.shape[1]
    assert dY.shape[0] == M and B.shape == (d_out, words_per_row(d_in))
    out = np.empty(d_out if axis == ROW else d_in, dtype=np.float64)
    _check(_load().pdelta_grad_v_ref(_ptr(X), _ptr(dY), _ptr(B), axis, M, d_out, d_in, dtype, _ptr(out)),
           "pdelta_grad_v_ref")
    return out


def linear_variants(X, W_b, Bs, vs, axis, x_dtype: int = F16) -> np.ndarray:
    """R requests that share W_b: row r of the result is the delta linear layer (Eq. 1 inside
    the layer forward) of token X[r] with request r's own (Bs[r], vs[r]) and its own axis (the
    per-layer Row/Col selection may have chosen differently for different fine-tunes of one
    base); `axis` is one mode for all requests or a sequence with one mode per request.  Written
    out as what it is: R independent single-token layers, one call of `linear` each."""
    X = _bits16(X)
    axes = [axis] * X.shape[0] if isinstance(axis, (int, np.integer)) else list(axis)
    if len(axes) != X.shape[0]:
        raise ValueError("one axis per request")
    rows = [linear(X[r:r + 1], W_b, Bs[r], vs[r], axes[r], x_dtype)[0] for r in range(X.shape[0])]
    return np.stack(rows) if rows else np.zeros((0, _bits16(W_b).shape[0]))


# ---- blockwise ("per-group") and scalar scales ----------------------------------------------
# v is [v_rows, d_in // group] fp16 bits with v_rows = d_out (a scale per output row and group of
# `group` consecutive inputs) or 1 (shared by all rows); v_rows = 1 with group = d_in is one
# scalar for the whole matrix.

def _group_args(W_b, B_packed, v, group):
    wb = _bits16(W_b)
    d_out, d_in = wb.shape
    B = np.ascontiguousarray(B_packed, dtype=np.uint32)
    vv = _bits16(v)
    if B.shape != (d_out, words_per_row(d_in)):
        raise ValueError("B_packed shape does not match W_b")
    if group <= 0 or d_in % group != 0 or vv.ndim != 2 or vv.shape[1] != d_in // group or vv.shape[0] not in (1, d_out):
        raise ValueError("v must be [d_out or 1, d_in // group] and group must divide d_in")
    return wb, B, vv, d_out, d_in, vv.shape[0]


def pack_group(W_f, W_b, group: int, shared_rows: bool = False, w_dtype: int = F16):
    """(B_packed, v [d_out or 1, d_in // group] fp16 bits): signs as `pack`, v = mean |dW| per block."""
    lib = _load()
    wf, wb = _bits16(W_f), _bits16(W_b)
    if wf.ndim != 2 or wf.shape != wb.shape:
        raise ValueError("W_f and W_b must be 2-D and of equal shape")
    d_out, d_in = wf.shape
    if group <= 0 or d_in % group != 0:
        raise ValueError("group must divide d_in")
    v_rows = 1 if shared_rows else d_out
    B = np.empty((d_out, words_per_row(d_in)), dtype=np.uint32)
    v = np.empty((v_rows, d_in // group), dtype=np.uint16)
    _check(lib.pdelta_pack_group_ref(_ptr(wf), _ptr(wb), d_out, d_in, w_dtype, group, v_rows, _ptr(B), _ptr(v)),
           "pack_group")
    return B, v


def patch_group(W_b, B_packed, v, group: int, w_dtype: int = F16) -> np.ndarray:
    """Exact fp64 W_hat = W_b + scale(o, i) B with blockwise scales."""
    wb, B, vv, d_out, d_in, v_rows = _group_args(W_b, B_packed, v, group)
    out = np.empty((d_out, d_in), dtype=np.float64)
    _check(_load().pdelta_patch_group_ref(_ptr(wb), _ptr(B), _ptr(vv), group, v_rows, d_out, d_in, w_dtype,
                                          _ptr(out)), "patch_group")
    return out


def patch_group_round(W_b, B_packed, v, group: int, w_dtype: int = F16) -> np.ndarray:
    wb, B, vv, d_out, d_in, v_rows = _group_args(W_b, B_packed, v, group)
    out = np.empty((d_out, d_in), dtype=np.uint16)
    _check(_load().pdelta_patch_group_round_ref(_ptr(wb), _ptr(B), _ptr(vv), group, v_rows, d_out, d_in, w_dtype,
                                                _ptr(out)), "patch_group_round")
    return out


def linear_group(X, W_b, B_packed, v, group: int, x_dtype: int = F16) -> np.ndarray:
    """fp64 Y [M, d_out] = X W_hat^T with W_hat rebuilt densely from blockwise scales."""
    wb, B, vv, d_out, d_in, v_rows = _group_args(W_b, B_packed, v, group)
    x = _bits16(X)
    if x.ndim != 2 or x.shape[1] != d_in:
        raise ValueError("X must be [M, d_in]")
    out = np.empty((x.shape[0], d_out), dtype=np.float64)
    _check(_load().pdelta_linear_group_ref(_ptr(x), _ptr(wb), _ptr(B), _ptr(vv), group, v_rows, x.shape[0],
                                           d_out, d_in, x_dtype, _ptr(out)), "linear_group")
    return out


def linear_group_at(X, W_b, B_packed, v, group: int, m_idx, o_idx, x_dtype: int = F16) -> np.ndarray:
    wb, B, vv, d_out, d_in, v_rows = _group_args(W_b, B_packed, v, group)
    x = _bits16(X)
    mi = np.ascontiguousarray(m_idx, dtype=np.int64)
    oi = np.ascontiguousarray(o_idx, dtype=np.int64)
    out = np.empty(mi.shape, dtype=np.float64)
    _check(_load().pdelta_linear_group_ref_at(_ptr(x), _ptr(wb), _ptr(B), _ptr(vv), group, v_rows, x.shape[0],
                                              d_out, d_in, x_dtype, mi.size, _ptr(mi), _ptr(oi), _ptr(out)),
           "linear_group_at")
    return out


def threads() -> int:
    return int(_load().pdelta_ref_threads())
