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
ROW, COL, PER_REQUEST = 0, 1, 2

OK, EINVAL, ESHAPE, EALIGN, EDTYPE, EWORKSPACE, EHIP = 0, -1, -2, -3, -4, -5, -6

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libpdelta.so")
_lib = None


class PdeltaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib().pdelta_status_string(status).decode()} ({status})")


class Layer(ctypes.Structure):
    """Mirror of the C struct ``pdelta_layer``."""
    _fields_ = [("X", ctypes.c_void_p), ("W_b", ctypes.c_void_p), ("B_packed", ctypes.c_void_p),
                ("v", ctypes.c_void_p), ("Y", ctypes.c_void_p), ("d_out", ctypes.c_int64),
                ("d_in", ctypes.c_int64), ("axis", ctypes.c_int32), ("first_block", ctypes.c_int32)]


class Variant(ctypes.Structure):
    """Mirror of the C struct ``pdelta_variant``."""
    _fields_ = [("B_packed", ctypes.c_void_p), ("v", ctypes.c_void_p), ("axis", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


class PackJob(ctypes.Structure):
    """Mirror of the C struct ``pdelta_pack_job``."""
    _fields_ = [("W_f", ctypes.c_void_p), ("W_b", ctypes.c_void_p), ("B_packed", ctypes.c_void_p),
                ("v_row", ctypes.c_void_p), ("v_col", ctypes.c_void_p), ("workspace", ctypes.c_void_p),
                ("workspace_bytes", ctypes.c_size_t), ("d_out", ctypes.c_int64), ("d_in", ctypes.c_int64),
                ("first_tile", ctypes.c_int32), ("first_fin_block", ctypes.c_int32),
                ("tile_blocks", ctypes.c_int32), ("reserved", ctypes.c_int32)]


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
        L.pdelta_pack_noalloc_max_bytes.restype = sz
        L.pdelta_pack_noalloc_max_bytes.argtypes = []
        L.pdelta_pack_noalloc.restype = i32
        L.pdelta_pack_noalloc.argtypes = [vp, vp, i64, i64, i32, vp, vp, vp, vp]
        for name in ("pdelta_linear_row", "pdelta_linear_col"):
            f = getattr(L, name)
            f.restype = i32
            f.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, i32, vp]
        L.pdelta_patch.restype = i32
        L.pdelta_patch.argtypes = [vp, vp, vp, i32, vp, i64, i64, i32, vp]
        L.pdelta_linear_batch_plan.restype = i32
        L.pdelta_linear_batch_plan.argtypes = [ctypes.POINTER(Layer), ctypes.c_int32]
        L.pdelta_linear_batch.restype = i32
        L.pdelta_linear_batch.argtypes = [ctypes.POINTER(Layer), vp, ctypes.c_int32, i64, i32, i32, vp]
        L.pdelta_patch_batch.restype = i32
        L.pdelta_patch_batch.argtypes = [ctypes.POINTER(Layer), vp, ctypes.c_int32, i32, vp]
        L.pdelta_pack_batch_plan.restype = i32
        L.pdelta_pack_batch_plan.argtypes = [ctypes.POINTER(PackJob), ctypes.c_int32]
        L.pdelta_pack_batch.restype = i32
        L.pdelta_pack_batch.argtypes = [ctypes.POINTER(PackJob), vp, ctypes.c_int32, i32, vp]
        L.pdelta_linear_variants.restype = i32
        L.pdelta_linear_variants.argtypes = [vp, vp, ctypes.POINTER(Variant), vp, ctypes.c_int32, i32, vp, i64, i64,
                                             i32, i32, vp]
        L.pdelta_grad_v_workspace_bytes.restype = sz
        L.pdelta_grad_v_workspace_bytes.argtypes = [i64, i64, i64, i32]
        L.pdelta_grad_v.restype = i32
        L.pdelta_grad_v.argtypes = [vp, vp, vp, i32, vp, i64, i64, i64, i32, vp, sz, vp]
        L.pdelta_pack_group_workspace_bytes.restype = sz
        L.pdelta_pack_group_workspace_bytes.argtypes = [i64, i64, i64, i32]
        L.pdelta_pack_group.restype = i32
        L.pdelta_pack_group.argtypes = [vp, vp, i64, i64, i32, i64, i32, vp, vp, vp, sz, vp]
        L.pdelta_linear_group.restype = i32
        L.pdelta_linear_group.argtypes = [vp, vp, vp, vp, i64, i32, vp, i64, i64, i64, i32, i32, vp]
        L.pdelta_patch_group.restype = i32
        L.pdelta_patch_group.argtypes = [vp, vp, vp, i64, i32, vp, i64, i64, i32, vp]
        L.pdelta_probe_read_stream.restype = i32
        L.pdelta_probe_read_stream.argtypes = [vp, sz, vp, vp]
        L.pdelta_probe_mfma.restype = i32
        L.pdelta_probe_mfma.argtypes = [i32, i32, i32, vp, vp]
        L.pdelta_probe_prefill_parts.restype = i32
        L.pdelta_probe_prefill_parts.argtypes = [i32, vp, vp, vp, vp, vp, i64, i64, i64, i32, vp]
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


try:                                       # raw current-stream handle without building a Stream object
    _raw_stream = torch._C._cuda_getCurrentRawStream
except AttributeError:                     # pragma: no cover - older torch
    _raw_stream = None


def _stream() -> int:
    if _raw_stream is not None:
        return _raw_stream(torch.cuda.current_device())
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


def pdelta_pack_noalloc(W_f: torch.Tensor, W_b: torch.Tensor, out):
    """pdelta_pack into the caller's ``out = (B_packed, v_row | None, v_col | None)`` with the
    partial sums in the library's own scratch array: nothing is allocated, here or in the library."""
    d_out, d_in = W_b.shape
    if W_f.shape != W_b.shape or W_f.dtype != W_b.dtype:
        raise ValueError("W_f and W_b must agree in shape and dtype")
    B, v_row, v_col = out
    rc = lib().pdelta_pack_noalloc(_dev(W_f, "W_f"), _dev(W_b, "W_b"), d_out, d_in, dtype_code(W_b.dtype),
                                   _dev(B, "B_packed"),
                                   _dev(v_row, "v_row") if v_row is not None else None,
                                   _dev(v_col, "v_col") if v_col is not None else None, _stream())
    _check(rc, "pdelta_pack_noalloc")
    return B, v_row, v_col


_DTYPE_CODE = {torch.float16: F16, torch.bfloat16: BF16, torch.float32: F32}


def _linear(fn_name: str, X, W_b, B_packed, v, out, out_dtype):
    M, d_in = X.shape
    d_out = W_b.shape[0]
    if W_b.shape[1] != d_in or X.dtype != W_b.dtype:
        raise ValueError("X and W_b must agree in d_in and dtype")
    if out is None:
        out = torch.empty((M, d_out), dtype=out_dtype or X.dtype, device=X.device)
    fn = getattr(_lib, fn_name) if _lib is not None else getattr(lib(), fn_name)
    rc = fn(_dev(X, "X"), _dev(W_b, "W_b"), _dev(B_packed, "B_packed"), _dev(v, "v"), _dev(out, "Y"),
            M, d_out, d_in, _DTYPE_CODE[X.dtype], _DTYPE_CODE[out.dtype], _stream())
    if rc != OK:
        raise PdeltaError(rc, fn_name)
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


class BatchPlan:
    """Host and device copies of a planned ``pdelta_layer`` array plus the tensors they point to."""

    def __init__(self, host, device, tensors, M, x_dtype, y_dtype):
        self.host, self.device, self.tensors = host, device, tensors
        self.M, self.x_dtype, self.y_dtype = M, x_dtype, y_dtype
        self.Y = [t[4] for t in tensors]

    def __len__(self):
        return len(self.host)


def pdelta_linear_batch_plan(layers, out_dtype=None) -> BatchPlan:
    """Describe independent layers for one batched launch.

    ``layers`` is a sequence of ``(X, W_b, B_packed, v, axis)`` or ``(X, W_b, B_packed, v, axis, Y)``
    with one common batch size and dtype; missing outputs are allocated.  The descriptor array is
    planned by the library on the host and copied to the GPU once.
    """
    layers = list(layers)
    if not layers:
        raise ValueError("no layers")
    M, x_dtype = layers[0][0].shape[0], layers[0][0].dtype
    host = (Layer * len(layers))()
    tensors = []
    for k, item in enumerate(layers):
        X, W_b, B_packed, v, axis = item[:5]
        Y = item[5] if len(item) > 5 else None
        d_out, d_in = W_b.shape
        if X.shape != (M, d_in) or X.dtype != x_dtype or W_b.dtype != x_dtype:
            raise ValueError("layers of one batch share M and dtype; X and W_b must agree in d_in")
        if Y is None:
            Y = torch.empty((M, d_out), dtype=out_dtype or x_dtype, device=X.device)
        host[k] = Layer(_dev(X, "X") or None, _dev(W_b, "W_b"), _dev(B_packed, "B_packed"), _dev(v, "v"),
                        _dev(Y, "Y") or None, d_out, d_in, axis, 0)
        tensors.append((X, W_b, B_packed, v, Y))
    y_dtype = tensors[0][4].dtype
    if any(t[4].dtype != y_dtype for t in tensors):
        raise ValueError("layers of one batch share the output dtype")
    _check(lib().pdelta_linear_batch_plan(host, len(layers)), "pdelta_linear_batch_plan")
    raw = torch.frombuffer(bytearray(bytes(host)), dtype=torch.uint8)
    device = raw.to(tensors[0][0].device)
    return BatchPlan(host, device, tensors, M, dtype_code(x_dtype), dtype_code(y_dtype))


def pdelta_linear_batch(plan: BatchPlan):
    """Run every layer of the plan (one launch when the layers fit the batched decode kernel)."""
    rc = lib().pdelta_linear_batch(plan.host, plan.device.data_ptr(), len(plan), plan.M, plan.x_dtype,
                                   plan.y_dtype, _stream())
    _check(rc, "pdelta_linear_batch")
    return plan.Y


def _to_device(host_array, device) -> torch.Tensor:
    return torch.frombuffer(bytearray(bytes(host_array)), dtype=torch.uint8).to(device)


class PatchPlan:
    """Host and device copies of a planned ``pdelta_layer`` array for ``pdelta_patch_batch``."""

    def __init__(self, host, device, tensors, w_dtype):
        self.host, self.device, self.tensors, self.w_dtype = host, device, tensors, w_dtype
        self.W_out = [t[3] for t in tensors]

    def __len__(self):
        return len(self.host)


def pdelta_patch_batch_plan(layers) -> PatchPlan:
    """``layers``: sequence of ``(W_b, B_packed, v, axis)`` or ``(W_b, B_packed, v, axis, W_out)``;
    pass ``W_out = W_b`` to merge in place, omit it to allocate the outputs."""
    layers = list(layers)
    if not layers:
        raise ValueError("no layers")
    host = (Layer * len(layers))()
    tensors = []
    dt = layers[0][0].dtype
    for k, item in enumerate(layers):
        W_b, B_packed, v, axis = item[:4]
        W_out = item[4] if len(item) > 4 else torch.empty_like(W_b)
        if W_b.dtype != dt or W_out.dtype != dt or W_out.shape != W_b.shape:
            raise ValueError("layers of one batch share the weight dtype; W_out matches W_b")
        d_out, d_in = W_b.shape
        host[k] = Layer(None, _dev(W_b, "W_b"), _dev(B_packed, "B_packed"), _dev(v, "v"),
                        _dev(W_out, "W_out"), d_out, d_in, axis, 0)
        tensors.append((W_b, B_packed, v, W_out))
    _check(lib().pdelta_linear_batch_plan(host, len(layers)), "pdelta_linear_batch_plan")
    return PatchPlan(host, _to_device(host, tensors[0][0].device), tensors, dtype_code(dt))


def pdelta_patch_batch(plan: PatchPlan):
    """Merge every layer of the plan in one launch; returns the list of W_out tensors."""
    rc = lib().pdelta_patch_batch(plan.host, plan.device.data_ptr(), len(plan), plan.w_dtype, _stream())
    _check(rc, "pdelta_patch_batch")
    return plan.W_out


class PackPlan:
    """Host and device copies of a planned ``pdelta_pack_job`` array plus outputs and workspaces."""

    def __init__(self, host, device, tensors, w_dtype):
        self.host, self.device, self.tensors, self.w_dtype = host, device, tensors, w_dtype
        self.out = [(t[2], t[3], t[4]) for t in tensors]

    def __len__(self):
        return len(self.host)


def pdelta_pack_batch_plan(pairs, want_row: bool = True, want_col: bool = True, out=None) -> PackPlan:
    """``pairs``: sequence of ``(W_f, W_b)``.  Outputs ``(B_packed, v_row, v_col)`` per pair are
    allocated unless ``out`` gives them; every job gets its own workspace."""
    pairs = list(pairs)
    if not pairs:
        raise ValueError("no layers")
    host = (PackJob * len(pairs))()
    tensors = []
    dt = pairs[0][1].dtype
    for k, (W_f, W_b) in enumerate(pairs):
        if W_f.shape != W_b.shape or W_f.dtype != dt or W_b.dtype != dt:
            raise ValueError("W_f and W_b must agree in shape; one dtype per batch")
        d_out, d_in = W_b.shape
        dev = W_b.device
        if out is None:
            B = torch.empty((d_out, d_in // 32), dtype=torch.int32, device=dev)
            v_row = torch.empty(d_out, dtype=torch.float16, device=dev) if want_row else None
            v_col = torch.empty(d_in, dtype=torch.float16, device=dev) if want_col else None
        else:
            B, v_row, v_col = out[k]
        ws = torch.empty(pdelta_pack_workspace_bytes(d_out, d_in), dtype=torch.uint8, device=dev)
        host[k] = PackJob(_dev(W_f, "W_f"), _dev(W_b, "W_b"), _dev(B, "B_packed"),
                          _dev(v_row, "v_row") if v_row is not None else None,
                          _dev(v_col, "v_col") if v_col is not None else None,
                          _dev(ws, "workspace"), ws.numel(), d_out, d_in, 0, 0, 0, 0)
        tensors.append((W_f, W_b, B, v_row, v_col, ws))
    _check(lib().pdelta_pack_batch_plan(host, len(pairs)), "pdelta_pack_batch_plan")
    return PackPlan(host, _to_device(host, tensors[0][0].device), tensors, dtype_code(dt))


def pdelta_pack_batch(plan: PackPlan):
    """Pack every pair of the plan (two launches); returns [(B_packed, v_row, v_col), ...]."""
    rc = lib().pdelta_pack_batch(plan.host, plan.device.data_ptr(), len(plan), plan.w_dtype, _stream())
    _check(rc, "pdelta_pack_batch")
    return plan.out


class VariantSet:
    """Host and device copies of a ``pdelta_variant`` array plus the tensors they point to."""

    def __init__(self, variants, axis):
        """``variants``: R pairs (B_packed, v); ``axis``: ROW or COL for all of them, or a sequence
        with one axis per request."""
        variants = list(variants)
        per_request = not isinstance(axis, int)
        axes = list(axis) if per_request else [axis] * len(variants)
        if len(axes) != len(variants):
            raise ValueError("one axis per variant")
        self.axis = PER_REQUEST if per_request else axis
        self.tensors = variants
        self.host = (Variant * max(len(variants), 1))()
        for r, (B_packed, v) in enumerate(variants):
            self.host[r] = Variant(_dev(B_packed, "B_packed"), _dev(v, "v"), int(axes[r]), 0)
        self.device = _to_device(self.host, variants[0][0].device) if variants else None

    def __len__(self):
        return len(self.tensors)


def pdelta_linear_variants(X, W_b, variants: VariantSet, out=None, out_dtype=None):
    """Y[r] = X[r] W_b^T + delta of request r; ``variants`` holds R pairs (B_packed, v)."""
    R, d_in = X.shape
    d_out = W_b.shape[0]
    if R != len(variants) or W_b.shape[1] != d_in or X.dtype != W_b.dtype:
        raise ValueError("one token per variant; X and W_b must agree in d_in and dtype")
    if out is None:
        out = torch.empty((R, d_out), dtype=out_dtype or X.dtype, device=X.device)
    rc = lib().pdelta_linear_variants(_dev(X, "X") or None, _dev(W_b, "W_b"), variants.host,
                                      variants.device.data_ptr() if variants.device is not None else None,
                                      R, variants.axis, _dev(out, "Y") or None, d_out, d_in,
                                      dtype_code(X.dtype), dtype_code(out.dtype), _stream())
    _check(rc, "pdelta_linear_variants")
    return out


def pdelta_grad_v_workspace_bytes(M: int, d_out: int, d_in: int, axis: int) -> int:
    return int(lib().pdelta_grad_v_workspace_bytes(M, d_out, d_in, axis))


def pdelta_grad_v(X, dY, B_packed, axis: int, out=None, workspace: torch.Tensor | None = None):
    """dL/dv (fp32) for upstream gradient dY: [d_out] in row mode, [d_in] in column mode."""
    M, d_in = X.shape
    d_out = dY.shape[1]
    if dY.shape[0] != M or dY.dtype != X.dtype:
        raise ValueError("X and dY must agree in M and dtype")
    if out is None:
        out = torch.empty(d_out if axis == ROW else d_in, dtype=torch.float32, device=X.device)
    if workspace is None:
        workspace = torch.empty(max(pdelta_grad_v_workspace_bytes(M, d_out, d_in, axis), 16), dtype=torch.uint8,
                                device=X.device)
    rc = lib().pdelta_grad_v(_dev(X, "X") or None, _dev(dY, "dY") or None, _dev(B_packed, "B_packed"), axis,
                             _dev(out, "grad_v"), M, d_out, d_in, dtype_code(X.dtype), _dev(workspace, "workspace"),
                             workspace.numel(), _stream())
    _check(rc, "pdelta_grad_v")
    return out


# ---- blockwise ("per-group") and scalar scales ----------------------------------------------
# v is fp16 [d_out or 1, d_in // group]; one row means the scales are shared by all output rows
# (with group = d_in: one scalar for the whole matrix).

def _group_args(W_b, v, group: int):
    d_out, d_in = W_b.shape
    if v.dim() != 2 or v.shape[1] * group != d_in or v.shape[0] not in (1, d_out):
        raise ValueError("v must be [d_out or 1, d_in // group]")
    return d_out, d_in, int(v.shape[0] == 1 and d_out != 1)


def pdelta_pack_group(W_f: torch.Tensor, W_b: torch.Tensor, group: int, shared_rows: bool = False):
    """(B_packed int32 [d_out, d_in/32], v fp16 [d_out or 1, d_in // group])."""
    d_out, d_in = W_b.shape
    if W_f.shape != W_b.shape or W_f.dtype != W_b.dtype:
        raise ValueError("W_f and W_b must agree in shape and dtype")
    dev = W_b.device
    B = torch.empty((d_out, d_in // 32), dtype=torch.int32, device=dev)
    v = torch.empty((1 if shared_rows else d_out, max(d_in // max(group, 1), 1)), dtype=torch.float16, device=dev)
    need = int(lib().pdelta_pack_group_workspace_bytes(d_out, d_in, group, int(shared_rows)))
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    rc = lib().pdelta_pack_group(_dev(W_f, "W_f"), _dev(W_b, "W_b"), d_out, d_in, dtype_code(W_b.dtype), group,
                                 int(shared_rows), _dev(B, "B_packed"), _dev(v, "v"), _dev(ws, "workspace"),
                                 ws.numel(), _stream())
    _check(rc, "pdelta_pack_group")
    return B, v


def pdelta_linear_group(X, W_b, B_packed, v, group: int, out=None, out_dtype=None):
    """Y = X W_hat^T with W_hat = W_b + scale(o, i) B and blockwise scales v."""
    M, d_in = X.shape
    d_out, _, shared = _group_args(W_b, v, group)
    if W_b.shape[1] != d_in or X.dtype != W_b.dtype:
        raise ValueError("X and W_b must agree in d_in and dtype")
    if out is None:
        out = torch.empty((M, d_out), dtype=out_dtype or X.dtype, device=X.device)
    rc = lib().pdelta_linear_group(_dev(X, "X") or None, _dev(W_b, "W_b"), _dev(B_packed, "B_packed"), _dev(v, "v"),
                                   group, shared, _dev(out, "Y") or None, M, d_out, d_in, dtype_code(X.dtype),
                                   dtype_code(out.dtype), _stream())
    _check(rc, "pdelta_linear_group")
    return out


def pdelta_patch_group(W_b, B_packed, v, group: int, out=None):
    """W_out = round(W_b + scale(o, i) B); pass out=W_b to merge in place."""
    d_out, d_in, shared = _group_args(W_b, v, group)
    if out is None:
        out = torch.empty_like(W_b)
    rc = lib().pdelta_patch_group(_dev(W_b, "W_b"), _dev(B_packed, "B_packed"), _dev(v, "v"), group, shared,
                                  _dev(out, "W_out"), d_out, d_in, dtype_code(W_b.dtype), _stream())
    _check(rc, "pdelta_patch_group")
    return out


# ---- bench helpers (include/pdelta_probes.h): what this GPU sustains, not part of the method ----

def pdelta_probe_read_stream(src: torch.Tensor, sink: torch.Tensor):
    """Enqueue one read-only pass over every byte of ``src`` (16-byte loads)."""
    rc = lib().pdelta_probe_read_stream(_dev(src, "src"), src.numel() * src.element_size(), _dev(sink, "sink"), _stream())
    _check(rc, "pdelta_probe_read_stream")


def pdelta_probe_mfma(waves_per_simd: int, random_operands: bool, iters: int, sink: torch.Tensor):
    """Enqueue the matrix-core loop; returns the flops it performs."""
    rc = lib().pdelta_probe_mfma(waves_per_simd, int(random_operands), iters, _dev(sink, "sink"), _stream())
    _check(rc, "pdelta_probe_mfma")
    return 256 * waves_per_simd * 4 * iters * 4 * 32768.0


PREFILL_PARTS = {"global loads": 1, "conversion and LDS writes": 2, "fragment reads": 4, "MFMAs": 8}
PREFILL_PARTS_BUILT = (0, 1, 2, 3, 4, 8, 12, 13, 14, 15)


def pdelta_probe_prefill_parts(parts: int, X, W_b, B_packed, v_row, out):
    """Enqueue the prefill kernel (bf16, row scales, more than 128 tokens) with only the parts of
    its loop named by the bit mask ``parts``; 15 is the product kernel."""
    M, d_in = X.shape
    d_out = W_b.shape[0]
    rc = lib().pdelta_probe_prefill_parts(parts, _dev(X, "X"), _dev(W_b, "W_b"), _dev(B_packed, "B_packed"),
                                          _dev(v_row, "v_row"), _dev(out, "Y"), M, d_out, d_in,
                                          _DTYPE_CODE[out.dtype], _stream())
    _check(rc, "pdelta_probe_prefill_parts")
    return out
