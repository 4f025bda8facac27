"""Thin Python binding of the C ABI in include/flce.h: argument marshalling only.

Every step of the path (projection, cross entropy, both gradients, the chunk
loop) runs inside libflce.so; PyTorch is used for device memory and streams.
There is no fallback: if the library is missing or a call fails, this raises.
"""
from __future__ import annotations

import ctypes
import os

import torch  # imported before the library so both share one HIP runtime

from . import _build

FLCE_F32, FLCE_BF16 = 0, 1
SKIP_DX, SKIP_DW = 1, 2
_DTYPES = {torch.float32: FLCE_F32, torch.bfloat16: FLCE_BF16}

_lib = None


class FlceError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: status {status} ({status_string(status)})")
        self.status = status


def lib() -> ctypes.CDLL:
    """Loads libflce.so, building it first when there is none or when a kernel source or
    the header is newer than the built library (so an edited kernel is never tested
    against an old binary)."""
    global _lib
    if _lib is None:
        if _build.is_stale():
            _build.build()
        L = ctypes.CDLL(_build.LIB_PATH)
        p, i64, sz, ci, u = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t, ctypes.c_int, ctypes.c_uint
        sigs = {
            "flce_fwd_bwd": ([p, p, p, i64, i64, i64, i64, ci, p, p, p, p], ci),
            "flce_fwd_bwd_ex": ([p, p, p, i64, i64, i64, i64, ci, p, p, p, u, p], ci),
            "flce_fwd_bwd_opt": ([p, p, p, i64, i64, i64, i64, ci, p, p, p, p, p], ci),
            "flce_default_options": ([p], None),
            "flce_workspace_bytes_opt": ([i64, i64, i64, ci, p], sz),
            "flce_multihead_fwd_bwd": ([p, p, p, p, ci, i64, i64, i64, i64, ci, p, p, p, p, u, p], ci),
            "flce_rmsnorm_fwd_bwd": ([p, p, ctypes.c_float, p, p, i64, i64, i64, i64, ci, p, p, p, p, u, p], ci),
            "flce_rmsnorm_workspace_bytes": ([i64, i64, i64, ci], sz),
            "flce_cross_entropy_inplace": ([p, p, i64, i64, i64, i64, ci, p, p], ci),
            "flce_cross_entropy_inplace_noalloc": ([p, p, i64, i64, i64, i64, ci, p, p], ci),
            "flce_workspace_bytes": ([i64, i64, i64, ci], sz),
            "flce_workspace_bytes_max": ([i64, i64, ci], sz),
            "flce_set_workspace": ([p, sz], ci),
            "flce_release_workspace": ([], ci),
            "flce_set_logits_budget_bytes": ([sz], ci),
            "flce_get_logits_budget_bytes": ([], sz),
            "flce_set_row_compaction": ([ci], ci),
            "flce_get_row_compaction": ([], ci),
            "flce_logits_budget_for_workspace": ([i64, i64, i64, ci, sz], sz),
            "flce_chunk_rows": ([i64, i64, i64, ci], i64),
            "flce_num_chunks": ([i64, i64, i64, ci], i64),
            "flce_dx_k_ranges": ([i64, i64, i64, ci], ci),
            "flce_paper_chunk_rows": ([i64, i64, i64], i64),
            "flce_full_logits_bytes": ([i64, i64, ci], sz),
            "flce_mfma_ceiling_launch": ([ci, ci, ci, ctypes.c_float, p, sz, p], ci),
            "flce_timing_enable": ([ci], ci),
            "flce_timing_collect": ([p, p], ci),
            "flce_status_string": ([ci], ctypes.c_char_p),
        }
        for name, (args, res) in sigs.items():
            fn = getattr(L, name)
            fn.argtypes, fn.restype = args, res
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().flce_status_string(int(status)).decode()


def _check(status: int, what: str):
    if status != 0:
        raise FlceError(status, what)


def _dtype_code(t: torch.Tensor) -> int:
    try:
        return _DTYPES[t.dtype]
    except KeyError:
        raise TypeError(f"unsupported dtype {t.dtype}; use float32 or bfloat16") from None


def _dev_ptr(t: torch.Tensor | None, name: str) -> int | None:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous (dense row-major)")
    return t.data_ptr()


def _stream_handle(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def flce_fwd_bwd(X, W, targets, ignore_index=-100, loss=None, dX=None, dW=None, flags=0,
                 stream=None):
    """loss, dX, dW of mean cross_entropy(X @ W.T, targets) on the GPU, chunked.

    X [BT, H], W [V, H] (float32 or bfloat16, same dtype), targets [BT] int64,
    all contiguous CUDA tensors.  Outputs are allocated when not passed.
    Asynchronous on `stream` (default: torch's current stream).
    """
    code = _dtype_code(X)
    if W.dtype != X.dtype:
        raise TypeError("X and W must have the same dtype")
    if X.dim() != 2 or W.dim() != 2 or X.shape[1] != W.shape[1] or targets.shape != (X.shape[0],):
        raise ValueError("expected X [BT, H], W [V, H], targets [BT]")
    if targets.dtype != torch.int64:
        raise TypeError("targets must be int64")
    BT, H = X.shape
    V = W.shape[0]
    if loss is None:
        loss = torch.empty((), dtype=torch.float32, device=X.device)
    if dX is None and not (flags & SKIP_DX):
        dX = torch.empty_like(X)
    if dW is None and not (flags & SKIP_DW):
        dW = torch.empty_like(W)
    for name, t, ref in (("dX", dX, X), ("dW", dW, W)):
        if t is not None and (t.shape != ref.shape or t.dtype != ref.dtype):
            raise ValueError(f"{name} must match its input in shape and dtype")
    with torch.cuda.device(X.device):
        st = lib().flce_fwd_bwd_ex(_dev_ptr(X, "X"), _dev_ptr(W, "W"), _dev_ptr(targets, "targets"),
                                   BT, H, V, int(ignore_index), code, _dev_ptr(loss, "loss"),
                                   _dev_ptr(dX, "dX"), _dev_ptr(dW, "dW"), int(flags),
                                   _stream_handle(stream))
    _check(st, "flce_fwd_bwd")
    return loss, dX, dW


class FlceOptions(ctypes.Structure):
    """flce_options of include/flce.h."""
    _fields_ = [("size", ctypes.c_size_t), ("logits_budget_bytes", ctypes.c_size_t),
                ("row_compaction", ctypes.c_int), ("flags", ctypes.c_uint),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t)]


def flce_options(logits_budget_bytes=None, row_compaction=None, flags=0, workspace=None) -> FlceOptions:
    """The process-wide settings (flce_default_options) with the given fields replaced.
    workspace: a device tensor the call uses as its scratch memory instead of the device's
    shared workspace (kept alive by the returned struct)."""
    o = FlceOptions()
    lib().flce_default_options(ctypes.byref(o))
    if workspace is not None:
        o.workspace = _dev_ptr(workspace, "workspace")
        o.workspace_bytes = workspace.numel() * workspace.element_size()
        o._workspace_tensor = workspace
    if logits_budget_bytes is not None:
        o.logits_budget_bytes = int(logits_budget_bytes)
    if row_compaction is not None:
        o.row_compaction = 1 if row_compaction else 0
    o.flags = int(flags)
    return o


def flce_fwd_bwd_opt(X, W, targets, options: FlceOptions, ignore_index=-100, loss=None, dX=None,
                     dW=None, stream=None):
    """flce_fwd_bwd with its settings passed along (see flce_options)."""
    code = _dtype_code(X)
    if W.dtype != X.dtype or targets.dtype != torch.int64:
        raise TypeError("X and W must have the same dtype, targets must be int64")
    if X.dim() != 2 or W.dim() != 2 or X.shape[1] != W.shape[1] or targets.shape != (X.shape[0],):
        raise ValueError("expected X [BT, H], W [V, H], targets [BT]")
    BT, H = X.shape
    V = W.shape[0]
    if loss is None:
        loss = torch.empty((), dtype=torch.float32, device=X.device)
    if dX is None and not (options.flags & SKIP_DX):
        dX = torch.empty_like(X)
    if dW is None and not (options.flags & SKIP_DW):
        dW = torch.empty_like(W)
    with torch.cuda.device(X.device):
        st = lib().flce_fwd_bwd_opt(_dev_ptr(X, "X"), _dev_ptr(W, "W"), _dev_ptr(targets, "targets"),
                                    BT, H, V, int(ignore_index), code, _dev_ptr(loss, "loss"),
                                    _dev_ptr(dX, "dX"), _dev_ptr(dW, "dW"), ctypes.byref(options),
                                    _stream_handle(stream))
    _check(st, "flce_fwd_bwd_opt")
    return loss, dX, dW


def flce_workspace_bytes_opt(BT, H, V, dtype, options: FlceOptions) -> int:
    return int(lib().flce_workspace_bytes_opt(BT, H, V, _DTYPES.get(dtype, dtype), ctypes.byref(options)))


def flce_multihead_fwd_bwd(X, Ws, targets, weights=None, ignore_index=-100, loss=None,
                           head_losses=None, dX=None, dWs=None, flags=0, stream=None):
    """Several heads on shared hidden states: loss = sum_j weights[j] * CE_j.

    X [BT, H]; Ws, targets: sequences of n_heads tensors W_j [V, H] and int64
    targets_j [BT]; weights: n_heads floats or None (all 1).  Returns
    (loss, head_losses [n_heads], dX, [dW_j]).  Outputs are allocated when not passed.
    """
    code = _dtype_code(X)
    n = len(Ws)
    if n < 1 or len(targets) != n or (weights is not None and len(weights) != n):
        raise ValueError("Ws, targets and weights must have one entry per head")
    if X.dim() != 2:
        raise ValueError("expected X [BT, H]")
    BT, H = X.shape
    V = Ws[0].shape[0]
    for W, t in zip(Ws, targets):
        if W.dtype != X.dtype or t.dtype != torch.int64:
            raise TypeError("every W must have X's dtype and every targets tensor must be int64")
        if W.shape != (V, H) or t.shape != (BT,):
            raise ValueError("expected every W [V, H] and every targets [BT]")
    if loss is None:
        loss = torch.empty((), dtype=torch.float32, device=X.device)
    if head_losses is None:
        head_losses = torch.empty(n, dtype=torch.float32, device=X.device)
    if head_losses.shape != (n,) or head_losses.dtype != torch.float32:
        raise ValueError("head_losses must be n_heads float32 values")
    if dX is None and not (flags & SKIP_DX):
        dX = torch.empty_like(X)
    if dX is not None and (dX.shape != X.shape or dX.dtype != X.dtype):
        raise ValueError("dX must match X in shape and dtype")
    if dWs is None and not (flags & SKIP_DW):
        dWs = [torch.empty_like(W) for W in Ws]
    if dWs is not None:
        if len(dWs) != n or any(d.shape != (V, H) or d.dtype != X.dtype for d in dWs):
            raise ValueError("dWs must hold one [V, H] tensor of X's dtype per head")
    ptr_array = ctypes.c_void_p * n
    w_arr = ptr_array(*[_dev_ptr(W, "W") for W in Ws])
    t_arr = ptr_array(*[_dev_ptr(t, "targets") for t in targets])
    dw_arr = ptr_array(*[_dev_ptr(d, "dW") for d in dWs]) if dWs is not None else None
    wt_arr = (ctypes.c_float * n)(*[float(w) for w in weights]) if weights is not None else None
    with torch.cuda.device(X.device):
        st = lib().flce_multihead_fwd_bwd(_dev_ptr(X, "X"), w_arr, t_arr, wt_arr, n, BT, H, V,
                                          int(ignore_index), code, _dev_ptr(loss, "loss"),
                                          _dev_ptr(head_losses, "head_losses"), _dev_ptr(dX, "dX"),
                                          dw_arr, int(flags), _stream_handle(stream))
    _check(st, "flce_multihead_fwd_bwd")
    return loss, head_losses, dX, dWs


def flce_rmsnorm_fwd_bwd(h, gamma, eps, W, targets, ignore_index=-100, loss=None, dh=None,
                         dgamma=None, dW=None, flags=0, stream=None):
    """loss, dh, dgamma, dW of mean cross_entropy(rmsnorm(h; gamma, eps) @ W.T, targets)."""
    code = _dtype_code(h)
    if W.dtype != h.dtype or gamma.dtype != h.dtype:
        raise TypeError("h, gamma and W must have the same dtype")
    if h.dim() != 2 or W.dim() != 2 or h.shape[1] != W.shape[1] or gamma.shape != (h.shape[1],) \
            or targets.shape != (h.shape[0],):
        raise ValueError("expected h [BT, H], gamma [H], W [V, H], targets [BT]")
    if targets.dtype != torch.int64:
        raise TypeError("targets must be int64")
    BT, H = h.shape
    V = W.shape[0]
    if loss is None:
        loss = torch.empty((), dtype=torch.float32, device=h.device)
    if not (flags & SKIP_DX):
        dh = torch.empty_like(h) if dh is None else dh
        dgamma = torch.empty_like(gamma) if dgamma is None else dgamma
    if dW is None and not (flags & SKIP_DW):
        dW = torch.empty_like(W)
    for name, t, ref in (("dh", dh, h), ("dgamma", dgamma, gamma), ("dW", dW, W)):
        if t is not None and (t.shape != ref.shape or t.dtype != ref.dtype):
            raise ValueError(f"{name} must match its input in shape and dtype")
    with torch.cuda.device(h.device):
        st = lib().flce_rmsnorm_fwd_bwd(_dev_ptr(h, "h"), _dev_ptr(gamma, "gamma"), float(eps),
                                        _dev_ptr(W, "W"), _dev_ptr(targets, "targets"), BT, H, V,
                                        int(ignore_index), code, _dev_ptr(loss, "loss"),
                                        _dev_ptr(dh, "dh"), _dev_ptr(dgamma, "dgamma"),
                                        _dev_ptr(dW, "dW"), int(flags), _stream_handle(stream))
    _check(st, "flce_rmsnorm_fwd_bwd")
    return loss, dh, dgamma, dW


def flce_rmsnorm_workspace_bytes(BT, H, V, dtype) -> int:
    return int(lib().flce_rmsnorm_workspace_bytes(BT, H, V, _DTYPES.get(dtype, dtype)))


CE_NOALLOC_MAX_ROWS = 65536


def flce_cross_entropy_inplace(Z, targets, ignore_index=-100, loss=None, stream=None, noalloc=False):
    """Replaces logits Z [BT, V] (row stride Z.stride(0)) by dL/dZ; returns the mean loss.
    noalloc=True calls flce_cross_entropy_inplace_noalloc (pass `loss`: this wrapper
    would otherwise allocate it)."""
    code = _dtype_code(Z)
    if Z.dim() != 2 or Z.stride(1) != 1 or targets.shape != (Z.shape[0],):
        raise ValueError("expected Z [BT, V] with unit column stride, targets [BT]")
    if targets.dtype != torch.int64 or not Z.is_cuda:
        raise TypeError("targets must be int64 and Z on the GPU")
    BT, V = Z.shape
    if loss is None:
        loss = torch.empty((), dtype=torch.float32, device=Z.device)
    with torch.cuda.device(Z.device):
        fn = lib().flce_cross_entropy_inplace_noalloc if noalloc else lib().flce_cross_entropy_inplace
        st = fn(Z.data_ptr(), _dev_ptr(targets, "targets"), BT, V,
                Z.stride(0) if BT > 1 else max(V, Z.stride(0)), int(ignore_index), code,
                _dev_ptr(loss, "loss"), _stream_handle(stream))
    _check(st, "flce_cross_entropy_inplace_noalloc" if noalloc else "flce_cross_entropy_inplace")
    return loss


def flce_cross_entropy_inplace_noalloc(Z, targets, ignore_index=-100, loss=None, stream=None):
    return flce_cross_entropy_inplace(Z, targets, ignore_index, loss, stream, noalloc=True)


def flce_workspace_bytes(BT, H, V, dtype) -> int:
    return int(lib().flce_workspace_bytes(BT, H, V, _DTYPES.get(dtype, dtype)))


def flce_workspace_bytes_max(H, V, dtype) -> int:
    return int(lib().flce_workspace_bytes_max(H, V, _DTYPES.get(dtype, dtype)))


def flce_set_workspace(ws: torch.Tensor | None):
    if ws is None:
        _check(lib().flce_set_workspace(None, 0), "flce_set_workspace")
    else:
        with torch.cuda.device(ws.device):
            _check(lib().flce_set_workspace(ws.data_ptr(), ws.numel() * ws.element_size()),
                   "flce_set_workspace")


def flce_release_workspace():
    _check(lib().flce_release_workspace(), "flce_release_workspace")


def flce_set_logits_budget_bytes(n: int):
    _check(lib().flce_set_logits_budget_bytes(int(n)), "flce_set_logits_budget_bytes")


def flce_get_logits_budget_bytes() -> int:
    return int(lib().flce_get_logits_budget_bytes())


def flce_set_row_compaction(on: bool):
    _check(lib().flce_set_row_compaction(1 if on else 0), "flce_set_row_compaction")


def flce_get_row_compaction() -> bool:
    return bool(lib().flce_get_row_compaction())


def flce_logits_budget_for_workspace(BT, H, V, dtype, max_workspace_bytes) -> int:
    return int(lib().flce_logits_budget_for_workspace(BT, H, V, _DTYPES.get(dtype, dtype), int(max_workspace_bytes)))


def flce_chunk_rows(BT, H, V, dtype) -> int:
    return int(lib().flce_chunk_rows(BT, H, V, _DTYPES.get(dtype, dtype)))


def flce_num_chunks(BT, H, V, dtype) -> int:
    return int(lib().flce_num_chunks(BT, H, V, _DTYPES.get(dtype, dtype)))


def flce_dx_k_ranges(BT, H, V, dtype) -> int:
    return int(lib().flce_dx_k_ranges(BT, H, V, _DTYPES.get(dtype, dtype)))


def flce_paper_chunk_rows(BT, H, V) -> int:
    return int(lib().flce_paper_chunk_rows(BT, H, V))


def flce_full_logits_bytes(BT, V, dtype) -> int:
    return int(lib().flce_full_logits_bytes(BT, V, _DTYPES.get(dtype, dtype)))


KERNEL_KINDS = ("logits_gemm", "ce_rows", "dx_gemm", "dw_gemm", "other")


def flce_mfma_ceiling_launch(pattern: int, workgroups: int, iters: int, std_b: float, out, stream=None):
    """Enqueues the MFMA-only loop (see include/flce.h); `out` is a float32 CUDA tensor
    of at least workgroups * 256 elements.  Returns the flops of the launch."""
    if out.dtype != torch.float32 or not out.is_cuda or not out.is_contiguous():
        raise ValueError("out must be a contiguous float32 CUDA tensor")
    _check(lib().flce_mfma_ceiling_launch(int(pattern), int(workgroups), int(iters), float(std_b),
                                          out.data_ptr(), out.numel(), _stream_handle(stream)),
           "flce_mfma_ceiling_launch")
    return workgroups * 4 * iters * 16 * 32768.0


def flce_timing_enable(on: bool):
    _check(lib().flce_timing_enable(1 if on else 0), "flce_timing_enable")


def flce_timing_collect() -> dict:
    """{kind: (total_ms, launches)} of the launches recorded since the last collect."""
    n = len(KERNEL_KINDS)
    ms = (ctypes.c_double * n)()
    cnt = (ctypes.c_int64 * n)()
    _check(lib().flce_timing_collect(ctypes.addressof(ms), ctypes.addressof(cnt)), "flce_timing_collect")
    return {k: (float(ms[i]), int(cnt[i])) for i, k in enumerate(KERNEL_KINDS)}
