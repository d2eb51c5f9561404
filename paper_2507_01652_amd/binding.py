"""Thin ctypes binding of liblasad's C ABI (see include/lasad.h).

Argument marshalling only: every step of the path runs in the HIP kernels.
PyTorch supplies device memory (``tensor.data_ptr()``) and the stream; there is
no CPU fallback -- a missing library is an error.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblasad.so")

F32, BF16 = 0, 1
RESET_LAST_COL, RESET_FIRST_COL, RESET_NONE = 0, 1, 2
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = 0, 1, 2, 3, 4

EXPORTS = (
    "lasad_decay_factors", "lasad_forward_workspace_bytes", "lasad_forward_chunked",
    "lasad_forward_static_scratch_bytes", "lasad_forward_chunked_static",
    "lasad_decode_step", "lasad_forward_gated", "lasad_decode_step_gated",
    "lasad_forward_layer", "lasad_decode_step_layer",
    "lasad_decode_step_rows", "lasad_decode_step_cached", "lasad_decode_step_gated_cached",
    "lasad_backward_workspace_bytes", "lasad_backward_chunked",
    "lasad_backward_carried_workspace_bytes", "lasad_backward_chunked_carried",
    "lasad_backward_gated_workspace_bytes", "lasad_backward_gated",
    "lasad_backward_gated_carried_workspace_bytes", "lasad_backward_gated_carried",
    "lasad_backward_layer_workspace_bytes", "lasad_backward_layer", "lasad_backward_layer_norm",
    "lasad_last_error", "lasad_version",
)


class LasadError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"liblasad status {status}: {message}")
        self.status = status


class Layout(ctypes.Structure):
    _fields_ = [("stride_b", ctypes.c_int64), ("stride_n", ctypes.c_int64), ("stride_h", ctypes.c_int64)]


_lib = None


def load() -> ctypes.CDLL:
    """Open liblasad.so (built in-tree by ``paper_2507_01652_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2507_01652_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    lp = ctypes.POINTER(Layout)
    lib.lasad_decay_factors.argtypes = [vp, ci, ci, ci, ci, ci, ci, vp, vp, vp]
    lib.lasad_decay_factors.restype = ci
    lib.lasad_forward_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
    lib.lasad_forward_workspace_bytes.restype = ctypes.c_size_t
    lib.lasad_forward_chunked.argtypes = [vp, vp, vp, vp, lp, lp, ci, ci, ci, ci, ci, ci, ci, ci, ci,
                                          vp, ci, cf, vp, vp, vp, ctypes.c_size_t, vp]
    lib.lasad_forward_chunked.restype = ci
    lib.lasad_forward_static_scratch_bytes.argtypes = []
    lib.lasad_forward_static_scratch_bytes.restype = ctypes.c_size_t
    lib.lasad_forward_chunked_static.argtypes = [vp, vp, vp, vp, lp, lp, ci, ci, ci, ci, ci, ci, ci, ci, ci,
                                                 vp, ci, cf, vp, vp, vp]
    lib.lasad_forward_chunked_static.restype = ci
    lib.lasad_decode_step.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, vp, ci, cf, vp, vp]
    lib.lasad_decode_step.restype = ci
    lib.lasad_forward_gated.argtypes = [vp, vp, vp, vp, vp, lp, lp, ci, ci, ci, ci, ci, ci, ci, ci, ci,
                                        ci, cf, vp, vp, vp]
    lib.lasad_forward_gated.restype = ci
    lib.lasad_decode_step_gated.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, ci, cf, vp, vp]
    lib.lasad_decode_step_gated.restype = ci
    lib.lasad_forward_layer.argtypes = [vp, vp, vp, vp, lp, lp, ci, ci, ci, ci, ci, ci, ci, ci, ci, ci, cf, vp, cf, vp, vp, vp]
    lib.lasad_forward_layer.restype = ci
    lib.lasad_decode_step_layer.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, ci, cf, vp, cf, vp, vp]
    lib.lasad_decode_step_layer.restype = ci
    lib.lasad_decode_step_rows.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp, vp, ci, cf, vp, vp]
    lib.lasad_decode_step_rows.restype = ci
    lib.lasad_decode_step_cached.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, ci, vp, ci, cf, vp]
    lib.lasad_decode_step_cached.restype = ci
    lib.lasad_decode_step_gated_cached.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, ci, ci, cf, vp]
    lib.lasad_decode_step_gated_cached.restype = ci
    lib.lasad_backward_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
    lib.lasad_backward_workspace_bytes.restype = ctypes.c_size_t
    lib.lasad_backward_chunked.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, lp, lp, ci, ci, ci, ci, ci, ci, ci, ci, ci,
                                           vp, ci, cf, vp, ctypes.c_size_t, vp]
    lib.lasad_backward_chunked.restype = ci
    lib.lasad_backward_carried_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
    lib.lasad_backward_carried_workspace_bytes.restype = ctypes.c_size_t
    lib.lasad_backward_chunked_carried.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, lp, lp, ci, ci, ci, ci, ci, ci, ci,
                                                   ci, ci, vp, ci, cf, vp, ctypes.c_size_t, vp]
    lib.lasad_backward_chunked_carried.restype = ci
    lib.lasad_backward_gated_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.lasad_backward_gated_workspace_bytes.restype = ctypes.c_size_t
    lib.lasad_backward_gated.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, lp, lp, ci, ci, ci, ci, ci, ci, ci, ci, ci, ci,
                                         ctypes.c_float, vp, ctypes.c_size_t, vp]
    lib.lasad_backward_gated.restype = ci
    lib.lasad_backward_gated_carried_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.lasad_backward_gated_carried_workspace_bytes.restype = ctypes.c_size_t
    lib.lasad_backward_gated_carried.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, lp, lp, ci, ci, ci, ci, ci, ci,
                                                 ci, ci, ci, ci, ctypes.c_float, vp, ctypes.c_size_t, vp]
    lib.lasad_backward_gated_carried.restype = ci
    lib.lasad_backward_layer_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, lp]
    lib.lasad_backward_layer_workspace_bytes.restype = ctypes.c_size_t
    lib.lasad_backward_layer.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, lp, lp, lp, ci, ci, ci, ci, ci, ci, ci, ci, ci, ci,
                                         ctypes.c_float, vp, ctypes.c_float, vp, ctypes.c_size_t, vp]
    lib.lasad_backward_layer.restype = ci
    lib.lasad_backward_layer_norm.argtypes = [vp, vp, vp, vp, vp, vp, lp, lp, lp, ci, ci, ci, ci, ci, ci, ci, ci, ci, ci,
                                              ctypes.c_float, vp, ctypes.c_float, vp, ctypes.c_size_t, vp]
    lib.lasad_backward_layer_norm.restype = ci
    lib.lasad_last_error.argtypes = []
    lib.lasad_last_error.restype = ctypes.c_char_p
    lib.lasad_version.argtypes = []
    lib.lasad_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _check(status: int):
    if status != OK:
        raise LasadError(status, load().lasad_last_error().decode())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _scratch(nbytes: int, device, stream) -> torch.Tensor:
    """A workspace from torch's caching allocator that stays reserved until the work queued on `stream`
    (None: the current stream) has run: a block freed on another stream could be handed out again while
    the kernels still use it."""
    t = torch.empty((nbytes,), dtype=torch.uint8, device=device)
    if stream is not None and stream != torch.cuda.current_stream():
        t.record_stream(stream)
    return t


def _layout(t: torch.Tensor) -> Layout:
    """Strides of a logical [B, n, Hh, d] tensor (any permutation with unit d stride)."""
    if t.dim() == 4 and t.numel() == 0:          # no element is addressed: dense strides stand in for whatever torch reports
        return Layout(t.shape[1] * t.shape[2] * t.shape[3], t.shape[2] * t.shape[3], t.shape[3])
    if t.dim() != 4 or (t.shape[3] > 1 and t.stride(3) != 1):
        raise ValueError("expected a [B, n_tokens, Hh, d] tensor with unit stride along d")
    return Layout(t.stride(0), t.stride(1), t.stride(2))


def version() -> str:
    return load().lasad_version().decode()


def lasad_decay_factors(gamma: torch.Tensor, grid_h: int, grid_w: int, start_pos: int, n_tokens: int,
                        boundary_mode: int = RESET_LAST_COL, want_lambda: bool = True,
                        want_cum_exp: bool = True, stream=None):
    """Decay table: returns (lambda[Hh, n] fp32 or None, cum_exp[n+1] int32 or None) on gamma's device."""
    assert gamma.dtype == torch.float32 and gamma.is_contiguous() and gamma.dim() == 1
    Hh = gamma.shape[0]
    lam = torch.empty((Hh, max(n_tokens, 0)), dtype=torch.float32, device=gamma.device) if want_lambda else None
    cum = torch.empty((max(n_tokens, 0) + 1,), dtype=torch.int32, device=gamma.device) if want_cum_exp else None
    _check(load().lasad_decay_factors(_ptr(gamma), Hh, grid_h, grid_w, start_pos, n_tokens, boundary_mode,
                                      _ptr(lam), _ptr(cum), _stream(stream)))
    return lam, cum


def lasad_forward_workspace_bytes(B: int, n_heads: int, n_tokens: int, d: int, io_dtype: int) -> int:
    return int(load().lasad_forward_workspace_bytes(B, n_heads, n_tokens, d, io_dtype))


def lasad_forward_chunked(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, gamma: torch.Tensor,
                          grid_h: int, grid_w: int, start_pos: int = 0,
                          boundary_mode: int = RESET_LAST_COL, q_scale: float = 1.0,
                          state_in: torch.Tensor | None = None, state_out: torch.Tensor | None = None,
                          out: torch.Tensor | None = None, out_dtype: torch.dtype | None = None,
                          workspace: torch.Tensor | None = None, use_workspace: bool = True,
                          stream=None) -> torch.Tensor:
    """Chunked forward over positions start_pos+1 .. start_pos+n.  q, k, v: logical [B, n, Hh, d]
    views sharing one set of strides; returns o (allocated like q unless `out` is given).
    `workspace`: a device buffer of lasad_forward_workspace_bytes(...) bytes; when None one is
    taken from torch's caching allocator (use_workspace=False passes NULL: single-pass kernel)."""
    B, n, Hh, d = q.shape
    if k.shape != q.shape or v.shape != q.shape or k.stride() != q.stride() or v.stride() != q.stride():
        raise ValueError("q, k, v must share shape and strides")
    if k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v must share a dtype")
    if out is None:
        out = torch.empty_like(q, dtype=out_dtype or q.dtype)
    elif out.shape != q.shape:
        raise ValueError("out has the wrong shape")
    for s in (state_in, state_out):
        if s is not None and (s.dtype != torch.float32 or not s.is_contiguous() or tuple(s.shape) != (B, Hh, d, d)):
            raise ValueError("states must be contiguous fp32 [B, Hh, d, d]")
    assert gamma.dtype == torch.float32 and gamma.is_contiguous() and tuple(gamma.shape) == (Hh,)
    lq, lo = _layout(q), _layout(out)
    if workspace is None and use_workspace and n > 0:
        need = lasad_forward_workspace_bytes(B, Hh, n, d, _dtype_code(q))
        if need:
            workspace = _scratch(need, q.device, stream)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().lasad_forward_chunked(
        _ptr(q), _ptr(k), _ptr(v), _ptr(out), ctypes.byref(lq), ctypes.byref(lo),
        _dtype_code(q), _dtype_code(out), B, Hh, d, grid_h, grid_w, start_pos, n,
        _ptr(gamma), boundary_mode, q_scale, _ptr(state_in), _ptr(state_out),
        _ptr(workspace), ws_bytes, _stream(stream)))
    return out


def lasad_forward_static_scratch_bytes() -> int:
    return int(load().lasad_forward_static_scratch_bytes())


def lasad_forward_chunked_static(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, gamma: torch.Tensor,
                                 grid_h: int, grid_w: int, out: torch.Tensor, start_pos: int = 0,
                                 boundary_mode: int = RESET_LAST_COL, q_scale: float = 1.0,
                                 state_in: torch.Tensor | None = None, state_out: torch.Tensor | None = None,
                                 stream=None) -> torch.Tensor:
    """lasad_forward_chunked over the library's built-in scratch array: nothing is allocated, so the
    caller passes every buffer, `out` included."""
    B, n, Hh, d = q.shape
    if k.shape != q.shape or v.shape != q.shape or k.stride() != q.stride() or v.stride() != q.stride():
        raise ValueError("q, k, v must share shape and strides")
    if k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v must share a dtype")
    if out.shape != q.shape:
        raise ValueError("out has the wrong shape")
    for s in (state_in, state_out):
        if s is not None and (s.dtype != torch.float32 or not s.is_contiguous() or tuple(s.shape) != (B, Hh, d, d)):
            raise ValueError("states must be contiguous fp32 [B, Hh, d, d]")
    assert gamma.dtype == torch.float32 and gamma.is_contiguous() and tuple(gamma.shape) == (Hh,)
    lq, lo = _layout(q), _layout(out)
    _check(load().lasad_forward_chunked_static(
        _ptr(q), _ptr(k), _ptr(v), _ptr(out), ctypes.byref(lq), ctypes.byref(lo),
        _dtype_code(q), _dtype_code(out), B, Hh, d, grid_h, grid_w, start_pos, n,
        _ptr(gamma), boundary_mode, q_scale, _ptr(state_in), _ptr(state_out), _stream(stream)))
    return out


def lasad_decode_step(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, gamma: torch.Tensor,
                      state: torch.Tensor, grid_h: int, grid_w: int, pos: int,
                      boundary_mode: int = RESET_LAST_COL, q_scale: float = 1.0,
                      out: torch.Tensor | None = None, out_dtype: torch.dtype | None = None,
                      stream=None) -> torch.Tensor:
    """One decode step at 0-indexed raster position `pos`.  q, k, v: contiguous [B, Hh, d];
    state: contiguous fp32 [B, Hh, d, d], updated in place.  Returns o [B, Hh, d]."""
    B, Hh, d = q.shape
    for t in (q, k, v):
        if t.shape != q.shape or t.dtype != q.dtype or not t.is_contiguous():
            raise ValueError("q, k, v must be contiguous [B, Hh, d] of one dtype")
    if state.dtype != torch.float32 or not state.is_contiguous() or tuple(state.shape) != (B, Hh, d, d):
        raise ValueError("state must be contiguous fp32 [B, Hh, d, d]")
    if out is None:
        out = torch.empty_like(q, dtype=out_dtype or q.dtype)
    elif out.shape != q.shape or not out.is_contiguous():
        raise ValueError("out must be contiguous [B, Hh, d]")
    assert gamma.dtype == torch.float32 and gamma.is_contiguous() and tuple(gamma.shape) == (Hh,)
    _check(load().lasad_decode_step(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _dtype_code(q), _dtype_code(out),
                                    B, Hh, d, grid_h, grid_w, pos, _ptr(gamma), boundary_mode, q_scale,
                                    _ptr(state), _stream(stream)))
    return out


def lasad_decode_step_cached(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, gamma: torch.Tensor,
                             k_cache: torch.Tensor, v_cache: torch.Tensor, grid_h: int, grid_w: int, pos: int,
                             boundary_mode: int = RESET_LAST_COL, q_scale: float = 1.0,
                             out: torch.Tensor | None = None, out_dtype: torch.dtype | None = None,
                             stream=None) -> torch.Tensor:
    """The decode step at position `pos` from key / value caches (contiguous [B, Hh, T, d] of q's dtype,
    rows 0..pos-1 filled by the earlier steps; this step's k, v are appended as row pos).  Returns o."""
    B, Hh, d = q.shape
    for t in (q, k, v):
        if t.shape != q.shape or t.dtype != q.dtype or not t.is_contiguous():
            raise ValueError("q, k, v must be contiguous [B, Hh, d] of one dtype")
    for t in (k_cache, v_cache):
        if t.dim() != 4 or tuple(t.shape[:2]) != (B, Hh) or t.shape[3] != d or t.dtype != q.dtype or not t.is_contiguous():
            raise ValueError("caches must be contiguous [B, Hh, T, d] of q's dtype")
    if k_cache.shape != v_cache.shape:
        raise ValueError("k_cache and v_cache differ in shape")
    if out is None:
        out = torch.empty_like(q, dtype=out_dtype or q.dtype)
    elif out.shape != q.shape or not out.is_contiguous():
        raise ValueError("out must be contiguous [B, Hh, d]")
    assert gamma.dtype == torch.float32 and gamma.is_contiguous() and tuple(gamma.shape) == (Hh,)
    _check(load().lasad_decode_step_cached(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(k_cache), _ptr(v_cache),
                                           k_cache.shape[2], _dtype_code(q), _dtype_code(out), B, Hh, d,
                                           grid_h, grid_w, pos, _ptr(gamma), boundary_mode, q_scale, _stream(stream)))
    return out


def lasad_decode_step_gated_cached(q: torch.Tensor, lam: torch.Tensor, v: torch.Tensor,
                                   lam_cache: torch.Tensor, v_cache: torch.Tensor, grid_h: int, grid_w: int, pos: int,
                                   k: torch.Tensor | None = None, k_cache: torch.Tensor | None = None,
                                   boundary_mode: int = RESET_LAST_COL, q_scale: float = 1.0,
                                   out: torch.Tensor | None = None, out_dtype: torch.dtype | None = None,
                                   stream=None) -> torch.Tensor:
    """The vector-decay decode step at position `pos` from caches of the gate rows and of v (and of k with an own
    key; contiguous [B, Hh, T, d] of q's dtype, rows 0..pos-1 filled by the earlier steps; this step's rows are
    appended as row pos).  Returns o."""
    B, Hh, d = q.shape
    if (k is None) != (k_cache is None):
        raise ValueError("k and k_cache go together")
    for t in (q, lam, v) + (() if k is None else (k,)):
        if t.shape != q.shape or t.dtype != q.dtype or not t.is_contiguous():
            raise ValueError("q, lam, k, v must be contiguous [B, Hh, d] of one dtype")
    for t in (lam_cache, v_cache) + (() if k_cache is None else (k_cache,)):
        if t.dim() != 4 or tuple(t.shape[:2]) != (B, Hh) or t.shape[3] != d or t.dtype != q.dtype or not t.is_contiguous():
            raise ValueError("caches must be contiguous [B, Hh, T, d] of q's dtype")
        if t.shape != lam_cache.shape:
            raise ValueError("the caches differ in shape")
    if out is None:
        out = torch.empty_like(q, dtype=out_dtype or q.dtype)
    elif out.shape != q.shape or not out.is_contiguous():
        raise ValueError("out must be contiguous [B, Hh, d]")
    _check(load().lasad_decode_step_gated_cached(_ptr(q), _ptr(lam), _ptr(k), _ptr(v), _ptr(out),
                                                 _ptr(lam_cache), _ptr(k_cache), _ptr(v_cache), lam_cache.shape[2],
                                                 _dtype_code(q), _dtype_code(out), B, Hh, d,
                                                 grid_h, grid_w, pos, boundary_mode, q_scale, _stream(stream)))
    return out


def lasad_forward_gated(q: torch.Tensor, lam: torch.Tensor, v: torch.Tensor, grid_h: int, grid_w: int,
                        k: torch.Tensor | None = None, start_pos: int = 0,
                        boundary_mode: int = RESET_LAST_COL, q_scale: float = 1.0,
                        state_in: torch.Tensor | None = None, state_out: torch.Tensor | None = None,
                        out: torch.Tensor | None = None, out_dtype: torch.dtype | None = None,
                        stream=None) -> torch.Tensor:
    """Vector-decay forward (Section 3.4 as written).  q, lam, v (and k, or None for k = 1 - lam):
    logical [B, n, Hh, d] views sharing one set of strides; returns o."""
    B, n, Hh, d = q.shape
    for t in (lam, v) + (() if k is None else (k,)):
        if t.shape != q.shape or t.stride() != q.stride() or t.dtype != q.dtype:
            raise ValueError("q, lam, k, v must share shape, strides and dtype")
    if out is None:
        out = torch.empty_like(q, dtype=out_dtype or q.dtype)
    elif out.shape != q.shape:
        raise ValueError("out has the wrong shape")
    for s in (state_in, state_out):
        if s is not None and (s.dtype != torch.float32 or not s.is_contiguous() or tuple(s.shape) != (B, Hh, d, d)):
            raise ValueError("states must be contiguous fp32 [B, Hh, d, d]")
    lq, lo = _layout(q), _layout(out)
    _check(load().lasad_forward_gated(
        _ptr(q), _ptr(lam), _ptr(k), _ptr(v), _ptr(out), ctypes.byref(lq), ctypes.byref(lo),
        _dtype_code(q), _dtype_code(out), B, Hh, d, grid_h, grid_w, start_pos, n,
        boundary_mode, q_scale, _ptr(state_in), _ptr(state_out), _stream(stream)))
    return out


def lasad_decode_step_gated(q: torch.Tensor, lam: torch.Tensor, v: torch.Tensor, state: torch.Tensor,
                            grid_h: int, grid_w: int, pos: int, k: torch.Tensor | None = None,
                            boundary_mode: int = RESET_LAST_COL, q_scale: float = 1.0,
                            out: torch.Tensor | None = None, out_dtype: torch.dtype | None = None,
                            stream=None) -> torch.Tensor:
    """One vector-decay decode step.  q, lam, v (k): contiguous [B, Hh, d]; state fp32 [B, Hh, d, d] in place."""
    B, Hh, d = q.shape
    for t in (q, lam, v) + (() if k is None else (k,)):
        if t.shape != q.shape or t.dtype != q.dtype or not t.is_contiguous():
            raise ValueError("q, lam, k, v must be contiguous [B, Hh, d] of one dtype")
    if state.dtype != torch.float32 or not state.is_contiguous() or tuple(state.shape) != (B, Hh, d, d):
        raise ValueError("state must be contiguous fp32 [B, Hh, d, d]")
    if out is None:
        out = torch.empty_like(q, dtype=out_dtype or q.dtype)
    elif out.shape != q.shape or not out.is_contiguous():
        raise ValueError("out must be contiguous [B, Hh, d]")
    _check(load().lasad_decode_step_gated(_ptr(q), _ptr(lam), _ptr(k), _ptr(v), _ptr(out),
                                          _dtype_code(q), _dtype_code(out), B, Hh, d, grid_h, grid_w, pos,
                                          boundary_mode, q_scale, _ptr(state), _stream(stream)))
    return out


def lasad_forward_layer(q_pre: torch.Tensor, z: torch.Tensor, v: torch.Tensor, grid_h: int, grid_w: int,
                        norm_weight: torch.Tensor | None = None, norm_eps: float = 1e-6,
                        start_pos: int = 0, boundary_mode: int = RESET_LAST_COL, q_scale: float = 1.0,
                        state_in: torch.Tensor | None = None, state_out: torch.Tensor | None = None,
                        out: torch.Tensor | None = None, out_dtype: torch.dtype | None = None,
                        stream=None) -> torch.Tensor:
    """Algorithm 1 between its Linear maps: SiLU(q_pre), sigmoid(z), k = 1 - lambda, recurrence, RMS norm.
    q_pre, z, v: logical [B, n, Hh, 64] views sharing strides; norm_eps < 0 switches the norm off."""
    B, n, Hh, d = q_pre.shape
    for t in (z, v):
        if t.shape != q_pre.shape or t.stride() != q_pre.stride() or t.dtype != q_pre.dtype:
            raise ValueError("q_pre, z, v must share shape, strides and dtype")
    if norm_weight is not None and (norm_weight.dtype != torch.float32 or not norm_weight.is_contiguous()
                                    or norm_weight.numel() != Hh * d):
        raise ValueError("norm_weight must be contiguous fp32 [Hh, d]")
    if out is None:
        out = torch.empty_like(q_pre, dtype=out_dtype or q_pre.dtype)
    for s in (state_in, state_out):
        if s is not None and (s.dtype != torch.float32 or not s.is_contiguous() or tuple(s.shape) != (B, Hh, d, d)):
            raise ValueError("states must be contiguous fp32 [B, Hh, d, d]")
    lq, lo = _layout(q_pre), _layout(out)
    _check(load().lasad_forward_layer(
        _ptr(q_pre), _ptr(z), _ptr(v), _ptr(out), ctypes.byref(lq), ctypes.byref(lo),
        _dtype_code(q_pre), _dtype_code(out), B, Hh, d, grid_h, grid_w, start_pos, n,
        boundary_mode, q_scale, _ptr(norm_weight), norm_eps, _ptr(state_in), _ptr(state_out), _stream(stream)))
    return out


def lasad_decode_step_layer(q_pre: torch.Tensor, z: torch.Tensor, v: torch.Tensor, state: torch.Tensor,
                            grid_h: int, grid_w: int, pos: int, norm_weight: torch.Tensor | None = None,
                            norm_eps: float = 1e-6, boundary_mode: int = RESET_LAST_COL, q_scale: float = 1.0,
                            out: torch.Tensor | None = None, out_dtype: torch.dtype | None = None,
                            stream=None) -> torch.Tensor:
    """One decode step of the fused layer.  q_pre, z, v: contiguous [B, Hh, d]; state fp32 in place."""
    B, Hh, d = q_pre.shape
    for t in (q_pre, z, v):
        if t.shape != q_pre.shape or t.dtype != q_pre.dtype or not t.is_contiguous():
            raise ValueError("q_pre, z, v must be contiguous [B, Hh, d] of one dtype")
    if state.dtype != torch.float32 or not state.is_contiguous() or tuple(state.shape) != (B, Hh, d, d):
        raise ValueError("state must be contiguous fp32 [B, Hh, d, d]")
    if out is None:
        out = torch.empty_like(q_pre, dtype=out_dtype or q_pre.dtype)
    _check(load().lasad_decode_step_layer(_ptr(q_pre), _ptr(z), _ptr(v), _ptr(out), _dtype_code(q_pre), _dtype_code(out),
                                          B, Hh, d, grid_h, grid_w, pos, boundary_mode, q_scale,
                                          _ptr(norm_weight), norm_eps, _ptr(state), _stream(stream)))
    return out


def lasad_decode_step_rows(q: torch.Tensor, v: torch.Tensor, state: torch.Tensor, pos_rows: torch.Tensor,
                           grid_h: int, grid_w: int, k: torch.Tensor | None = None,
                           lam: torch.Tensor | None = None, gamma: torch.Tensor | None = None,
                           boundary_mode: int = RESET_LAST_COL, q_scale: float = 1.0,
                           out: torch.Tensor | None = None, out_dtype: torch.dtype | None = None,
                           stream=None) -> torch.Tensor:
    """One decode step with a raster position per batch row (pos_rows: int32 [B] on the device; entries
    outside the grid mark inactive rows).  Scalar decay: give gamma and k; vector decay: give lam (k optional)."""
    B, Hh, d = q.shape
    for t in (q, v) + tuple(x for x in (k, lam) if x is not None):
        if t.shape != q.shape or t.dtype != q.dtype or not t.is_contiguous():
            raise ValueError("q, lam, k, v must be contiguous [B, Hh, d] of one dtype")
    if state.dtype != torch.float32 or not state.is_contiguous() or tuple(state.shape) != (B, Hh, d, d):
        raise ValueError("state must be contiguous fp32 [B, Hh, d, d]")
    if pos_rows.dtype != torch.int32 or pos_rows.numel() != B or not pos_rows.is_contiguous():
        raise ValueError("pos_rows must be contiguous int32 [B]")
    if out is None:
        out = torch.empty_like(q, dtype=out_dtype or q.dtype)
    elif out.shape != q.shape or not out.is_contiguous():
        raise ValueError("out must be contiguous [B, Hh, d]")
    _check(load().lasad_decode_step_rows(_ptr(q), _ptr(lam), _ptr(k), _ptr(v), _ptr(out),
                                         _dtype_code(q), _dtype_code(out), B, Hh, d, grid_h, grid_w,
                                         _ptr(pos_rows), _ptr(gamma), boundary_mode, q_scale, _ptr(state),
                                         _stream(stream)))
    return out


def lasad_backward_workspace_bytes(B: int, n_heads: int, n_tokens: int, d: int, io_dtype: int) -> int:
    return int(load().lasad_backward_workspace_bytes(B, n_heads, n_tokens, d, io_dtype))


def lasad_backward_chunked(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, d_o: torch.Tensor,
                           gamma: torch.Tensor, grid_h: int, grid_w: int, start_pos: int = 0,
                           boundary_mode: int = RESET_LAST_COL, q_scale: float = 1.0,
                           grads: tuple | None = None, grad_dtype: torch.dtype | None = None,
                           dgamma: torch.Tensor | None = None, workspace: torch.Tensor | None = None,
                           stream=None):
    """Gradients of lasad_forward_chunked (zero initial state).  q, k, v, d_o: logical [B, n, Hh, d]
    views sharing strides and dtype.  Returns (dq, dk, dv, dgamma); `grads` may give the three
    output tensors (sharing one set of strides), `workspace` a uint8 device tensor."""
    B, n, Hh, d = q.shape
    for t in (k, v, d_o):
        if t.shape != q.shape or t.stride() != q.stride() or t.dtype != q.dtype:
            raise ValueError("q, k, v, d_o must share shape, strides and dtype")
    if grads is None:
        grads = tuple(torch.empty_like(q, dtype=grad_dtype or q.dtype) for _ in range(3))
    dq, dk, dv = grads
    for t in (dk, dv):
        if t.shape != q.shape or t.stride() != dq.stride() or t.dtype != dq.dtype:
            raise ValueError("dq, dk, dv must share shape, strides and dtype")
    if dq.shape != q.shape:
        raise ValueError("gradient tensors have the wrong shape")
    if gamma.dtype != torch.float32 or gamma.numel() != Hh or not gamma.is_contiguous():
        raise ValueError("gamma must be contiguous fp32 [Hh]")
    if dgamma is None:
        dgamma = torch.empty((Hh,), dtype=torch.float32, device=q.device)
    need = lasad_backward_workspace_bytes(B, Hh, n, d, _dtype_code(q))
    if workspace is None and need:
        workspace = _scratch(need, q.device, stream)
    li, lg = _layout(q), _layout(dq)
    _check(load().lasad_backward_chunked(
        _ptr(q), _ptr(k), _ptr(v), _ptr(d_o), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dgamma),
        ctypes.byref(li), ctypes.byref(lg), _dtype_code(q), _dtype_code(dq),
        B, Hh, d, grid_h, grid_w, start_pos, n, _ptr(gamma), boundary_mode, q_scale,
        _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream(stream)))
    return dq, dk, dv, dgamma


def lasad_backward_carried_workspace_bytes(B: int, n_heads: int, n_tokens: int, d: int, io_dtype: int) -> int:
    return int(load().lasad_backward_carried_workspace_bytes(B, n_heads, n_tokens, d, io_dtype))


def lasad_backward_chunked_carried(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, d_o: torch.Tensor,
                                   gamma: torch.Tensor, grid_h: int, grid_w: int,
                                   state_in: torch.Tensor | None = None, d_state_out: torch.Tensor | None = None,
                                   start_pos: int = 0, boundary_mode: int = RESET_LAST_COL, q_scale: float = 1.0,
                                   grads: tuple | None = None, grad_dtype: torch.dtype | None = None,
                                   dgamma: torch.Tensor | None = None, d_state_in: torch.Tensor | None = None,
                                   workspace: torch.Tensor | None = None, stream=None):
    """lasad_backward_chunked for a call that starts from state_in and whose final state enters the loss with
    gradient d_state_out (fp32 [B, Hh, d, d] each, or None).  Returns (dq, dk, dv, dgamma, d_state_in)."""
    B, n, Hh, d = q.shape
    for t in (k, v, d_o):
        if t.shape != q.shape or t.stride() != q.stride() or t.dtype != q.dtype:
            raise ValueError("q, k, v, d_o must share shape, strides and dtype")
    if grads is None:
        grads = tuple(torch.empty_like(q, dtype=grad_dtype or q.dtype) for _ in range(3))
    dq, dk, dv = grads
    for t in (dk, dv):
        if t.shape != q.shape or t.stride() != dq.stride() or t.dtype != dq.dtype:
            raise ValueError("dq, dk, dv must share shape, strides and dtype")
    for st in (state_in, d_state_out, d_state_in):
        if st is not None and (st.dtype != torch.float32 or not st.is_contiguous() or tuple(st.shape) != (B, Hh, d, d)):
            raise ValueError("states must be contiguous fp32 [B, Hh, d, d]")
    if gamma.dtype != torch.float32 or gamma.numel() != Hh or not gamma.is_contiguous():
        raise ValueError("gamma must be contiguous fp32 [Hh]")
    if dgamma is None:
        dgamma = torch.empty((Hh,), dtype=torch.float32, device=q.device)
    if d_state_in is None:
        d_state_in = torch.empty((B, Hh, d, d), dtype=torch.float32, device=q.device)
    need = lasad_backward_carried_workspace_bytes(B, Hh, n, d, _dtype_code(q))
    if workspace is None and need:
        workspace = _scratch(need, q.device, stream)
    li, lg = _layout(q), _layout(dq)
    _check(load().lasad_backward_chunked_carried(
        _ptr(q), _ptr(k), _ptr(v), _ptr(d_o), _ptr(state_in), _ptr(d_state_out),
        _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dgamma), _ptr(d_state_in),
        ctypes.byref(li), ctypes.byref(lg), _dtype_code(q), _dtype_code(dq),
        B, Hh, d, grid_h, grid_w, start_pos, n, _ptr(gamma), boundary_mode, q_scale,
        _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream(stream)))
    return dq, dk, dv, dgamma, d_state_in


def lasad_backward_gated_workspace_bytes(B: int, n_heads: int, n_tokens: int, d: int) -> int:
    return int(load().lasad_backward_gated_workspace_bytes(B, n_heads, n_tokens, d))


def lasad_backward_gated(q: torch.Tensor, lam: torch.Tensor, v: torch.Tensor, d_o: torch.Tensor,
                         grid_h: int, grid_w: int, k: torch.Tensor | None = None, start_pos: int = 0,
                         boundary_mode: int = RESET_LAST_COL, q_scale: float = 1.0,
                         grads: tuple | None = None, grad_dtype: torch.dtype | None = None,
                         workspace: torch.Tensor | None = None, stream=None):
    """Gradients of lasad_forward_gated (zero initial state).  q, lam, v, d_o (and k, or None for the
    tied key): logical [B, n, Hh, d] views sharing strides and dtype.  Returns (dq, dlam, dv) with the
    tied key, (dq, dlam, dv, dk) with an own key; `grads` may give these output tensors (sharing one set
    of strides), `workspace` a uint8 device tensor."""
    B, n, Hh, d = q.shape
    for t in (lam, v, d_o) + (() if k is None else (k,)):
        if t.shape != q.shape or t.stride() != q.stride() or t.dtype != q.dtype:
            raise ValueError("q, lam, k, v, d_o must share shape, strides and dtype")
    if grads is None:
        grads = tuple(torch.empty_like(q, dtype=grad_dtype or q.dtype) for _ in range(3 if k is None else 4))
    if len(grads) != (3 if k is None else 4):
        raise ValueError("grads must hold dq, dlam, dv (and dk with an own key)")
    dq, dlam, dv = grads[:3]
    dk = None if k is None else grads[3]
    for t in grads:
        if t.shape != q.shape or t.stride() != dq.stride() or t.dtype != dq.dtype:
            raise ValueError("gradient tensors must share q's shape and one set of strides and dtype")
    need = lasad_backward_gated_workspace_bytes(B, Hh, n, d)
    if workspace is None and need:
        workspace = _scratch(need, q.device, stream)
    li, lg = _layout(q), _layout(dq)
    _check(load().lasad_backward_gated(
        _ptr(q), _ptr(lam), _ptr(k), _ptr(v), _ptr(d_o), _ptr(dq), _ptr(dlam), _ptr(dk), _ptr(dv),
        ctypes.byref(li), ctypes.byref(lg), _dtype_code(q), _dtype_code(dq),
        B, Hh, d, grid_h, grid_w, start_pos, n, boundary_mode, q_scale,
        _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream(stream)))
    return (dq, dlam, dv) if k is None else (dq, dlam, dv, dk)


def lasad_backward_gated_carried_workspace_bytes(B: int, n_heads: int, n_tokens: int, d: int) -> int:
    return int(load().lasad_backward_gated_carried_workspace_bytes(B, n_heads, n_tokens, d))


def lasad_backward_gated_carried(q: torch.Tensor, lam: torch.Tensor, v: torch.Tensor, d_o: torch.Tensor,
                                 grid_h: int, grid_w: int, k: torch.Tensor | None = None,
                                 state_in: torch.Tensor | None = None, d_state_out: torch.Tensor | None = None,
                                 start_pos: int = 0, boundary_mode: int = RESET_LAST_COL, q_scale: float = 1.0,
                                 grads: tuple | None = None, grad_dtype: torch.dtype | None = None,
                                 d_state_in: torch.Tensor | None = None,
                                 workspace: torch.Tensor | None = None, stream=None):
    """lasad_backward_gated for a call that starts from state_in and whose final state enters the loss with gradient
    d_state_out (fp32 [B, Hh, d, d] each, or None).  Returns (dq, dlam, dv[, dk], d_state_in)."""
    B, n, Hh, d = q.shape
    for t in (lam, v, d_o) + (() if k is None else (k,)):
        if t.shape != q.shape or t.stride() != q.stride() or t.dtype != q.dtype:
            raise ValueError("q, lam, k, v, d_o must share shape, strides and dtype")
    if grads is None:
        grads = tuple(torch.empty_like(q, dtype=grad_dtype or q.dtype) for _ in range(3 if k is None else 4))
    if len(grads) != (3 if k is None else 4):
        raise ValueError("grads must hold dq, dlam, dv (and dk with an own key)")
    dq, dlam, dv = grads[:3]
    dk = None if k is None else grads[3]
    for t in grads:
        if t.shape != q.shape or t.stride() != dq.stride() or t.dtype != dq.dtype:
            raise ValueError("gradient tensors must share q's shape and one set of strides and dtype")
    for st in (state_in, d_state_out, d_state_in):
        if st is not None and (st.dtype != torch.float32 or not st.is_contiguous() or tuple(st.shape) != (B, Hh, d, d)):
            raise ValueError("states must be contiguous fp32 [B, Hh, d, d]")
    if d_state_in is None:
        d_state_in = torch.empty((B, Hh, d, d), dtype=torch.float32, device=q.device)
    need = lasad_backward_gated_carried_workspace_bytes(B, Hh, n, d)
    if workspace is None and need:
        workspace = _scratch(need, q.device, stream)
    li, lg = _layout(q), _layout(dq)
    _check(load().lasad_backward_gated_carried(
        _ptr(q), _ptr(lam), _ptr(k), _ptr(v), _ptr(d_o), _ptr(state_in), _ptr(d_state_out),
        _ptr(dq), _ptr(dlam), _ptr(dk), _ptr(dv), _ptr(d_state_in),
        ctypes.byref(li), ctypes.byref(lg), _dtype_code(q), _dtype_code(dq),
        B, Hh, d, grid_h, grid_w, start_pos, n, boundary_mode, q_scale,
        _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream(stream)))
    return ((dq, dlam, dv) if k is None else (dq, dlam, dv, dk)) + (d_state_in,)


def lasad_backward_layer_workspace_bytes(q_pre: torch.Tensor) -> int:
    B, n, Hh, d = q_pre.shape
    lq = _layout(q_pre)
    return int(load().lasad_backward_layer_workspace_bytes(B, Hh, n, d, _dtype_code(q_pre), ctypes.byref(lq)))


def lasad_backward_layer(q_pre: torch.Tensor, z: torch.Tensor, v: torch.Tensor, d_out: torch.Tensor,
                         grid_h: int, grid_w: int, norm_weight: torch.Tensor | None = None, norm_eps: float = 1e-6,
                         start_pos: int = 0, boundary_mode: int = RESET_LAST_COL, q_scale: float = 1.0,
                         grads: tuple | None = None, grad_dtype: torch.dtype | None = None,
                         dweight: torch.Tensor | None = None, want_dweight: bool = True,
                         workspace: torch.Tensor | None = None, stream=None):
    """Gradients of lasad_forward_layer (zero initial state).  q_pre, z, v: logical [B, n, Hh, 64] views
    sharing strides and dtype; d_out of the same shape and dtype with strides of its own.  Returns
    (dq_pre, dz, dv, dweight); dweight is fp32 [Hh, d], or None with want_dweight=False."""
    B, n, Hh, d = q_pre.shape
    for t in (z, v):
        if t.shape != q_pre.shape or t.stride() != q_pre.stride() or t.dtype != q_pre.dtype:
            raise ValueError("q_pre, z, v must share shape, strides and dtype")
    if d_out.shape != q_pre.shape or d_out.dtype != q_pre.dtype:
        raise ValueError("d_out must have q_pre's shape and dtype")
    if norm_weight is not None and (norm_weight.dtype != torch.float32 or not norm_weight.is_contiguous()
                                    or norm_weight.numel() != Hh * d):
        raise ValueError("norm_weight must be contiguous fp32 [Hh, d]")
    if grads is None:
        grads = tuple(torch.empty_like(q_pre, dtype=grad_dtype or q_pre.dtype) for _ in range(3))
    dq, dz, dv = grads
    for t in grads:
        if t.shape != q_pre.shape or t.stride() != dq.stride() or t.dtype != dq.dtype:
            raise ValueError("gradient tensors must share q_pre's shape and one set of strides and dtype")
    if dweight is None and want_dweight:
        dweight = torch.empty((Hh, d), dtype=torch.float32, device=q_pre.device)
    if dweight is not None and (dweight.dtype != torch.float32 or not dweight.is_contiguous() or dweight.numel() != Hh * d):
        raise ValueError("dweight must be contiguous fp32 [Hh, d]")
    need = lasad_backward_layer_workspace_bytes(q_pre)
    if workspace is None and need:
        workspace = _scratch(need, q_pre.device, stream)
    li, lo, lg = _layout(q_pre), _layout(d_out), _layout(dq)
    _check(load().lasad_backward_layer(
        _ptr(q_pre), _ptr(z), _ptr(v), _ptr(d_out), _ptr(dq), _ptr(dz), _ptr(dv), _ptr(dweight),
        ctypes.byref(li), ctypes.byref(lo), ctypes.byref(lg), _dtype_code(q_pre), _dtype_code(dq),
        B, Hh, d, grid_h, grid_w, start_pos, n, boundary_mode, q_scale, _ptr(norm_weight), norm_eps,
        _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream(stream)))
    return dq, dz, dv, dweight


def lasad_backward_layer_norm(q_pre: torch.Tensor, z: torch.Tensor, v: torch.Tensor, d_out: torch.Tensor,
                              grid_h: int, grid_w: int, norm_weight: torch.Tensor | None = None, norm_eps: float = 1e-6,
                              start_pos: int = 0, boundary_mode: int = RESET_LAST_COL, q_scale: float = 1.0,
                              d_o: torch.Tensor | None = None, d_o_dtype: torch.dtype | None = None,
                              want_dweight: bool = True, workspace: torch.Tensor | None = None, stream=None):
    """The normalisation's part of lasad_backward_layer alone: returns (d_o, dweight), d_o = dL/d(recurrence
    output) in the inputs' dtype (or fp32 on request)."""
    B, n, Hh, d = q_pre.shape
    for t in (z, v):
        if t.shape != q_pre.shape or t.stride() != q_pre.stride() or t.dtype != q_pre.dtype:
            raise ValueError("q_pre, z, v must share shape, strides and dtype")
    if d_out.shape != q_pre.shape or d_out.dtype != q_pre.dtype:
        raise ValueError("d_out must have q_pre's shape and dtype")
    if d_o is None:
        d_o = torch.empty(q_pre.shape, dtype=d_o_dtype or q_pre.dtype, device=q_pre.device)
    if d_o.shape != q_pre.shape:
        raise ValueError("d_o must have q_pre's shape")
    dweight = torch.empty((Hh, d), dtype=torch.float32, device=q_pre.device) if want_dweight else None
    need = lasad_backward_layer_workspace_bytes(q_pre)
    if workspace is None and need:
        workspace = _scratch(need, q_pre.device, stream)
    li, lo, ld = _layout(q_pre), _layout(d_out), _layout(d_o)
    _check(load().lasad_backward_layer_norm(
        _ptr(q_pre), _ptr(z), _ptr(v), _ptr(d_out), _ptr(d_o), _ptr(dweight),
        ctypes.byref(li), ctypes.byref(lo), ctypes.byref(ld), _dtype_code(q_pre), _dtype_code(d_o),
        B, Hh, d, grid_h, grid_w, start_pos, n, boundary_mode, q_scale, _ptr(norm_weight), norm_eps,
        _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream(stream)))
    return d_o, dweight


# ---- host <-> device helpers for seeded numpy inputs (no arithmetic) ---------

def to_device(x, dtype: str, device="cuda"):
    """Upload a float32 numpy array (values already storage-rounded) as an f32 or bf16 tensor,
    keeping the numpy array's strides (so a transposed view stays a transposed view)."""
    import numpy as np
    t = torch.from_numpy(np.ascontiguousarray(x))
    if not x.flags.c_contiguous:
        # rebuild the same permutation on the device
        order = sorted(range(x.ndim), key=lambda i: -x.strides[i])
        t = torch.from_numpy(np.ascontiguousarray(x.transpose(order)))
        inv = [order.index(i) for i in range(x.ndim)]
        t = t.to(device).permute(inv)
    else:
        t = t.to(device)
    if dtype == "bf16":
        return t.to(torch.bfloat16)    # exact: the values are already bf16-representable
    if dtype == "f32":
        return t
    raise ValueError(dtype)
