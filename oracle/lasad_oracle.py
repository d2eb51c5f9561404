"""ctypes front-end of the LASAD CPU oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
module.  It compiles ``lasad_oracle.c`` with gcc (fp64, OpenMP, no BLAS) into
``liblasad_oracle.so`` next to the source and marshals numpy arrays; every bit
of arithmetic is in the C file.  It imports nothing from the HIP package.

Array convention at this level: q, k, v, o are ``[B, n, Hh, d]`` (what a
projection producing model width Hh*d yields, Algorithm 1 input X[B, N, D]);
states are ``[B, Hh, d, d]`` with S[i, j] = sum_t k_t[i] v_t[j].
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lasad_oracle.c")
_LIB = os.path.join(_HERE, "liblasad_oracle.so")

RESET_LAST_COL, RESET_FIRST_COL, RESET_NONE = 0, 1, 2

_lib = None


def build(force: bool = True) -> str:
    """Compile the C oracle (gcc -O2 -fopenmp).  Returns the library path.

    With force=False an existing library is kept as it is (the loader's case:
    it only compiles when nothing has been built yet)."""
    if force or not os.path.exists(_LIB):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build(force=False))
        dp = ctypes.POINTER(ctypes.c_double)
        fp = ctypes.POINTER(ctypes.c_float)
        ip = ctypes.POINTER(ctypes.c_int32)
        ci = ctypes.c_int
        lib.lasad_oracle_decay_factors.argtypes = [fp, ci, ci, ci, ci, ci, ci, fp, ip]
        lib.lasad_oracle_decay_factors.restype = ci
        for name in ("lasad_oracle_forward_fullmask", "lasad_oracle_recurrent"):
            f = getattr(lib, name)
            f.argtypes = [dp, dp, dp, dp, ctypes.c_double, dp, dp, dp, ci, ci, ci, ci]
            f.restype = ci
        lib.lasad_oracle_decode_step.argtypes = [dp, dp, dp, dp, ctypes.c_double, dp, dp, ci, ci, ci]
        lib.lasad_oracle_decode_step.restype = ci
        lib.lasad_oracle_bruteforce.argtypes = [dp, dp, dp, dp, ctypes.c_double, dp, ci, ci]
        lib.lasad_oracle_bruteforce.restype = ci
        lib.lasad_oracle_gated_recurrent.argtypes = [dp, dp, dp, dp, ctypes.c_double, dp, dp, dp,
                                                     ci, ci, ci, ci, ci, ci, ci]
        lib.lasad_oracle_gated_backward.argtypes = [dp, dp, dp, dp, ctypes.c_double, dp, dp, dp, dp, dp,
                                                    ci, ci, ci, ci, ci, ci, ci]
        lib.lasad_oracle_gated_backward.restype = ci
        lib.lasad_oracle_gated_recurrent.restype = ci
        lib.lasad_oracle_gated_bruteforce.argtypes = [dp, dp, dp, dp, ctypes.c_double, dp, ci, ci, ci, ci, ci]
        lib.lasad_oracle_gated_bruteforce.restype = ci
        lib.lasad_oracle_backward.argtypes = [dp, dp, dp, dp, ctypes.c_double, dp, dp, dp, dp, dp, ci, ci, ci, ci]
        lib.lasad_oracle_backward.restype = ci
        lib.lasad_oracle_backward_carried.argtypes = [dp, dp, dp, dp, ctypes.c_double, dp, dp, dp, dp, dp, dp, dp, dp,
                                                      ci, ci, ci, ci]
        lib.lasad_oracle_backward_carried.restype = ci
        lib.lasad_oracle_gated_backward_carried.argtypes = [dp, dp, dp, dp, ctypes.c_double, dp, dp, dp, dp, dp, dp, dp, dp,
                                                            ci, ci, ci, ci, ci, ci, ci]
        lib.lasad_oracle_gated_backward_carried.restype = ci
        lib.lasad_oracle_dgamma.argtypes = [dp, ci, ci, ci, ci, ci, ci, dp]
        lib.lasad_oracle_dgamma.restype = ci
        lib.lasad_oracle_num_threads.argtypes = []
        lib.lasad_oracle_num_threads.restype = ci
        _lib = lib
    return _lib


def _dptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _f64c(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def num_threads() -> int:
    return int(_load().lasad_oracle_num_threads())


def decay_factors(gamma, grid_h, grid_w, start_pos, n_tokens, mode=RESET_LAST_COL):
    """Return (lam[Hh, n] float32, cum_exp[n+1] int32) for positions start_pos+1..start_pos+n."""
    g = np.ascontiguousarray(np.asarray(gamma, dtype=np.float32))
    lam = np.empty((g.shape[0], n_tokens), dtype=np.float32)
    cum = np.empty((n_tokens + 1,), dtype=np.int32)
    rc = _load().lasad_oracle_decay_factors(
        g.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), g.shape[0], grid_h, grid_w,
        start_pos, n_tokens, mode,
        lam.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
        cum.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    if rc != 0:
        raise ValueError(f"lasad_oracle_decay_factors: bad arguments (rc={rc})")
    return lam, cum


def _sequence_call(fn_name, q, k, v, lam, q_scale, s0, want_state):
    q, k, v = (np.asarray(x, dtype=np.float64) for x in (q, k, v))
    B, n, Hh, d = q.shape
    assert k.shape == q.shape and v.shape == q.shape
    lam = _f64c(lam)
    assert lam.shape == (Hh, n), (lam.shape, (Hh, n))
    # [B, n, Hh, d] -> [B, Hh, n, d]
    qh, kh, vh = (np.ascontiguousarray(x.transpose(0, 2, 1, 3)) for x in (q, k, v))
    oh = np.empty_like(qh)
    s0c = None if s0 is None else _f64c(s0)
    if s0c is not None:
        assert s0c.shape == (B, Hh, d, d)
    s_out = np.empty((B, Hh, d, d), dtype=np.float64) if want_state else None
    rc = getattr(_load(), fn_name)(_dptr(qh), _dptr(kh), _dptr(vh), _dptr(lam), float(q_scale),
                                   _dptr(s0c), _dptr(oh), _dptr(s_out), B, Hh, n, d)
    if rc != 0:
        raise RuntimeError(f"{fn_name} failed (rc={rc})")
    o = np.ascontiguousarray(oh.transpose(0, 2, 1, 3))
    return (o, s_out) if want_state else o


def forward_fullmask(q, k, v, lam, q_scale=1.0, s0=None, want_state=False):
    """O = (q_scale QK^T (.) M) V with the full n x n decay mask (plus carried-state terms)."""
    return _sequence_call("lasad_oracle_forward_fullmask", q, k, v, lam, q_scale, s0, want_state)


def recurrent(q, k, v, lam, q_scale=1.0, s0=None, want_state=False):
    """The sequential recurrence of Algorithm 1 in fp64."""
    return _sequence_call("lasad_oracle_recurrent", q, k, v, lam, q_scale, s0, want_state)


def decode_step(q, k, v, lam_t, state, q_scale=1.0):
    """One token for every (b, h).  q, k, v: [B, Hh, d]; state [B, Hh, d, d] fp64 updated IN PLACE."""
    q, k, v = (_f64c(x) for x in (q, k, v))
    B, Hh, d = q.shape
    lam_t = _f64c(lam_t)
    assert lam_t.shape == (Hh,)
    assert state.dtype == np.float64 and state.flags.c_contiguous and state.shape == (B, Hh, d, d)
    o = np.empty_like(q)
    rc = _load().lasad_oracle_decode_step(_dptr(q), _dptr(k), _dptr(v), _dptr(lam_t), float(q_scale),
                                          _dptr(state), _dptr(o), B, Hh, d)
    if rc != 0:
        raise RuntimeError(f"lasad_oracle_decode_step failed (rc={rc})")
    return o


def bruteforce(q, k, v, lam, q_scale=1.0):
    """Per-pair sums for ONE sequence: q, k, v [n, d], lam [n]."""
    q, k, v, lam = (_f64c(x) for x in (q, k, v, lam))
    n, d = q.shape
    assert lam.shape == (n,)
    o = np.empty_like(q)
    rc = _load().lasad_oracle_bruteforce(_dptr(q), _dptr(k), _dptr(v), _dptr(lam), float(q_scale),
                                         _dptr(o), n, d)
    if rc != 0:
        raise RuntimeError(f"lasad_oracle_bruteforce failed (rc={rc})")
    return o


# ---- gradients of the scalar-decay path --------------------------------------------------------

def backward(q, k, v, lam, d_o, q_scale=1.0):
    """Gradients of the recurrence from a zero state.  q, k, v, d_o: [B, n, Hh, d]; lam [Hh, n].
    Returns dq, dk, dv [B, n, Hh, d] and dlam [B, Hh, n] (per sequence and token)."""
    q, k, v, d_o = (np.asarray(x, dtype=np.float64) for x in (q, k, v, d_o))
    B, n, Hh, d = q.shape
    assert k.shape == q.shape and v.shape == q.shape and d_o.shape == q.shape
    lam = _f64c(lam)
    assert lam.shape == (Hh, n)
    qh, kh, vh, gh = (np.ascontiguousarray(x.transpose(0, 2, 1, 3)) for x in (q, k, v, d_o))
    dqh, dkh, dvh = np.empty_like(qh), np.empty_like(qh), np.empty_like(qh)
    dlam = np.empty((B, Hh, n), dtype=np.float64)
    rc = _load().lasad_oracle_backward(_dptr(qh), _dptr(kh), _dptr(vh), _dptr(lam), float(q_scale), _dptr(gh),
                                       _dptr(dqh), _dptr(dkh), _dptr(dvh), _dptr(dlam), B, Hh, n, d)
    if rc != 0:
        raise RuntimeError(f"lasad_oracle_backward failed (rc={rc})")
    dq, dk, dv = (np.ascontiguousarray(x.transpose(0, 2, 1, 3)) for x in (dqh, dkh, dvh))
    return dq, dk, dv, dlam


def _state(x, B, Hh, d):
    if x is None:
        return None
    x = _f64c(x)
    assert x.shape == (B, Hh, d, d)
    return x


def backward_carried(q, k, v, lam, d_o, s0=None, d_state=None, q_scale=1.0):
    """Gradients of the recurrence for a call that starts from the state s0 [B, Hh, d, d] (None: zero) and whose
    final state s_n also enters the loss with gradient d_state = dL/ds_n (None: zero).  Other arguments as
    backward().  Returns dq, dk, dv [B, n, Hh, d], dlam [B, Hh, n] and d_s0 = dL/ds_0 [B, Hh, d, d]."""
    q, k, v, d_o = (np.asarray(x, dtype=np.float64) for x in (q, k, v, d_o))
    B, n, Hh, d = q.shape
    assert k.shape == q.shape and v.shape == q.shape and d_o.shape == q.shape
    lam = _f64c(lam)
    assert lam.shape == (Hh, n)
    s0, d_state = _state(s0, B, Hh, d), _state(d_state, B, Hh, d)
    qh, kh, vh, gh = (np.ascontiguousarray(x.transpose(0, 2, 1, 3)) for x in (q, k, v, d_o))
    dqh, dkh, dvh = np.empty_like(qh), np.empty_like(qh), np.empty_like(qh)
    dlam = np.empty((B, Hh, n), dtype=np.float64)
    d_s0 = np.empty((B, Hh, d, d), dtype=np.float64)
    rc = _load().lasad_oracle_backward_carried(_dptr(qh), _dptr(kh), _dptr(vh), _dptr(lam), float(q_scale), _dptr(gh),
                                               _dptr(s0), _dptr(d_state), _dptr(dqh), _dptr(dkh), _dptr(dvh),
                                               _dptr(dlam), _dptr(d_s0), B, Hh, n, d)
    if rc != 0:
        raise RuntimeError(f"lasad_oracle_backward_carried failed (rc={rc})")
    dq, dk, dv = (np.ascontiguousarray(x.transpose(0, 2, 1, 3)) for x in (dqh, dkh, dvh))
    return dq, dk, dv, dlam, d_s0


def dgamma(dlam, grid_w, start_pos=0, mode=RESET_LAST_COL):
    """Sum of the per-token decay gradients over the non-boundary positions and the batch: [Hh]."""
    dlam = _f64c(dlam)
    B, Hh, n = dlam.shape
    out = np.empty((Hh,), dtype=np.float64)
    rc = _load().lasad_oracle_dgamma(_dptr(dlam), B, Hh, n, int(grid_w), int(start_pos), int(mode), _dptr(out))
    if rc != 0:
        raise RuntimeError(f"lasad_oracle_dgamma failed (rc={rc})")
    return out


# ---- vector, data-dependent decay (Section 3.4 / Algorithm 1 as written) ----------------------

def gated_recurrent(q, lam, v, grid_w, k=None, start_pos=0, mode=RESET_LAST_COL, q_scale=1.0, s0=None,
                    want_state=False):
    """Sequential recurrence with a decay vector per token.  q, lam, v (and k, or None for
    k = 1 - lam): [B, n, Hh, d]; returns o [B, n, Hh, d] (and the final state [B, Hh, d, d])."""
    q, lam, v = (np.asarray(x, dtype=np.float64) for x in (q, lam, v))
    B, n, Hh, d = q.shape
    assert lam.shape == q.shape and v.shape == q.shape
    tr = lambda x: np.ascontiguousarray(x.transpose(0, 2, 1, 3))
    qh, lh, vh = tr(q), tr(lam), tr(v)
    kh = None if k is None else tr(np.asarray(k, dtype=np.float64))
    oh = np.empty_like(qh)
    s0c = None if s0 is None else _f64c(s0)
    s_out = np.empty((B, Hh, d, d), dtype=np.float64) if want_state else None
    rc = _load().lasad_oracle_gated_recurrent(_dptr(qh), _dptr(lh), _dptr(kh), _dptr(vh), float(q_scale),
                                              _dptr(s0c), _dptr(oh), _dptr(s_out), B, Hh, n, d,
                                              grid_w, start_pos, mode)
    if rc != 0:
        raise RuntimeError(f"lasad_oracle_gated_recurrent failed (rc={rc})")
    o = np.ascontiguousarray(oh.transpose(0, 2, 1, 3))
    return (o, s_out) if want_state else o


def gated_bruteforce(q, lam, v, grid_w, k=None, start_pos=0, mode=RESET_LAST_COL, q_scale=1.0):
    """Per-pair, per-channel sums for ONE sequence: q, lam, v (k) are [n, d]."""
    q, lam, v = (_f64c(x) for x in (q, lam, v))
    kc = None if k is None else _f64c(k)
    n, d = q.shape
    o = np.empty_like(q)
    rc = _load().lasad_oracle_gated_bruteforce(_dptr(q), _dptr(lam), _dptr(kc), _dptr(v), float(q_scale),
                                               _dptr(o), n, d, grid_w, start_pos, mode)
    if rc != 0:
        raise RuntimeError(f"lasad_oracle_gated_bruteforce failed (rc={rc})")
    return o


def gated_backward(q, lam, v, d_o, grid_w, k=None, start_pos=0, mode=RESET_LAST_COL, q_scale=1.0):
    """Gradients of gated_recurrent (zero initial state) for d_o = dL/do.  All [B, n, Hh, d].
    Tied key (k None): returns (dq, dlam, dv) with dlam the gradient for the lambda INPUT (through the
    decay where the position is no boundary, and through k = 1 - lambda).  Own key: (dq, dlam, dv, dk)."""
    q, lam, v, d_o = (np.asarray(x, dtype=np.float64) for x in (q, lam, v, d_o))
    B, n, Hh, d = q.shape
    assert lam.shape == q.shape and v.shape == q.shape and d_o.shape == q.shape
    tr = lambda x: np.ascontiguousarray(x.transpose(0, 2, 1, 3))
    qh, lh, vh, gh = tr(q), tr(lam), tr(v), tr(d_o)
    kh = None if k is None else tr(np.asarray(k, dtype=np.float64))
    dq, dl, dv = np.empty_like(qh), np.empty_like(qh), np.empty_like(qh)
    dk = None if k is None else np.empty_like(qh)
    rc = _load().lasad_oracle_gated_backward(_dptr(qh), _dptr(lh), _dptr(kh), _dptr(vh), float(q_scale), _dptr(gh),
                                             _dptr(dq), _dptr(dl), _dptr(dk), _dptr(dv), B, Hh, n, d,
                                             grid_w, start_pos, mode)
    if rc != 0:
        raise RuntimeError(f"lasad_oracle_gated_backward failed (rc={rc})")
    back = lambda x: np.ascontiguousarray(x.transpose(0, 2, 1, 3))
    if k is None:
        return back(dq), back(dl), back(dv)
    return back(dq), back(dl), back(dv), back(dk)


def gated_backward_carried(q, lam, v, d_o, grid_w, k=None, s0=None, d_state=None, start_pos=0, mode=RESET_LAST_COL,
                           q_scale=1.0):
    """gated_backward for a call that starts from the state s0 (None: zero) and whose final state enters the loss
    with gradient d_state (None: zero).  Returns (dq, dlam, dv[, dk], d_s0), d_s0 = dL/ds_0 [B, Hh, d, d]."""
    q, lam, v, d_o = (np.asarray(x, dtype=np.float64) for x in (q, lam, v, d_o))
    B, n, Hh, d = q.shape
    assert lam.shape == q.shape and v.shape == q.shape and d_o.shape == q.shape
    s0, d_state = _state(s0, B, Hh, d), _state(d_state, B, Hh, d)
    tr = lambda x: np.ascontiguousarray(x.transpose(0, 2, 1, 3))
    qh, lh, vh, gh = tr(q), tr(lam), tr(v), tr(d_o)
    kh = None if k is None else tr(np.asarray(k, dtype=np.float64))
    dq, dl, dv = np.empty_like(qh), np.empty_like(qh), np.empty_like(qh)
    dk = None if k is None else np.empty_like(qh)
    d_s0 = np.empty((B, Hh, d, d), dtype=np.float64)
    rc = _load().lasad_oracle_gated_backward_carried(_dptr(qh), _dptr(lh), _dptr(kh), _dptr(vh), float(q_scale), _dptr(gh),
                                                     _dptr(s0), _dptr(d_state), _dptr(dq), _dptr(dl), _dptr(dk), _dptr(dv),
                                                     _dptr(d_s0), B, Hh, n, d, grid_w, start_pos, mode)
    if rc != 0:
        raise RuntimeError(f"lasad_oracle_gated_backward_carried failed (rc={rc})")
    back = lambda x: np.ascontiguousarray(x.transpose(0, 2, 1, 3))
    if k is None:
        return back(dq), back(dl), back(dv), d_s0
    return back(dq), back(dl), back(dv), back(dk), d_s0


# ---- Algorithm 1's elementwise steps around the recurrence --------------------------------------

def silu(x):
    """SiLU(x) = x * sigmoid(x) (Algorithm 1, the line after the projections), fp64."""
    x = np.asarray(x, dtype=np.float64)
    return x * sigmoid(x)


def sigmoid(x):
    """1 / (1 + exp(-x)), fp64, evaluated without overflow on either side."""
    x = np.asarray(x, dtype=np.float64)
    e = np.exp(-np.abs(x))
    return np.where(x >= 0, 1.0 / (1.0 + e), e / (1.0 + e))


def rms_norm(o, weight=None, eps=1e-6):
    """Norm(o_t) of Algorithm 1's last line, read as a root-mean-square normalisation over the d
    channels of each head: o / sqrt(mean(o^2) + eps), times an optional per-(head, channel) weight."""
    o = np.asarray(o, dtype=np.float64)
    out = o / np.sqrt(np.mean(o * o, axis=-1, keepdims=True) + eps)
    if weight is not None:
        out = out * np.asarray(weight, dtype=np.float64)       # [Hh, d] broadcast over [B, n, Hh, d]
    return out


def gated_layer(q_pre, z, v, grid_w, norm_weight=None, eps=1e-6, start_pos=0, mode=RESET_LAST_COL,
                q_scale=1.0, s0=None, want_state=False):
    """Algorithm 1's loop body between the two Linear maps: q = SiLU(q_pre), lambda = sigmoid(z),
    k = 1 - lambda, the spatially aware recurrence, then Norm(o).  Shapes as gated_recurrent."""
    r = gated_recurrent(silu(q_pre), sigmoid(z), v, grid_w, k=None, start_pos=start_pos, mode=mode,
                        q_scale=q_scale, s0=s0, want_state=want_state)
    o, s = (r if want_state else (r, None))
    o = rms_norm(o, norm_weight, eps)
    return (o, s) if want_state else o


def layer_norm_backward(q_pre, z, v, d_out, grid_w, norm_weight=None, eps=1e-6, start_pos=0, mode=RESET_LAST_COL,
                        q_scale=1.0):
    """The normalisation's part of the layer's backward: d_o = dL/d(recurrence output) [B, n, Hh, d] and
    dweight [Hh, d] (without a weight: the gradient at a weight of ones) for d_out = dL/d(layer output).
    y = o rstd w with rstd = (mean_c(o^2) + eps)^(-1/2), so with gw = d_out w:
    d_o = rstd gw - o rstd^3 mean_c(gw o)."""
    q_pre, z, v, d_out = (np.asarray(x, dtype=np.float64) for x in (q_pre, z, v, d_out))
    d = q_pre.shape[-1]
    o = gated_recurrent(silu(q_pre), sigmoid(z), v, grid_w, k=None, start_pos=start_pos, mode=mode, q_scale=q_scale)
    rstd = 1.0 / np.sqrt(np.mean(o * o, axis=-1, keepdims=True) + eps)
    w = np.ones(q_pre.shape[-2:]) if norm_weight is None else np.asarray(norm_weight, dtype=np.float64)
    gw = d_out * w
    d_o = rstd * gw - o * (rstd ** 3) * np.sum(gw * o, axis=-1, keepdims=True) / d
    dweight = np.sum(d_out * o * rstd, axis=(0, 1))
    return d_o, dweight


def layer_core_backward(q_pre, z, v, d_o, grid_w, start_pos=0, mode=RESET_LAST_COL, q_scale=1.0):
    """The recurrence's and the activations' part: dq_pre, dz, dv for d_o = dL/d(recurrence output), through
    lasad_oracle_gated_backward (tied key) and SiLU'(x) = s (1 + x (1 - s)), s = sigmoid(x); sigmoid' = lam (1 - lam)."""
    q_pre, z = np.asarray(q_pre, dtype=np.float64), np.asarray(z, dtype=np.float64)
    lam = sigmoid(z)
    dq, dlam, dv = gated_backward(silu(q_pre), lam, v, d_o, grid_w, k=None, start_pos=start_pos, mode=mode, q_scale=q_scale)
    sg = sigmoid(q_pre)
    return dq * sg * (1.0 + q_pre * (1.0 - sg)), dlam * lam * (1.0 - lam), dv


def gated_layer_backward(q_pre, z, v, d_out, grid_w, norm_weight=None, eps=1e-6, start_pos=0, mode=RESET_LAST_COL,
                         q_scale=1.0):
    """Gradients of gated_layer (zero initial state) for d_out = dL/d(layer output): layer_norm_backward, then
    layer_core_backward.  Returns dq_pre, dz, dv [B, n, Hh, d] and dweight [Hh, d]."""
    d_o, dweight = layer_norm_backward(q_pre, z, v, d_out, grid_w, norm_weight, eps, start_pos, mode, q_scale)
    dq_pre, dz, dv = layer_core_backward(q_pre, z, v, d_o, grid_w, start_pos, mode, q_scale)
    return dq_pre, dz, dv, dweight
