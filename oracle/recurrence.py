"""ctypes loader for the fp64 C oracle (TEST INFRASTRUCTURE, not product code).

The arithmetic lives in ``kda_oracle.c`` (paper Section 3, Eq. (1)); this file
only compiles it with gcc, marshals numpy arrays and widens nothing itself:
inputs are passed as float32 (bf16 and fp32 values are exact in float32) and
the C code widens them to double before use.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kda_oracle.c")
_LIB = os.path.join(_HERE, "libkda_oracle.so")
_lib = None


def build(force=False):
    """Compile kda_oracle.c with gcc (OpenMP) into libkda_oracle.so."""
    global _lib
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
        _lib = None
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.kda_oracle_num_threads.restype = ctypes.c_int
        lib.kda_oracle_forward.restype = ctypes.c_int
        lib.kda_oracle_forward.argtypes = [
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p]
        lib.kda_oracle_backward.restype = ctypes.c_int
        lib.kda_oracle_backward.argtypes = [
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int64] + [ctypes.c_void_p] * 7 + [ctypes.c_double] + [ctypes.c_void_p] * 8
        _lib = lib
    return _lib


def num_threads():
    """Threads the oracle's parallel loop over (sequence, head) will use."""
    return int(_load().kda_oracle_num_threads())


def _f32(x, shape=None):
    a = np.ascontiguousarray(np.asarray(x), dtype=np.float32)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError("expected shape %r, got %r" % (tuple(shape), a.shape))
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def kda_forward(q, k, v, log_alpha, beta, h0=None, cu_seqlens=None, scale=1.0,
                want_o=True, want_hT=True):
    """Run the fp64 recurrence.

    q, k, log_alpha: [B,T,H,dk]; v: [B,T,H,dv]; beta: [B,T,H] (any float array;
    taken as float32).  h0: [N,H,dk,dv] or None.  cu_seqlens: int array [N+1]
    (then B must be 1) or None (then N = B).  Returns (o, hT) as float64 arrays
    (None for the ones not wanted).
    """
    q = _f32(q)
    B, T, H, dk = q.shape
    k = _f32(k, (B, T, H, dk))
    log_alpha = _f32(log_alpha, (B, T, H, dk))
    v = _f32(v)
    dv = v.shape[-1]
    if v.shape != (B, T, H, dv):
        raise ValueError("bad v shape %r" % (v.shape,))
    beta = _f32(beta, (B, T, H))
    cu = None
    if cu_seqlens is not None:
        cu = np.ascontiguousarray(np.asarray(cu_seqlens), dtype=np.int64)
        N = cu.shape[0] - 1
    else:
        N = B
    h0d = None
    if h0 is not None:
        h0d = np.ascontiguousarray(np.asarray(h0), dtype=np.float64)
        if h0d.shape != (N, H, dk, dv):
            raise ValueError("bad h0 shape %r" % (h0d.shape,))
    o = np.empty((B, T, H, dv), dtype=np.float64) if want_o else None
    hT = np.empty((N, H, dk, dv), dtype=np.float64) if want_hT else None
    rc = _load().kda_oracle_forward(B, T, H, dk, dv, N, _ptr(q), _ptr(k), _ptr(v),
                                    _ptr(log_alpha), _ptr(beta), _ptr(h0d), _ptr(cu),
                                    float(scale), _ptr(o), _ptr(hT))
    if rc != 0:
        raise ValueError("kda_oracle_forward rejected the call (code %d)" % rc)
    if want_o and cu is not None and cu[-1] < T:
        o[:, cu[-1]:] = 0.0  # tokens past the last sequence belong to nobody
    return o, hT


def kda_step(q, k, v, log_alpha, beta, S, scale=1.0):
    """One decode step of Eq. (1) for N sequences.

    q, k, log_alpha: [N,H,dk]; v: [N,H,dv]; beta: [N,H]; S: [N,H,dk,dv].
    Returns (o [N,H,dv], S_new [N,H,dk,dv]) in float64; S is not modified.
    """
    q = np.asarray(q)
    N, H, dk = q.shape
    o, S_new = kda_forward(np.asarray(q)[:, None], np.asarray(k)[:, None],
                           np.asarray(v)[:, None], np.asarray(log_alpha)[:, None],
                           np.asarray(beta)[:, None], h0=S, scale=scale)
    return o[:, 0], S_new


def kda_steps_pooled(q, k, v, log_alpha, beta, S_pool, state_indices=None, scale=1.0):
    """Decode over a state pool (Section 6.3, Eq. (1) applied Tq times per sequence).

    q, k, log_alpha: [N,Tq,H,dk]; v: [N,Tq,H,dv]; beta: [N,Tq,H]; S_pool: [P,H,dk,dv];
    state_indices: int [N] (negative = sequence skipped) or None for 0..N-1.
    Returns (o [N,Tq,H,dv], S_pool_new [P,H,dk,dv]) in float64; rows of o that belong to
    skipped sequences are NaN, so a test notices if it compares them.  S_pool is not modified.
    """
    q = np.asarray(q)
    N, Tq, H, dk = q.shape
    dv = np.asarray(v).shape[-1]
    idx = np.arange(N) if state_indices is None else np.asarray(state_indices).astype(np.int64)
    pool = np.array(S_pool, dtype=np.float64, copy=True)
    o = np.full((N, Tq, H, dv), np.nan)
    act = np.nonzero(idx >= 0)[0]
    if act.size:
        o_a, S_a = kda_forward(q[act], np.asarray(k)[act], np.asarray(v)[act], np.asarray(log_alpha)[act],
                               np.asarray(beta)[act], h0=pool[idx[act]], scale=scale)
        o[act] = o_a
        pool[idx[act]] = S_a
    return o, pool


def kda_backward(q, k, v, log_alpha, beta, do, dhT=None, h0=None, cu_seqlens=None, scale=1.0):
    """Gradients of sum(o * do) + sum(hT * dhT) with respect to the inputs of `kda_forward`
    (reverse-mode differentiation of Eq. (1), token by token, in float64).

    do: [B,T,H,dv]; dhT: [N,H,dk,dv] or None (zeros).  Returns a dict with dq, dk, dlog_alpha
    [B,T,H,dk], dv [B,T,H,dv], dbeta [B,T,H] and dh0 [N,H,dk,dv], float64.  Rows of `do` that
    belong to no sequence of a packed batch are ignored and their gradients are zero.
    """
    q = _f32(q)
    B, T, H, dk = q.shape
    k = _f32(k, (B, T, H, dk))
    log_alpha = _f32(log_alpha, (B, T, H, dk))
    v = _f32(v)
    dv = v.shape[-1]
    beta = _f32(beta, (B, T, H))
    cu = None
    if cu_seqlens is not None:
        cu = np.ascontiguousarray(np.asarray(cu_seqlens), dtype=np.int64)
        N = cu.shape[0] - 1
    else:
        N = B
    h0d = None if h0 is None else np.ascontiguousarray(np.asarray(h0), dtype=np.float64)
    if h0d is not None and h0d.shape != (N, H, dk, dv):
        raise ValueError("bad h0 shape %r" % (h0d.shape,))
    dod = np.ascontiguousarray(np.asarray(do), dtype=np.float64)
    if dod.shape != (B, T, H, dv):
        raise ValueError("bad do shape %r" % (dod.shape,))
    dhTd = None if dhT is None else np.ascontiguousarray(np.asarray(dhT), dtype=np.float64)
    if dhTd is not None and dhTd.shape != (N, H, dk, dv):
        raise ValueError("bad dhT shape %r" % (dhTd.shape,))
    out = {"dq": np.empty((B, T, H, dk)), "dk": np.empty((B, T, H, dk)),
           "dv": np.empty((B, T, H, dv)), "dlog_alpha": np.empty((B, T, H, dk)),
           "dbeta": np.empty((B, T, H)), "dh0": np.empty((N, H, dk, dv))}
    rc = _load().kda_oracle_backward(B, T, H, dk, dv, N, _ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha),
                                     _ptr(beta), _ptr(h0d), _ptr(cu), float(scale), _ptr(dod),
                                     _ptr(dhTd), _ptr(out["dq"]), _ptr(out["dk"]), _ptr(out["dv"]),
                                     _ptr(out["dlog_alpha"]), _ptr(out["dbeta"]), _ptr(out["dh0"]))
    if rc != 0:
        raise ValueError("kda_oracle_backward rejected the call (code %d)" % rc)
    return out
