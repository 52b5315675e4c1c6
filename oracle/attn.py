"""ctypes front end of the fp64 attention oracle (``attn_oracle.c``).

TEST INFRASTRUCTURE ONLY (see the package docstring).  The functions follow the
definition stated at the top of ``attn_oracle.c``: per-sample softmax attention
on a packed token stream (paper section 2.2.1 (1) and (2)), causal or prefix-LM
inside a sample, no attention across samples.
"""
import ctypes
import os

import numpy as np

from . import build as _build

MASK_CAUSAL = 0
MASK_PREFIX_BIDIR_SUFFIX = 1
MASK_PREFIX_CAUSAL_SUFFIX = 2
MASK_THREE_BLOCK = 3     # prefix_lens holds [num_seqs, 2]: the ends (P, P2) of the first two blocks
MASK_SLIDING_WINDOW = 4  # causal, row i sees the keys i - W + 1 .. i; prefix_lens holds W >= 1 per sample

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = ctypes.CDLL(path)
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _i32(a):
    if a is None:
        return None, None
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _mode(prefix_lens, mask_mode):
    if mask_mode is None:
        return MASK_CAUSAL if prefix_lens is None else MASK_PREFIX_BIDIR_SUFFIX
    return mask_mode


def attn_fwd(q, k, v, cu_seqlens, prefix_lens=None, scale=None, sel=None,
             mask_mode=None, nthreads=0):
    """q [T,Hq,D], k,v [T,Hkv,D] (values already rounded to the storage type).

    Returns (out [T,Hq,D] float64, lse [Hq,T] float64).  Rows of samples not in
    ``sel`` are NaN.
    """
    lib = _load()
    q, qp = _f32(q)
    k, kp = _f32(k)
    v, vp = _f32(v)
    cu, cup = _i32(cu_seqlens)
    pl, plp = _i32(prefix_lens)
    sl, slp = _i32(sel)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == (T, Hkv, D) and v.shape == (T, Hkv, D)
    n = len(cu) - 1
    assert cu[0] == 0 and cu[n] == T
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    out = np.full((T, Hq, D), np.nan, dtype=np.float64)
    lse = np.full((Hq, T), np.nan, dtype=np.float64)
    rc = lib.oracle_attn_fwd(qp, kp, vp, cup, plp, ctypes.c_int(_mode(pl, mask_mode)),
                             ctypes.c_int(n), ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(D),
                             ctypes.c_double(scale), slp, ctypes.c_int(0 if sl is None else len(sl)),
                             out.ctypes.data_as(ctypes.c_void_p), lse.ctypes.data_as(ctypes.c_void_p),
                             ctypes.c_int(nthreads))
    if rc != 0:
        raise ValueError(f"oracle_attn_fwd failed: {rc}")
    return out, lse


def attn_bwd(q, k, v, dout, cu_seqlens, prefix_lens=None, scale=None, sel=None,
             mask_mode=None, nthreads=0):
    """Returns (dq [T,Hq,D], dk [T,Hkv,D], dv [T,Hkv,D]) in float64; rows of
    samples not in ``sel`` are NaN."""
    lib = _load()
    q, qp = _f32(q)
    k, kp = _f32(k)
    v, vp = _f32(v)
    do, dop = _f32(dout)
    cu, cup = _i32(cu_seqlens)
    pl, plp = _i32(prefix_lens)
    sl, slp = _i32(sel)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    n = len(cu) - 1
    assert cu[0] == 0 and cu[n] == T and do.shape == q.shape
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    dq = np.full((T, Hq, D), np.nan, dtype=np.float64)
    dk = np.full((T, Hkv, D), np.nan, dtype=np.float64)
    dv = np.full((T, Hkv, D), np.nan, dtype=np.float64)
    rc = lib.oracle_attn_bwd(qp, kp, vp, dop, cup, plp, ctypes.c_int(_mode(pl, mask_mode)),
                             ctypes.c_int(n), ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(D),
                             ctypes.c_double(scale), slp, ctypes.c_int(0 if sl is None else len(sl)),
                             dq.ctypes.data_as(ctypes.c_void_p), dk.ctypes.data_as(ctypes.c_void_p),
                             dv.ctypes.data_as(ctypes.c_void_p), ctypes.c_int(nthreads))
    if rc != 0:
        raise ValueError(f"oracle_attn_bwd failed: {rc}")
    return dq, dk, dv


def attn_probs(q, k, v, dout, cu_seqlens, prefix_lens, s, h, scale=None, mask_mode=None):
    """Dense [L,L] probabilities p and score gradients dS of one (sample, head)."""
    lib = _load()
    q, qp = _f32(q)
    k, kp = _f32(k)
    v, vp = _f32(v)
    do, dop = _f32(dout)
    cu, cup = _i32(cu_seqlens)
    pl, plp = _i32(prefix_lens)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    L = int(cu[s + 1] - cu[s])
    p = np.zeros((L, L), dtype=np.float64)
    ds = np.zeros((L, L), dtype=np.float64)
    lib.oracle_attn_probs(qp, kp, vp, dop, cup, plp, ctypes.c_int(_mode(pl, mask_mode)),
                          ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(D), ctypes.c_double(scale),
                          ctypes.c_int(s), ctypes.c_int(h),
                          p.ctypes.data_as(ctypes.c_void_p), ds.ctypes.data_as(ctypes.c_void_p))
    return p, ds
