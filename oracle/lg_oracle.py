"""ctypes front end of the fp64 CPU oracle (lg_oracle.c).

TEST INFRASTRUCTURE, not product code: only tests/, __graft_entry__.smoke()
and bench.py's cpu_baseline leg may import this.  It shares nothing with the
HIP path.  Arrays in: numpy float32 (stored values, exactly widened from bf16
where the GPU side uses bf16).  Arrays out: numpy float64.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lg_oracle.c")
_LIB = os.path.join(_HERE, "liblg_oracle.so")
_lib = None


def build(force=False):
    """Compile lg_oracle.c with gcc (fp64, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        # LG_ORACLE_LIB: load this build of lg_oracle.c instead (the sanitizer test points it at a copy
        # compiled with -fsanitize=address,undefined)
        alt = os.environ.get("LG_ORACLE_LIB")
        if not alt:
            build()
        L = ctypes.CDLL(alt or _LIB)
        lng, dbl = ctypes.c_long, ctypes.c_double
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        L.lgo_live.argtypes = [lng] * 6
        L.lgo_live.restype = ctypes.c_int
        L.lgo_mask.argtypes = [ctypes.POINTER(ctypes.c_uint8)] + [lng] * 5
        L.lgo_mask.restype = None
        L.lgo_row_count.argtypes = [lng] * 5
        L.lgo_row_count.restype = lng
        L.lgo_ring_slot.argtypes = [lng] * 3
        L.lgo_ring_slot.restype = lng
        L.lgo_strided_slot.argtypes = [lng] * 5
        L.lgo_strided_slot.restype = lng
        L.lgo_cache_slots.argtypes = [lng] * 5
        L.lgo_cache_slots.restype = lng
        L.lgo_ring_append.argtypes = [ctypes.c_void_p, ctypes.c_void_p] + [lng] * 9
        L.lgo_ring_append.restype = None
        L.lgo_threads.argtypes = []
        L.lgo_threads.restype = ctypes.c_int
        L.lgo_fwd.argtypes = [fp, fp, fp, dp, dp] + [lng] * 9 + [dbl, lng, lng]
        L.lgo_fwd.restype = None
        L.lgo_bwd.argtypes = [fp, fp, fp, fp, dp, dp, dp, dp, dp] + [lng] * 9 + [dbl]
        L.lgo_bwd.restype = None
        L.lgo_bwd_part.argtypes = [fp, fp, fp, fp, dp, dp, dp, dp, dp] + [lng] * 9 + [dbl] + [lng] * 4
        L.lgo_bwd_part.restype = None
        L.lgo_decode.argtypes = [fp, fp, fp, dp, dp] + [lng] * 7 + [dbl]
        L.lgo_decode.restype = None
        _lib = L
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def threads():
    return int(_load().lgo_threads())


def live(i, j, sink, window, block=1, stride=0):
    return bool(_load().lgo_live(i, j, sink, window, block, stride))


def mask(N, sink, window, block=1, stride=0):
    """Dense [N,N] uint8 matrix of the predicate, row = query."""
    m = np.zeros((N, N), dtype=np.uint8)
    _load().lgo_mask(m.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), N, sink, window, block, stride)
    return m


def row_count(i, sink, window, block=1, stride=0):
    return int(_load().lgo_row_count(i, sink, window, block, stride))


def ring_slot(p, sink, window):
    return int(_load().lgo_ring_slot(p, sink, window))


def strided_slot(p, sink, window, block=1, stride=0):
    """Slot of token p in the retained-strided-blocks part of a cache row, or -1."""
    return int(_load().lgo_strided_slot(p, sink, window, block, stride))


def cache_slots(n_max, sink, window, block=1, stride=0):
    return int(_load().lgo_cache_slots(n_max, sink, window, block, stride))


def ring_append(rows_new, cache, pos, sink, window, block=1, stride=0):
    """Append rows_new [B,Hkv,T,D] (positions pos..pos+T-1) to cache [B,Hkv,slots,D] in place.
    Any dtype; bytes are copied."""
    rows_new = np.ascontiguousarray(rows_new)
    assert cache.flags["C_CONTIGUOUS"] and cache.dtype == rows_new.dtype
    B, H, T, D = rows_new.shape
    assert cache.shape[:2] == (B, H) and cache.shape[3] == D
    _load().lgo_ring_append(rows_new.ctypes.data, cache.ctypes.data, B * H, T, pos,
                            D * rows_new.dtype.itemsize, cache.shape[2], sink, window, block, stride)
    return cache


def _scale(scale, D):
    return float(scale) if scale is not None and scale > 0 else 1.0 / float(np.sqrt(D))


def fwd(q, k, v, sink, window, block=1, stride=0, scale=None, rows=None):
    """q [B,Hq,N,D], k,v [B,Hkv,N,D] float32 -> (out [B,Hq,N,D], lse [B,Hq,N]) float64.

    rows=(i0,i1) computes only those query rows (others are NaN)."""
    q, qp = _f32(q)
    k, kp = _f32(k)
    v, vp = _f32(v)
    B, Hq, N, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == (B, Hkv, N, D) and v.shape == k.shape and Hq % Hkv == 0
    out = np.full((B, Hq, N, D), np.nan, dtype=np.float64)
    lse = np.full((B, Hq, N), np.nan, dtype=np.float64)
    i0, i1 = (0, N) if rows is None else rows
    _load().lgo_fwd(qp, kp, vp, _dptr(out), _dptr(lse), B, Hq, Hkv, N, D,
                    sink, window, block, stride, _scale(scale, D), i0, i1)
    return out, lse


def bwd(q, k, v, dout, sink, window, block=1, stride=0, scale=None, rows=None, keys=None):
    """-> dict(dq, dk, dv, out, lse) float64; out/lse are the oracle's own forward.

    rows=(i0,i1) / keys=(j0,j1) restrict dq to those query rows and dk/dv to those keys (the
    rest is NaN); the forward is then only computed for the rows that are needed."""
    q, qp = _f32(q)
    k, kp = _f32(k)
    v, vp = _f32(v)
    dout, gp = _f32(dout)
    B, Hq, N, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == (B, Hkv, N, D) and v.shape == k.shape and dout.shape == q.shape
    dq = np.full((B, Hq, N, D), np.nan, dtype=np.float64)
    dk = np.full((B, Hkv, N, D), np.nan, dtype=np.float64)
    dv = np.full((B, Hkv, N, D), np.nan, dtype=np.float64)
    out = np.full((B, Hq, N, D), np.nan, dtype=np.float64)
    lse = np.full((B, Hq, N), np.nan, dtype=np.float64)
    i0, i1 = (0, N) if rows is None else rows
    j0, j1 = (0, N) if keys is None else keys
    _load().lgo_bwd_part(qp, kp, vp, gp, _dptr(dq), _dptr(dk), _dptr(dv), _dptr(out), _dptr(lse),
                         B, Hq, Hkv, N, D, sink, window, block, stride, _scale(scale, D), i0, i1, j0, j1)
    return dict(dq=dq, dk=dk, dv=dv, out=out, lse=lse)


def decode(q, k_cache, v_cache, N, sink, window, scale=None):
    """q [B,Hq,D], caches [B,Hkv,sink+window,D] float32 -> (out [B,Hq,D], lse [B,Hq]) float64."""
    q, qp = _f32(q)
    kc, kp = _f32(k_cache)
    vc, vp = _f32(v_cache)
    B, Hq, D = q.shape
    Hkv = kc.shape[1]
    assert kc.shape == (B, Hkv, sink + window, D) and vc.shape == kc.shape
    out = np.zeros((B, Hq, D), dtype=np.float64)
    lse = np.zeros((B, Hq), dtype=np.float64)
    _load().lgo_decode(qp, kp, vp, _dptr(out), _dptr(lse), B, Hq, Hkv, N, D, sink, window, _scale(scale, D))
    return out, lse


def build_ring_cache(k, v, sink, window):
    """Place the k/v rows of a full context [B,Hkv,N,D] into rolling-buffer caches
    [B,Hkv,sink+window,D] by the slot map, later tokens overwriting earlier ones."""
    k = np.asarray(k)
    v = np.asarray(v)
    B, H, N, D = k.shape
    C = sink + window
    kc = np.zeros((B, H, C, D), dtype=k.dtype)
    vc = np.zeros((B, H, C, D), dtype=v.dtype)
    for p in range(N):
        s = ring_slot(p, sink, window)
        kc[:, :, s] = k[:, :, p]
        vc[:, :, s] = v[:, :, p]
    return kc, vc
