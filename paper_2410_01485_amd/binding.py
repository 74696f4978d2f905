"""ctypes binding of liblonggen_attn.so: same names as the C ABI, argument marshalling only.

Tensors are torch tensors on a HIP device (contiguous, dense layouts of
include/longgen_attn.h); their data pointers and the current stream are handed to the
library.  Nothing here computes: a missing or unbuilt library is an error, never a fallback.
"""
import ctypes
import os

LG_F32, LG_BF16 = 0, 1
_HERE = os.path.dirname(os.path.abspath(__file__))
# LONGGEN_ATTN_LIB: path of another build of the same library (e.g. one with sanitized host code)
_LIB_PATH = os.environ.get("LONGGEN_ATTN_LIB") or os.path.join(_HERE, "liblonggen_attn.so")
_lib = None

_vp, _i, _f, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t


class LgError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, status_str(status), status))


def lib_path():
    return _LIB_PATH


def lib():
    """The loaded library; raises if it has not been built (python -m paper_2410_01485_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError("liblonggen_attn.so is not built: run `python -m paper_2410_01485_amd.build`")
        L = ctypes.CDLL(_LIB_PATH)
        L.lg_status_str.argtypes = [_i]
        L.lg_status_str.restype = ctypes.c_char_p
        L.lg_sparse_attn_fwd.argtypes = [_vp] * 5 + [_i] * 9 + [_i, _f, _vp]
        L.lg_sparse_attn_fwd.restype = _i
        L.lg_sparse_attn_bwd_workspace_bytes.argtypes = [_i] * 10
        L.lg_sparse_attn_bwd_workspace_bytes.restype = _sz
        L.lg_sparse_attn_bwd.argtypes = [_vp] * 9 + [_vp, _sz] + [_i] * 9 + [_i, _f, _vp]
        L.lg_sparse_attn_bwd.restype = _i
        L.lg_debug_bwd_kernel_ms.argtypes = [_vp] * 9 + [_vp, _sz] + [_i] * 9 + [_i, _f, _vp,
                                                                             ctypes.POINTER(_f)]
        L.lg_debug_bwd_kernel_ms.restype = _i
        _ip = ctypes.POINTER(_i)
        L.lg_sparse_attn_fwd_varlen.argtypes = [_vp] * 5 + [_ip] + [_i] * 8 + [_i, _f, _vp]
        L.lg_sparse_attn_fwd_varlen.restype = _i
        L.lg_sparse_attn_bwd_varlen_workspace_bytes.argtypes = [_ip] + [_i] * 9
        L.lg_sparse_attn_bwd_varlen_workspace_bytes.restype = _sz
        L.lg_sparse_attn_bwd_varlen.argtypes = [_vp] * 9 + [_vp, _sz] + [_ip] + [_i] * 8 + [_i, _f, _vp]
        L.lg_sparse_attn_bwd_varlen.restype = _i
        L.lg_sparse_attn_decode_workspace_bytes.argtypes = [_i] * 8
        L.lg_sparse_attn_decode_workspace_bytes.restype = _sz
        L.lg_sparse_attn_decode.argtypes = [_vp] * 5 + [_vp, _sz] + [_i] * 9 + [_i, _f, _vp]
        L.lg_sparse_attn_decode.restype = _i
        L.lg_kv_cache_slots.argtypes = [_i] * 5
        L.lg_kv_cache_slots.restype = _sz
        L.lg_kv_ring_append.argtypes = [_vp] * 4 + [_i] * 11 + [_vp]
        L.lg_kv_ring_append.restype = _i
        L.lg_sparse_attn_decode_cache_workspace_bytes.argtypes = [_i] * 10
        L.lg_sparse_attn_decode_cache_workspace_bytes.restype = _sz
        L.lg_sparse_attn_decode_cache.argtypes = [_vp] * 5 + [_vp, _sz] + [_i] * 10 + [_i, _f, _vp]
        L.lg_sparse_attn_decode_cache.restype = _i
        L.lg_sparse_attn_decode_cache_static.argtypes = [_vp] * 5 + [_i] * 10 + [_i, _f, _vp]
        L.lg_sparse_attn_decode_cache_static.restype = _i
        L.lg_sparse_attn_decode_paged_workspace_bytes.argtypes = [_i] * 10
        L.lg_sparse_attn_decode_paged_workspace_bytes.restype = _sz
        L.lg_sparse_attn_decode_paged.argtypes = [_vp] * 7 + [_vp, _sz] + [_i] * 12 + [_i, _f, _vp]
        L.lg_sparse_attn_decode_paged.restype = _i
        L.lg_kv_paged_append.argtypes = [_vp] * 6 + [_i] * 12 + [_i, _vp]
        L.lg_kv_paged_append.restype = _i
        L.lg_debug_decode_split_headdim_workspace_bytes.argtypes = [_i] * 4
        L.lg_debug_decode_split_headdim_workspace_bytes.restype = _sz
        L.lg_debug_decode_split_headdim.argtypes = [_vp] * 5 + [_vp, _sz] + [_i] * 7 + [_i, _f, _vp]
        L.lg_debug_decode_split_headdim.restype = _i
        L.lg_debug_decode_segments.argtypes = [_i] * 5 + [ctypes.POINTER(_i), _vp, _vp]
        L.lg_debug_decode_segments.restype = _i
        L.lg_debug_tile_walk.argtypes = [_i] * 7 + [_vp, _sz, ctypes.POINTER(_sz)]
        L.lg_debug_tile_walk.restype = _i
        L.lg_debug_partial_tile_bits.argtypes = [_i] * 9 + [ctypes.POINTER(ctypes.c_uint32)]
        L.lg_debug_partial_tile_bits.restype = _i
        L.lg_debug_pattern_fields.argtypes = [_i] * 6 + [ctypes.POINTER(ctypes.c_int32)]
        L.lg_debug_pattern_fields.restype = _i
        L.lg_debug_tile_map.argtypes = [_i] * 7 + [ctypes.POINTER(_i), ctypes.POINTER(_i), _vp, _sz,
                                                   _vp, _vp, _sz, ctypes.POINTER(_sz), ctypes.POINTER(_sz)]
        L.lg_debug_tile_map.restype = _i
        _lib = L
    return _lib


def status_str(status):
    return lib().lg_status_str(int(status)).decode()


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return LG_F32
    if t.dtype == torch.bfloat16:
        return LG_BF16
    raise TypeError("unsupported dtype %s" % t.dtype)


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream(t):
    import torch
    return torch.cuda.current_stream(t.device).cuda_stream


def _check(t, *shape, like=None, dtype=None):
    """t must be a contiguous device tensor of this shape; like / dtype: of that tensor's / that element type
    (the library reads every buffer of a call with the one dtype code it is given)."""
    if not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != tuple(shape):
        raise ValueError("expected a contiguous device tensor of shape %s, got %s" % (shape, tuple(t.shape)))
    want = like.dtype if like is not None else dtype
    if want is not None and t.dtype != want:
        raise TypeError("expected dtype %s, got %s" % (want, t.dtype))


def _check_lse(lse, *shape):
    import torch
    _check(lse, *shape, dtype=torch.float32)


def _ws_bytes(workspace):
    """Size of a workspace tensor (None: 0); it must live on the device."""
    if workspace is None:
        return 0
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise TypeError("the workspace must be a contiguous device tensor")
    return workspace.numel() * workspace.element_size()


def lg_sparse_attn_fwd(q, k, v, out, lse, sink, window, block=1, stride=0, scale=0.0):
    """out, lse <- sparse attention forward of q [B,Hq,N,D], k,v [B,Hkv,N,D]; lse may be None."""
    B, Hq, N, D = q.shape
    Hkv = k.shape[1]
    _check(q, B, Hq, N, D), _check(k, B, Hkv, N, D, like=q), _check(v, B, Hkv, N, D, like=q)
    _check(out, B, Hq, N, D, like=q)
    if lse is not None:
        _check_lse(lse, B, Hq, N)
    st = lib().lg_sparse_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), B, Hq, Hkv, N, D,
                                  sink, window, block, stride, _dtype_code(q), scale, _stream(q))
    if st != 0:
        raise LgError(st, "lg_sparse_attn_fwd")


def bwd_workspace_bytes(B, Hq, Hkv, N, D, sink, window, block, stride, dtype):
    return int(lib().lg_sparse_attn_bwd_workspace_bytes(B, Hq, Hkv, N, D, sink, window, block, stride, dtype))


def lg_sparse_attn_bwd(q, k, v, out, lse, dout, dq, dk, dv, workspace, sink, window, block=1, stride=0,
                       scale=0.0):
    """dq, dk, dv <- backward of lg_sparse_attn_fwd; workspace is a uint8 device tensor."""
    B, Hq, N, D = q.shape
    Hkv = k.shape[1]
    for t in (q, out, dout, dq):
        _check(t, B, Hq, N, D, like=q)
    for t in (k, v, dk, dv):
        _check(t, B, Hkv, N, D, like=q)
    _check_lse(lse, B, Hq, N)
    st = lib().lg_sparse_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(dout), _ptr(dq),
                                  _ptr(dk), _ptr(dv), _ptr(workspace), _ws_bytes(workspace),
                                  B, Hq, Hkv, N, D, sink, window, block, stride, _dtype_code(q), scale,
                                  _stream(q))
    if st != 0:
        raise LgError(st, "lg_sparse_attn_bwd")


def lg_debug_bwd_kernel_ms(q, k, v, out, lse, dout, dq, dk, dv, workspace, sink, window, block=1, stride=0,
                           scale=0.0):
    """lg_sparse_attn_bwd with per-kernel HIP-event timing: returns [delta_ms, dq_ms, dkdv_ms]."""
    B, Hq, N, D = q.shape
    Hkv = k.shape[1]
    ms = (_f * 3)()
    for t in (q, out, dout, dq):
        _check(t, B, Hq, N, D, like=q)
    for t in (k, v, dk, dv):
        _check(t, B, Hkv, N, D, like=q)
    _check_lse(lse, B, Hq, N)
    st = lib().lg_debug_bwd_kernel_ms(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(dout), _ptr(dq),
                                      _ptr(dk), _ptr(dv), _ptr(workspace), _ws_bytes(workspace),
                                      B, Hq, Hkv, N, D, sink, window, block, stride, _dtype_code(q), scale,
                                      _stream(q), ms)
    if st != 0:
        raise LgError(st, "lg_debug_bwd_kernel_ms")
    return [float(x) for x in ms]


def _cu_array(cu_seqlens):
    """The host array of offsets the *_varlen calls take: (ctypes int array, number of sequences)."""
    cu = [int(x) for x in cu_seqlens]
    if len(cu) < 2:
        raise ValueError("cu_seqlens needs at least two entries (one sequence)")
    return (_i * len(cu))(*cu), len(cu) - 1


def lg_sparse_attn_fwd_varlen(q, k, v, out, lse, cu_seqlens, sink, window, block=1, stride=0, scale=0.0):
    """Forward over packed sequences: q,out [Hq,T,D], k,v [Hkv,T,D], lse [Hq,T] or None; cu_seqlens is a host
    sequence of num_seqs + 1 offsets (0 first, T last)."""
    Hq, T, D = q.shape
    Hkv = k.shape[0]
    cu, ns = _cu_array(cu_seqlens)
    if cu[ns] != T:
        raise ValueError("cu_seqlens ends at %d, the tensors hold %d tokens" % (cu[ns], T))
    _check(q, Hq, T, D), _check(k, Hkv, T, D, like=q), _check(v, Hkv, T, D, like=q), _check(out, Hq, T, D, like=q)
    if lse is not None:
        _check_lse(lse, Hq, T)
    st = lib().lg_sparse_attn_fwd_varlen(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), cu, ns, Hq, Hkv, D,
                                         sink, window, block, stride, _dtype_code(q), scale, _stream(q))
    if st != 0:
        raise LgError(st, "lg_sparse_attn_fwd_varlen")


def bwd_varlen_workspace_bytes(cu_seqlens, Hq, Hkv, D, sink, window, block, stride, dtype):
    cu, ns = _cu_array(cu_seqlens)
    return int(lib().lg_sparse_attn_bwd_varlen_workspace_bytes(cu, ns, Hq, Hkv, D, sink, window, block, stride,
                                                               dtype))


def lg_sparse_attn_bwd_varlen(q, k, v, out, lse, dout, dq, dk, dv, workspace, cu_seqlens, sink, window, block=1,
                              stride=0, scale=0.0):
    """dq, dk, dv <- backward of lg_sparse_attn_fwd_varlen (same packed layout)."""
    Hq, T, D = q.shape
    Hkv = k.shape[0]
    cu, ns = _cu_array(cu_seqlens)
    if cu[ns] != T:
        raise ValueError("cu_seqlens ends at %d, the tensors hold %d tokens" % (cu[ns], T))
    for t in (q, out, dout, dq):
        _check(t, Hq, T, D, like=q)
    for t in (k, v, dk, dv):
        _check(t, Hkv, T, D, like=q)
    _check_lse(lse, Hq, T)
    st = lib().lg_sparse_attn_bwd_varlen(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(dout), _ptr(dq),
                                         _ptr(dk), _ptr(dv), _ptr(workspace), _ws_bytes(workspace), cu, ns,
                                         Hq, Hkv, D, sink, window, block, stride, _dtype_code(q), scale,
                                         _stream(q))
    if st != 0:
        raise LgError(st, "lg_sparse_attn_bwd_varlen")


def lg_debug_pattern_fields(n_made_for, n, sink, window, block=1, stride=0):
    """The 9 pattern fields the kernels hold for a sequence of n tokens, derived from the pattern made for
    n_made_for tokens (host-only)."""
    f = (ctypes.c_int32 * 9)()
    st = lib().lg_debug_pattern_fields(n_made_for, n, sink, window, block, stride, f)
    if st != 0:
        raise LgError(st, "lg_debug_pattern_fields")
    return [int(x) for x in f]


def decode_workspace_bytes(B, Hq, Hkv, N, D, sink, window, dtype):
    return int(lib().lg_sparse_attn_decode_workspace_bytes(B, Hq, Hkv, N, D, sink, window, dtype))


def lg_sparse_attn_decode(q, k_cache, v_cache, out, lse, workspace, N, sink, window, block=1, stride=0,
                          scale=0.0):
    """out, lse <- one-token attention of q [B,Hq,D] over caches [B,Hkv,sink+window,D]."""
    B, Hq, D = q.shape
    Hkv = k_cache.shape[1]
    _check(q, B, Hq, D), _check(k_cache, B, Hkv, sink + window, D, like=q)
    _check(v_cache, B, Hkv, sink + window, D, like=q), _check(out, B, Hq, D, like=q)
    if lse is not None:
        _check_lse(lse, B, Hq)
    st = lib().lg_sparse_attn_decode(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(out), _ptr(lse),
                                     _ptr(workspace), _ws_bytes(workspace),
                                     B, Hq, Hkv, N, D, sink, window, block, stride, _dtype_code(q), scale,
                                     _stream(q))
    if st != 0:
        raise LgError(st, "lg_sparse_attn_decode")


def lg_kv_cache_slots(n_max, sink, window, block=1, stride=0):
    """Slots per cache row for contexts of up to n_max tokens (0 if the arguments are invalid)."""
    return int(lib().lg_kv_cache_slots(n_max, sink, window, block, stride))


def lg_kv_ring_append(k_new, v_new, k_cache, v_cache, pos, sink, window, block=1, stride=0):
    """Store k_new, v_new [B,Hkv,T,D] (positions pos..pos+T-1) into caches [B,Hkv,slots,D] in place."""
    B, Hkv, T, D = k_new.shape
    slots = k_cache.shape[2]
    _check(v_new, B, Hkv, T, D), _check(k_new, B, Hkv, T, D)
    _check(k_cache, B, Hkv, slots, D), _check(v_cache, B, Hkv, slots, D)
    if k_cache.dtype != k_new.dtype or v_cache.dtype != k_new.dtype or v_new.dtype != k_new.dtype:
        raise TypeError("caches and new rows must share one dtype")
    st = lib().lg_kv_ring_append(_ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache), B, Hkv, D, T, pos, slots,
                                 sink, window, block, stride, _dtype_code(k_new), _stream(k_new))
    if st != 0:
        raise LgError(st, "lg_kv_ring_append")


def decode_cache_workspace_bytes(B, Hq, Hkv, N, D, sink, window, block, stride, dtype):
    return int(lib().lg_sparse_attn_decode_cache_workspace_bytes(B, Hq, Hkv, N, D, sink, window, block, stride,
                                                                 dtype))


def lg_sparse_attn_decode_cache(q, k_cache, v_cache, out, lse, workspace, N, sink, window, block=1, stride=0,
                                scale=0.0):
    """out, lse <- one-token attention of q [B,Hq,D] over caches [B,Hkv,slots,D] of any pattern."""
    B, Hq, D = q.shape
    Hkv, slots = k_cache.shape[1], k_cache.shape[2]
    _check(q, B, Hq, D), _check(k_cache, B, Hkv, slots, D, like=q), _check(v_cache, B, Hkv, slots, D, like=q)
    _check(out, B, Hq, D, like=q)
    if lse is not None:
        _check_lse(lse, B, Hq)
    st = lib().lg_sparse_attn_decode_cache(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(out), _ptr(lse),
                                           _ptr(workspace), _ws_bytes(workspace),
                                           B, Hq, Hkv, N, D, sink, window, block, stride, slots, _dtype_code(q),
                                           scale, _stream(q))
    if st != 0:
        raise LgError(st, "lg_sparse_attn_decode_cache")


def lg_sparse_attn_decode_cache_static(q, k_cache, v_cache, out, lse, N, sink, window, block=1, stride=0, scale=0.0):
    """lg_sparse_attn_decode_cache without a workspace argument: the library's built-in scratch array is used."""
    B, Hq, D = q.shape
    Hkv, slots = k_cache.shape[1], k_cache.shape[2]
    _check(q, B, Hq, D), _check(k_cache, B, Hkv, slots, D, like=q), _check(v_cache, B, Hkv, slots, D, like=q)
    _check(out, B, Hq, D, like=q)
    if lse is not None:
        _check_lse(lse, B, Hq)
    st = lib().lg_sparse_attn_decode_cache_static(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(out), _ptr(lse),
                                                  B, Hq, Hkv, N, D, sink, window, block, stride, slots,
                                                  _dtype_code(q), scale, _stream(q))
    if st != 0:
        raise LgError(st, "lg_sparse_attn_decode_cache_static")


def decode_paged_workspace_bytes(B, Hq, Hkv, n_max, D, sink, window, block, stride, dtype):
    return int(lib().lg_sparse_attn_decode_paged_workspace_bytes(B, Hq, Hkv, n_max, D, sink, window, block, stride,
                                                                 dtype))


def _check_i32(t, *shape):
    import torch
    if t.dtype != torch.int32:
        raise TypeError("expected an int32 tensor")
    _check(t, *shape)


def lg_sparse_attn_decode_paged(q, k_pages, v_pages, page_table, seq_lens, out, lse, workspace, n_max, sink, window,
                                block=1, stride=0, scale=0.0):
    """Decode over a paged cache: k_pages, v_pages [pages, Hkv, page_size, D]; page_table [B, pages_per_seq] and
    seq_lens [B] int32 on the device."""
    B, Hq, D = q.shape
    num_pages, Hkv, page_size = k_pages.shape[0], k_pages.shape[1], k_pages.shape[2]
    _check(q, B, Hq, D), _check(k_pages, num_pages, Hkv, page_size, D, like=q)
    _check(v_pages, num_pages, Hkv, page_size, D, like=q), _check(out, B, Hq, D, like=q)
    _check_i32(page_table, B, page_table.shape[1]), _check_i32(seq_lens, B)
    if lse is not None:
        _check_lse(lse, B, Hq)
    st = lib().lg_sparse_attn_decode_paged(_ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(page_table), _ptr(seq_lens),
                                           _ptr(out), _ptr(lse), _ptr(workspace), _ws_bytes(workspace),
                                           B, Hq, Hkv, n_max, D, sink, window, block, stride, page_size,
                                           page_table.shape[1], num_pages, _dtype_code(q), scale, _stream(q))
    if st != 0:
        raise LgError(st, "lg_sparse_attn_decode_paged")


def lg_kv_paged_append(k_new, v_new, k_pages, v_pages, page_table, positions, n_max, sink, window, block=1,
                       stride=0):
    """Store k_new, v_new [B,Hkv,T,D] (sequence b: positions[b] .. +T-1) into the paged caches in place."""
    B, Hkv, T, D = k_new.shape
    num_pages, page_size = k_pages.shape[0], k_pages.shape[2]
    _check(v_new, B, Hkv, T, D, like=k_new), _check(k_new, B, Hkv, T, D)
    _check(k_pages, num_pages, Hkv, page_size, D, like=k_new), _check(v_pages, num_pages, Hkv, page_size, D, like=k_new)
    _check_i32(page_table, B, page_table.shape[1]), _check_i32(positions, B)
    st = lib().lg_kv_paged_append(_ptr(k_new), _ptr(v_new), _ptr(k_pages), _ptr(v_pages), _ptr(page_table),
                                  _ptr(positions), B, Hkv, D, T, n_max, sink, window, block, stride, page_size,
                                  page_table.shape[1], num_pages, _dtype_code(k_new), _stream(k_new))
    if st != 0:
        raise LgError(st, "lg_kv_paged_append")


def lg_debug_decode_segments(N, sink, window, block=1, stride=0):
    """Host-only: [(first slot, length), ...] of the slot runs a decode step at context N reads."""
    import numpy as np
    n = _i(0)
    start = np.zeros(4, dtype=np.int32)
    length = np.zeros(4, dtype=np.int32)
    st = lib().lg_debug_decode_segments(N, sink, window, block, stride, ctypes.byref(n), start.ctypes.data,
                                        length.ctypes.data)
    if st != 0:
        raise LgError(st, "lg_debug_decode_segments")
    return [(int(start[x]), int(length[x])) for x in range(n.value)]


def lg_debug_tile_map(N, sink, window, block, stride, dtype, transposed):
    """Host-only: (tq, tk, row_ptr, col_idx, kind) numpy arrays of the scheduler's live tiles."""
    import numpy as np
    tq, tk = _i(0), _i(0)
    rows, need = _sz(0), _sz(0)
    st = lib().lg_debug_tile_map(N, sink, window, block, stride, dtype, transposed, ctypes.byref(tq),
                                 ctypes.byref(tk), None, 0, None, None, 0, ctypes.byref(rows), ctypes.byref(need))
    if st != 0:
        raise LgError(st, "lg_debug_tile_map")
    row_ptr = np.zeros(rows.value + 1, dtype=np.int32)
    col = np.zeros(max(need.value, 1), dtype=np.int32)
    kind = np.zeros(max(need.value, 1), dtype=np.uint8)
    st = lib().lg_debug_tile_map(N, sink, window, block, stride, dtype, transposed, ctypes.byref(tq),
                                 ctypes.byref(tk), row_ptr.ctypes.data, row_ptr.size, col.ctypes.data,
                                 kind.ctypes.data, need.value, ctypes.byref(rows), ctypes.byref(need))
    if st != 0:
        raise LgError(st, "lg_debug_tile_map")
    return tq.value, tk.value, row_ptr, col[:need.value], kind[:need.value]


def lg_debug_partial_tile_bits(N, sink, window, block, stride, transposed, fixed, tile0, half):
    """Host-only: the 32-bit register mask of a lane on a PARTIAL tile (see the header)."""
    bits = ctypes.c_uint32(0)
    st = lib().lg_debug_partial_tile_bits(N, sink, window, block, stride, transposed, fixed, tile0, half,
                                          ctypes.byref(bits))
    if st != 0:
        raise LgError(st, "lg_debug_partial_tile_bits")
    return int(bits.value)


def lg_debug_tile_walk(N, sink, window, block, stride, transposed, row):
    """Host-only: the order in which the bf16 kernels visit the live tiles of one row of the tile map."""
    import numpy as np
    cnt = _sz(0)
    st = lib().lg_debug_tile_walk(N, sink, window, block, stride, transposed, row, None, 0, ctypes.byref(cnt))
    if st != 0:
        raise LgError(st, "lg_debug_tile_walk")
    order = np.zeros(max(cnt.value, 1), dtype=np.int32)
    st = lib().lg_debug_tile_walk(N, sink, window, block, stride, transposed, row, order.ctypes.data, cnt.value,
                                  ctypes.byref(cnt))
    if st != 0:
        raise LgError(st, "lg_debug_tile_walk")
    return order[:cnt.value]


def lg_debug_decode_split_headdim(q, k_cache, v_cache, out, lse, N, sink, window, scale=0.0):
    """Measurement aid: decode with the work split over the head dimension (the paper's design)."""
    import torch
    B, Hq, D = q.shape
    Hkv = k_cache.shape[1]
    _check(q, B, Hq, D), _check(k_cache, B, Hkv, sink + window, D, like=q)
    _check(v_cache, B, Hkv, sink + window, D, like=q), _check(out, B, Hq, D, like=q)
    if lse is not None:
        _check_lse(lse, B, Hq)
    need = int(lib().lg_debug_decode_split_headdim_workspace_bytes(B, Hq, sink, window))
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    st = lib().lg_debug_decode_split_headdim(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(out), _ptr(lse), _ptr(ws),
                                             need, B, Hq, Hkv, N, D, sink, window, _dtype_code(q), scale, _stream(q))
    if st != 0:
        raise LgError(st, "lg_debug_decode_split_headdim")
    return ws
