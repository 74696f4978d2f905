"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching the HIP runtime."""
import ctypes
import os
import re

import pytest

import paper_2410_01485_amd as lg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = 0x1000  # a non-null, 16-byte aligned fake device pointer (never dereferenced on these paths)


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "longgen_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lg_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = lg.lib()
    names = declared_symbols()
    assert {"lg_sparse_attn_fwd", "lg_sparse_attn_bwd", "lg_sparse_attn_decode", "lg_status_str",
            "lg_debug_tile_map", "lg_sparse_attn_bwd_workspace_bytes",
            "lg_sparse_attn_decode_workspace_bytes"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_status_strings():
    assert lg.status_str(0) == "ok"
    for s in range(1, 6):
        assert lg.status_str(s) and lg.status_str(s) != lg.status_str(0)
    assert "unknown" in lg.status_str(99)


def fwd(q=P, k=P, v=P, out=P, lse=P, B=1, Hq=2, Hkv=1, N=64, D=64, sink=4, window=8, block=1, stride=0,
        dtype=lg.LG_BF16):
    return lg.lib().lg_sparse_attn_fwd(q, k, v, out, lse, B, Hq, Hkv, N, D, sink, window, block, stride,
                                       dtype, 0.0, None)


def test_fwd_argument_errors():
    assert fwd(q=None) == 1 and fwd(k=None) == 1 and fwd(v=None) == 1 and fwd(out=None) == 1
    assert fwd(B=0) == 2 and fwd(N=0) == 2 and fwd(Hq=0) == 2 and fwd(Hkv=0) == 2
    assert fwd(Hq=3, Hkv=2) == 2
    assert fwd(sink=-1) == 2 and fwd(window=0) == 2 and fwd(block=-1) == 2 and fwd(stride=-2) == 2
    assert fwd(block=8, sink=4, window=8) == 2      # sink not a multiple of block
    assert fwd(block=8, sink=8, window=12) == 2     # window not a multiple of block
    assert fwd(q=P + 4) == 2                        # misaligned
    assert fwd(D=96) == 3 and fwd(D=256) == 3 and fwd(dtype=7) == 3
    assert fwd(B=1 << 20, Hq=1 << 10, Hkv=1, N=1 << 20, D=128) == 2   # beyond 2^40 elements


def test_bwd_argument_errors():
    L = lg.lib()

    def bwd(ws=P, ws_bytes=1 << 30, q=P, dq=P, lse=P, D=64, window=8):
        return L.lg_sparse_attn_bwd(q, P, P, P, lse, P, dq, P, P, ws, ws_bytes, 1, 2, 1, 64, D, 4, window, 1, 0,
                                    lg.LG_BF16, 0.0, None)

    assert bwd(q=None) == 1 and bwd(dq=None) == 1 and bwd(lse=None) == 1
    assert bwd(window=0) == 2 and bwd(D=80) == 3
    need = lg.bwd_workspace_bytes(1, 2, 1, 64, 64, 4, 8, 1, 0, lg.LG_BF16)
    assert need >= 2 * 64 * 4
    assert bwd(ws=None) == 4 and bwd(ws_bytes=need - 1) == 4
    assert lg.bwd_workspace_bytes(1, 3, 2, 64, 64, 4, 8, 1, 0, lg.LG_BF16) == 0   # invalid -> 0


def test_varlen_argument_errors_and_workspace():
    """The packed, different-lengths calls validate the offsets and everything else before the first HIP call;
    a pack of empty sequences enqueues nothing and succeeds; the workspace is the largest any sequence needs."""
    L = lg.lib()

    def cu_arr(cu):
        return None if cu is None else (ctypes.c_int * len(cu))(*cu)

    def fwd_v(cu=(0, 100, 300), ns=None, q=P, lse=P, Hq=4, Hkv=2, D=128, window=8, block=1, sink=4, dtype=lg.LG_BF16):
        ns = (len(cu) - 1 if cu is not None else 1) if ns is None else ns
        return L.lg_sparse_attn_fwd_varlen(q, P, P, P, lse, cu_arr(cu), ns, Hq, Hkv, D, sink, window, block, 0,
                                           dtype, 0.0, None)

    def bwd_v(cu=(0, 100, 300), ws=P, ws_bytes=1 << 30, lse=P, dq=P, D=128):
        return L.lg_sparse_attn_bwd_varlen(P, P, P, P, lse, P, dq, P, P, ws, ws_bytes, cu_arr(cu), len(cu) - 1, 4, 2,
                                           D, 4, 8, 1, 0, lg.LG_BF16, 0.0, None)

    assert fwd_v(cu=None) == 1 and fwd_v(q=None) == 1
    assert fwd_v(ns=0) == 2 and fwd_v(cu=(1, 100)) == 2 and fwd_v(cu=(0, 100, 99)) == 2
    assert fwd_v(Hq=3) == 2 and fwd_v(window=0) == 2 and fwd_v(block=8, sink=4) == 2 and fwd_v(q=P + 4) == 2
    assert fwd_v(D=32) == 3 and fwd_v(dtype=7) == 3
    assert fwd_v(cu=(0, (1 << 30) + 1)) == 2                       # a sequence beyond 2^30 tokens
    assert fwd_v(cu=(0, 1 << 30, (1 << 31) - 1), Hq=32, Hkv=32) == 2   # Hq * T * D beyond 2^40 elements
    assert fwd_v(cu=(0, 0, 0, 0)) == 0 and fwd_v(cu=(0, 0), lse=None) == 0   # nothing to do: no HIP call made
    assert bwd_v(lse=None) == 1 and bwd_v(dq=P + 8) == 2 and bwd_v(D=48) == 3
    assert bwd_v(cu=(0, 5, 3)) == 2 and bwd_v(cu=(0, 0)) == 0
    need = lg.bwd_varlen_workspace_bytes([0, 100, 300, 300, 350], 4, 2, 128, 4, 8, 1, 0, lg.LG_BF16)
    assert need == max(lg.bwd_workspace_bytes(1, 4, 2, n, 128, 4, 8, 1, 0, lg.LG_BF16) for n in (100, 200, 50))
    assert bwd_v(ws_bytes=need - 1, cu=(0, 100, 300, 300, 350)) == 4 and bwd_v(ws=None, cu=(0, 100, 300)) == 4
    assert lg.bwd_varlen_workspace_bytes([0, 0], 4, 2, 128, 4, 8, 1, 0, lg.LG_BF16) == 256
    assert lg.bwd_varlen_workspace_bytes([0, 5, 3], 4, 2, 128, 4, 8, 1, 0, lg.LG_BF16) == 0
    assert lg.bwd_varlen_workspace_bytes([0, 5], 4, 2, 48, 4, 8, 1, 0, lg.LG_BF16) == 0
    with pytest.raises(ValueError):
        lg.bwd_varlen_workspace_bytes([0], 4, 2, 128, 4, 8, 1, 0, lg.LG_BF16)


def test_decode_argument_errors():
    L = lg.lib()

    def dec(q=P, ws=P, ws_bytes=1 << 30, B=2, Hq=4, Hkv=2, N=100, D=128, sink=4, window=28, block=1, stride=0):
        return L.lg_sparse_attn_decode(q, P, P, P, P, ws, ws_bytes, B, Hq, Hkv, N, D, sink, window, block,
                                       stride, lg.LG_BF16, 0.0, None)

    assert dec(q=None) == 1
    assert dec(N=0) == 2 and dec(window=0) == 2 and dec(Hq=3) == 2
    # a strided pattern needs the retained-block part of the cache: lg_sparse_attn_decode_cache
    assert dec(stride=4) == 3 and dec(block=4, sink=4, window=28, stride=2) == 3 and dec(D=32) == 3
    assert dec(Hq=64, Hkv=2) == 3                                        # group larger than 16
    need = lg.decode_workspace_bytes(1, 1, 1, 100000, 128, 64, 4096, lg.LG_BF16)
    assert need > 0
    assert L.lg_sparse_attn_decode(P, P, P, P, P, None, 0, 1, 1, 1, 100000, 128, 64, 4096, 1, 0,
                                   lg.LG_BF16, 0.0, None) == 4
    assert L.lg_sparse_attn_decode(P, P, P, P, P, P, need - 1, 1, 1, 1, 100000, 128, 64, 4096, 1, 0,
                                   lg.LG_BF16, 0.0, None) == 4


def test_python_binding_raises_lg_error():
    with pytest.raises(lg.LgError):
        lg.lg_debug_tile_map(0, 0, 1, 1, 0, lg.LG_BF16, 0)
