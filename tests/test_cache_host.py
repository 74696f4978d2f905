"""Host logic of the reduced KV cache: the slot runs a decode step reads (the same source the
decode launch uses, exported as lg_debug_decode_segments) must name every live key of row N-1
exactly once.  The cache contents come from the oracle's append, the live set from the oracle's
predicate.  No GPU needed."""
import numpy as np
import pytest

import paper_2410_01485_amd as lg
from oracle import lg_oracle as O
from test_oracle_cache import CASES, append_all, tagged

MORE = [(4160, 64, 4096, 1, 0), (4161, 64, 4096, 1, 0), (9000, 64, 4096, 1, 0), (2112 + 64 * 5 + 3, 64, 2048, 64, 0),
        (64 * 64 * 3 + 17, 64, 2048, 64, 64), (1000, 0, 128, 64, 2), (640, 128, 128, 64, 1)]


@pytest.mark.parametrize("N,sink,window,block,stride", CASES + MORE)
def test_segments_name_the_live_set(N, sink, window, block, stride):
    rows = tagged(N, heads=1, D=1)
    cache = append_all(rows, sink, window, block, stride, [N])
    segs = lg.lg_debug_decode_segments(N, sink, window, block, stride)
    assert 1 <= len(segs) <= 4
    slots = [s for a, n in segs for s in range(a, a + n)]
    assert len(set(slots)) == len(slots), "a slot is read twice"
    assert max(slots) < lg.lg_kv_cache_slots(N, sink, window, block, stride)
    tags = sorted(int(cache[0, 0, s, 0]) for s in slots)
    live = [j for j in range(N) if O.mask(N, sink, window, block, stride)[N - 1, j]] if N <= 1200 else \
        [j for j in range(N) if O.live(N - 1, j, sink, window, block, stride)]
    assert tags == live
    assert len(slots) == O.row_count(N - 1, sink, window, block, stride)


@pytest.mark.parametrize("N,sink,window,block,stride", CASES + MORE)
def test_cache_slots_matches_oracle(N, sink, window, block, stride):
    for n in (1, N // 2 + 1, N, N + 1, 4 * N):
        assert lg.lg_kv_cache_slots(n, sink, window, block, stride) == O.cache_slots(n, sink, window, block, stride)


def test_cache_argument_checks():
    L = lg.lib()
    p = 4096  # a non-NULL, 16-byte aligned stand-in: every check below fails before any HIP call
    INVALID, NULL, UNSUP = 2, 1, 3
    ok_tail = (64, 192, 64, 8, lg.LG_BF16, None)
    assert L.lg_kv_ring_append(None, p, p, p, 1, 1, 128, 1, 0, 512, *ok_tail) == NULL
    assert L.lg_kv_ring_append(p, p, p, p, 1, 1, 128, 0, 0, 512, *ok_tail) == INVALID      # T < 1
    assert L.lg_kv_ring_append(p, p, p, p, 1, 1, 128, 1, -1, 512, *ok_tail) == INVALID     # pos < 0
    assert L.lg_kv_ring_append(p, p, p, p, 1, 1, 128, 600, 0, 256, *ok_tail) == INVALID    # row too short
    assert L.lg_kv_ring_append(p, p, p, p, 1, 1, 96, 1, 0, 512, *ok_tail) == UNSUP         # head dim
    assert L.lg_kv_ring_append(p, p, p, p, 1, 1, 128, 1, 0, 512, 60, 192, 64, 8, lg.LG_BF16, None) == INVALID
    assert L.lg_kv_ring_append(p, p, p + 8, p, 1, 1, 128, 1, 0, 512, *ok_tail) == INVALID  # alignment
    assert lg.lg_kv_cache_slots(1000, 60, 192, 64, 8) == 0
    # decode over the cache: capacity below what the context needs, strided pattern through the
    # fixed-size entry point
    assert L.lg_sparse_attn_decode_cache(p, p, p, p, None, None, 0, 1, 1, 1, 100000, 128, 64, 192, 64, 8, 300,
                                         lg.LG_BF16, 0.0, None) == INVALID
    assert L.lg_sparse_attn_decode(p, p, p, p, None, None, 0, 1, 1, 1, 1000, 128, 64, 192, 64, 8,
                                   lg.LG_BF16, 0.0, None) == UNSUP


def test_paged_argument_checks():
    L = lg.lib()
    p = 4096
    INVALID, NULL = 2, 1
    # q, k_pages, v_pages, page_table, seq_lens, out, lse, ws, ws_bytes, B, Hq, Hkv, n_max, D, sink, window, block,
    # stride, page_size, pages_per_seq, num_pages, dtype, scale, stream
    def dec(page_size=64, pps=8, num_pages=100, table=p, **kw):
        a = dict(n_max=400, sink=64, window=192, block=64, stride=8)
        a.update(kw)
        return L.lg_sparse_attn_decode_paged(p, p, p, table, p, p, None, None, 0, 2, 4, 2, a["n_max"], 128, a["sink"],
                                             a["window"], a["block"], a["stride"], page_size, pps, num_pages,
                                             lg.LG_BF16, 0.0, None)
    assert dec(table=None) == NULL
    assert dec(page_size=48) == INVALID and dec(page_size=8) == INVALID and dec(page_size=8192) == INVALID
    assert dec(pps=3) == INVALID            # 3 pages of 64 slots cannot hold 64 + 192 + 0 slots
    assert dec(n_max=100000, pps=8) == INVALID
    assert dec(num_pages=0) == INVALID
    assert L.lg_kv_paged_append(p, p, p, p, p, p, 2, 2, 128, 0, 400, 64, 192, 64, 8, 64, 8, 100, lg.LG_BF16,
                                None) == INVALID   # T < 1
    assert L.lg_kv_paged_append(p, p, p, p, None, p, 2, 2, 128, 1, 400, 64, 192, 64, 8, 64, 8, 100, lg.LG_BF16,
                                None) == NULL
