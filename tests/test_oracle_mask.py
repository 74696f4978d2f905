"""Pins for the oracle's mask predicate, row counts and rolling-buffer slot map.

Nothing here calls the HIP path.  The predicate is checked against matrices written
out by hand (tests/golden), closed-form row counts, and the retained-token budgets
the paper states for its two settings (Section 4.1).
"""
import numpy as np
import pytest

from conftest import GOLDEN_MASKS, load_golden_mask
from oracle import lg_oracle as O


@pytest.mark.parametrize("name", GOLDEN_MASKS)
def test_mask_equals_hand_written_fixture(name):
    p, want = load_golden_mask(name)
    got = O.mask(p["N"], p["sink"], p["window"], p["block"], p["stride"])
    assert got.shape == want.shape
    assert np.array_equal(got, want)
    for i in range(p["N"]):
        assert O.row_count(i, p["sink"], p["window"], p["block"], p["stride"]) == int(want[i].sum())
        for j in range(p["N"]):
            assert O.live(i, j, p["sink"], p["window"], p["block"], p["stride"]) == bool(want[i, j])


def cnt_closed_form(i, sink, window):
    # window keys ending at i (clipped at 0) plus the sink keys that lie before the window
    return min(i + 1, window) + min(sink, max(0, i - window + 1))


@pytest.mark.parametrize("sink,window", [(0, 1), (0, 7), (3, 1), (16, 128), (5, 300), (64, 50)])
def test_token_row_counts_closed_form(sink, window):
    N = 257
    m = O.mask(N, sink, window)
    for i in range(N):
        assert int(m[i].sum()) == cnt_closed_form(i, sink, window)
        assert O.row_count(i, sink, window) == cnt_closed_form(i, sink, window)
    assert not np.triu(m, 1).any()          # causal
    assert np.all(np.diag(m) == 1)          # a query always sees itself


def test_live_pair_totals_of_the_benchmark_configs():
    # config 1: N=1024, sink=16, window=128
    assert int(O.mask(1024, 16, 128).sum()) == 137160
    assert sum(cnt_closed_form(i, 16, 128) for i in range(1024)) == 137160
    # configs 3/4: N=131072, sink=64, window=4096 (closed form; sampled rows by brute force)
    N, s, w = 131072, 64, 4096
    assert sum(cnt_closed_form(i, s, w) for i in range(N)) == 536608800
    for i in (0, 63, 64, 4095, 4096, 4159, 4160, 70000, N - 1):
        assert O.row_count(i, s, w) == cnt_closed_form(i, s, w)
    # config 2: N=32768, 64-token blocks, own + 2 preceding blocks, block 0, every 8th block
    nb = 32768 // 64
    blocks = 0
    for qb in range(nb):
        cols = {0} | {kb for kb in range(max(0, qb - 2), qb + 1)} | {kb for kb in range(qb + 1) if kb % 8 == 7}
        blocks += len(cols)
    assert blocks == 18044
    for i in (0, 63, 64, 1000, 4096 + 17, 32767):
        qb = i // 64
        cols = {0} | {kb for kb in range(max(0, qb - 2), qb + 1)} | {kb for kb in range(qb + 1) if kb % 8 == 7}
        want = sum(64 if kb < qb else (i % 64) + 1 for kb in cols)
        assert O.row_count(i, 64, 192, 64, 8) == want


def test_paper_retained_token_budgets():
    """Section 4.1: 64-token blocks; AttnSink keeps the first block and the 32 most recent
    blocks; BlockSparse keeps one block in every 64; both about 2K tokens at 128K."""
    N = 131072
    assert O.row_count(N - 1, 64, 32 * 64, 64, 0) == 64 + 32 * 64 == 2112
    assert O.row_count(N - 1, 0, 64, 64, 64) == (N // 64 // 64) * 64 == 2048
    # KV bytes of one sparse layer's reduced cache (bf16, 4096 = 32 heads * 128), 20 such layers,
    # plus 12 full layers at 128K: Section 4.3 quotes 26.5 GB.
    sparse = 20 * 2 * 2112 * 4096 * 2
    full = 12 * 2 * N * 4096 * 2
    assert abs((sparse + full) / 1e9 - 26.5) < 0.05


def test_block_mode_properties():
    N, b, sink, window, stride = 200, 8, 16, 24, 5
    m = O.mask(N, sink, window, b, stride)
    i = np.arange(N)[:, None]
    j = np.arange(N)[None, :]
    causal = j <= i
    assert not (m & ~causal).any()
    # own block and the two preceding blocks are live under the causal mask
    assert np.all(m[causal & (i // b - j // b < 3)] == 1)
    # a column's pattern depends on its block only (static, block-granular columns)
    for kb in range(N // b):
        col = m[(kb + 1) * b:, kb * b:(kb + 1) * b]
        assert np.all(col == col[:, :1])
    # strided columns stay live for every later query, non-strided non-sink ones die out
    for kb in range(N // b):
        last_row = m[N - 1, kb * b]
        always = kb < sink // b or kb % stride == stride - 1 or (N - 1) // b - kb < window // b
        assert bool(last_row) == always
    # stride == 1 keeps every block: plain causal attention
    assert np.array_equal(O.mask(50, 0, 4, 4, 1), np.tril(np.ones((50, 50), np.uint8)))
    # window >= N keeps everything
    assert np.array_equal(O.mask(50, 0, 64), np.tril(np.ones((50, 50), np.uint8)))


def test_ring_slot_map():
    # sink=2, window=3: tokens 0,1 pinned; 2,3,4 fill slots 2,3,4; then the window rolls
    assert [O.ring_slot(p, 2, 3) for p in range(9)] == [0, 1, 2, 3, 4, 2, 3, 4, 2]
    # after N tokens the cache holds exactly the keys live for the last row
    for name in GOLDEN_MASKS[:1]:
        p, want = load_golden_mask(name)
        for N in range(1, p["N"] + 1):
            held = {}
            for t in range(N):
                held[O.ring_slot(t, p["sink"], p["window"])] = t
            valid = min(N, p["sink"] + p["window"])
            assert sorted(held.keys()) == list(range(valid))
            assert sorted(held.values()) == [j for j in range(N) if want[N - 1, j]]
