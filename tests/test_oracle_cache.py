"""Pins for the oracle's reduced-KV-cache bookkeeping (paper Section 3.2: rolling buffer for the
sink + window variant, fixed retention rule for the block-sparse variant; Section 4.1: one
retained block per `stride` blocks).  CPU only.

What fixes the behaviour independently of the append routine itself:
  * the set a decode step needs is row N-1 of the mask (the oracle's own predicate, pinned by the
    hand-written fixtures): after appending tokens 0..N-1 every live key must be retrievable
    from the slot the layout rule names, with its own bytes;
  * the token-granular case must reproduce the rolling buffer built by the slot map alone;
  * the result cannot depend on how the tokens were batched into append calls.
"""
import numpy as np
import pytest

from oracle import lg_oracle as O

CASES = [
    # N, sink, window, block, stride
    (1, 4, 8, 1, 0), (5, 4, 8, 1, 0), (12, 4, 8, 1, 0), (13, 4, 8, 1, 0), (100, 4, 8, 1, 0),
    (77, 0, 16, 1, 0), (300, 16, 128, 1, 0),
    (64, 16, 32, 16, 0), (65, 16, 32, 16, 0), (200, 16, 48, 16, 0), (207, 16, 48, 16, 0),
    (200, 16, 48, 16, 4), (207, 16, 48, 16, 4), (255, 16, 16, 16, 2), (256, 16, 16, 16, 2), (257, 16, 16, 16, 2),
    (500, 64, 192, 64, 8), (1000, 64, 128, 64, 3), (97, 4, 8, 1, 5), (300, 8, 24, 8, 1),
]


def tagged(N, heads=2, D=4):
    """Row p of head h holds the value 1000*h + p in every element."""
    a = np.zeros((1, heads, N, D), dtype=np.float32)
    a += np.arange(N, dtype=np.float32)[None, None, :, None]
    a += 1000.0 * np.arange(heads, dtype=np.float32)[None, :, None, None]
    return a


def append_all(rows, sink, window, block, stride, chunks, slots=None):
    N = rows.shape[2]
    slots = slots or O.cache_slots(N, sink, window, block, stride)
    cache = np.full((rows.shape[0], rows.shape[1], slots, rows.shape[3]), -1.0, dtype=rows.dtype)
    pos = 0
    for T in chunks:
        O.ring_append(rows[:, :, pos:pos + T], cache, pos, sink, window, block, stride)
        pos += T
    assert pos == N
    return cache


def chunking(N, seed):
    rng = np.random.default_rng(seed)
    out, left = [], N
    while left > 0:
        T = int(min(left, rng.integers(1, max(2, N // 2))))
        out.append(T)
        left -= T
    return out


@pytest.mark.parametrize("N,sink,window,block,stride", CASES)
def test_every_live_key_is_retrievable(N, sink, window, block, stride):
    rows = tagged(N)
    cache = append_all(rows, sink, window, block, stride, chunking(N, N + sink))
    t = N - 1
    live = O.mask(N, sink, window, block, stride)[t]
    for j in range(N):
        if not live[j]:
            continue
        if j < sink or j > t - window:
            s = O.ring_slot(j, sink, window)
        else:  # older than the window and not a sink token: only a retained strided block can hold it
            s = O.strided_slot(j, sink, window, block, stride)
            assert s >= 0, (j, "live key outside sink and window must be in a retained block")
        assert s < cache.shape[2]
        for h in range(rows.shape[1]):
            assert np.all(cache[0, h, s] == 1000.0 * h + j), (j, s, cache[0, h, s])


@pytest.mark.parametrize("N,sink,window", [(1, 4, 8), (7, 4, 8), (12, 4, 8), (40, 4, 8), (300, 16, 128), (50, 0, 7)])
def test_token_mode_is_the_rolling_buffer(N, sink, window):
    rows = tagged(N)
    want_k, _ = O.build_ring_cache(rows, rows, sink, window)   # slot map only, token by token
    got = append_all(rows, sink, window, 1, 0, chunking(N, 3 * N), slots=sink + window)
    valid = min(N, sink + window)
    # slots never written keep the fill value; the slot-map build leaves zeros there
    written = got[0, 0, :, 0] >= 0
    assert written.sum() == valid
    assert np.array_equal(got[:, :, written], want_k[:, :, written])


@pytest.mark.parametrize("N,sink,window,block,stride", CASES)
def test_result_does_not_depend_on_batching(N, sink, window, block, stride):
    rows = tagged(N, heads=1)
    one = append_all(rows, sink, window, block, stride, [N])
    single = append_all(rows, sink, window, block, stride, [1] * N)
    mixed = append_all(rows, sink, window, block, stride, chunking(N, 7 * N + 1))
    assert np.array_equal(one, single) and np.array_equal(one, mixed)


@pytest.mark.parametrize("n_max,sink,window,block,stride", CASES)
def test_cache_slots_is_tight(n_max, sink, window, block, stride):
    slots = O.cache_slots(n_max, sink, window, block, stride)
    top = max([O.strided_slot(p, sink, window, block, stride) for p in range(n_max)] + [sink + window - 1])
    b = max(block, 1)
    # a retained block is allocated whole, even if the context ends inside it
    assert top < slots
    if stride > 0 and slots > sink + window:
        assert slots - top <= b
    else:
        assert slots == sink + window


def test_paper_budget_block_sparse():
    # Section 4.1: 128K context, 64-token blocks, one retained block per 64 blocks -> 32 blocks = 2048 tokens
    assert O.cache_slots(131072, 0, 0, 64, 64) == 2048
    # attention-sink variant: 1 sink block + 32 local blocks = 2112 tokens, no growth with context
    assert O.cache_slots(131072, 64, 2048, 64, 0) == 2112 == O.cache_slots(10 ** 6, 64, 2048, 64, 0)
