"""The block-skipping tile scheduler, bit-exact against brute force over the oracle's predicate.

lg_debug_tile_map runs on the host the same source the kernels compile; the brute-force side
builds the dense mask with the oracle and reduces it per tile.  No GPU needed."""
import numpy as np
import pytest

import paper_2410_01485_amd as lg
from oracle import lg_oracle as O


def brute_tiles(mask, Tq, Tk, transposed):
    N = mask.shape[0]
    nq, nk = -(-N // Tq), -(-N // Tk)
    rows = []
    for a in range(nk if transposed else nq):
        row = []
        for c in range(nq if transposed else nk):
            u, t = (c, a) if transposed else (a, c)
            sub = mask[u * Tq:(u + 1) * Tq, t * Tk:(t + 1) * Tk]
            if sub.any():
                # FULL: every pair of the nominal Tq x Tk tile exists and is live
                full = bool(sub.all()) and sub.shape == (min(Tq, N - u * Tq), Tk)
                row.append((c, int(full)))
        rows.append(row)
    return rows


def check(N, sink, window, block, stride, dtype, transposed):
    tq, tk, rp, ci, kd = lg.lg_debug_tile_map(N, sink, window, block, stride, dtype, transposed)
    want = brute_tiles(O.mask(N, sink, window, block, stride), tq, tk, transposed)
    assert len(rp) == len(want) + 1
    got = [[(int(ci[x]), int(kd[x])) for x in range(rp[r], rp[r + 1])] for r in range(len(want))]
    assert got == want, (N, sink, window, block, stride, dtype, transposed)


CASES = [
    (1, 0, 1, 1, 0), (63, 0, 1, 1, 0), (64, 5, 7, 1, 0), (65, 16, 128, 1, 0), (200, 0, 64, 1, 0),
    (1024, 16, 128, 1, 0), (777, 64, 130, 1, 0), (513, 100, 1, 1, 0), (600, 700, 5, 1, 0),
    (600, 3, 900, 1, 0), (1000, 0, 300, 1, 3), (999, 7, 20, 1, 64), (1024, 64, 192, 64, 8),
    (1500, 64, 64, 64, 4), (1100, 48, 96, 48, 3), (900, 32, 32, 16, 5), (1111, 0, 8, 8, 1),
    (1000, 40, 120, 40, 2), (2048, 256, 512, 128, 4), (1300, 96, 192, 96, 7), (700, 0, 24, 24, 1000),
]


@pytest.mark.parametrize("dtype", [lg.LG_F32, lg.LG_BF16])
@pytest.mark.parametrize("transposed", [0, 1])
def test_tile_map_equals_brute_force(dtype, transposed):
    for c in CASES:
        check(*c, dtype, transposed)


def test_tile_map_randomised():
    rng = np.random.default_rng(7)
    for _ in range(60):
        b = int(rng.choice([1, 1, 2, 3, 16, 64, 100]))
        N = int(rng.integers(1, 1400))
        sink = int(rng.integers(0, 6)) * b * int(rng.choice([1, 3]))
        window = int(rng.integers(1, 12)) * b * int(rng.choice([1, 5]))
        stride = int(rng.choice([0, 0, 1, 2, 3, 8, 50]))
        for tr in (0, 1):
            check(N, sink, window, b, stride, int(rng.integers(0, 2)), tr)


def test_live_tile_totals_of_benchmark_configs():
    # config 2: 64-token blocks, tile = one block of keys: live key blocks per 64-row query block
    # summed over the rows of the bf16 kernel's query tiles
    tq, tk, rp, ci, kd = lg.lg_debug_tile_map(32768, 64, 192, 64, 8, lg.LG_BF16, 0)
    assert tk == 64
    # every live 64x64 block is covered by exactly one (query tile, key tile) pair per 64-row slice
    m_blocks = 0
    per_qtile = tq // 64
    nb = 32768 // 64
    live_blocks = set()
    for qb in range(nb):
        for kb in range(qb + 1):
            if kb < 1 or qb - kb < 3 or kb % 8 == 7:
                live_blocks.add((qb, kb))
    assert len(live_blocks) == 18044
    covered = set()
    for u in range(len(rp) - 1):
        for x in range(rp[u], rp[u + 1]):
            for s in range(per_qtile):
                covered.add((u * per_qtile + s, int(ci[x])))
    assert live_blocks <= covered
    # config 3: sink 64 + window 4096 at 128K: each query tile sees at most 1 sink + window + edge tiles
    tq, tk, rp, ci, kd = lg.lg_debug_tile_map(131072, 64, 4096, 1, 0, lg.LG_BF16, 0)
    per_row = np.diff(rp)
    assert per_row.max() <= 1 + (4096 + tq) // tk + 1
    assert int(per_row[-1]) == 1 + (4096 + tq - 1 + tk - 1) // tk


@pytest.mark.parametrize("N,sink,window,block,stride", CASES + [(5000, 64, 1000, 1, 0), (20000, 64, 4096, 1, 0),
                                                                (4000, 0, 64, 64, 4), (3000, 300, 100, 1, 0)])
@pytest.mark.parametrize("transposed", [0, 1])
def test_walk_order_visits_exactly_the_rows_tiles(N, sink, window, block, stride, transposed):
    # the kernels do not walk a row of the tile map in increasing order (rotated walks): whatever the
    # order, it must be a permutation of the row
    tq, tk, rp, ci, kd = lg.lg_debug_tile_map(N, sink, window, block, stride, lg.LG_BF16, transposed)
    for r in range(len(rp) - 1):
        order = lg.lg_debug_tile_walk(N, sink, window, block, stride, transposed, r)
        assert sorted(order.tolist()) == ci[rp[r]:rp[r + 1]].tolist(), (r, order[:8])


def test_rotated_walks_align_neighbours():
    # token pattern, steady state: at step x every query tile is at the key tile congruent to x modulo
    # its run length, so neighbouring query tiles are on the same key tile wherever their runs overlap
    N, sink, window = 40000, 64, 4096
    a = lg.lg_debug_tile_walk(N, sink, window, 1, 0, 0, 100)
    b = lg.lg_debug_tile_walk(N, sink, window, 1, 0, 0, 101)
    assert len(a) == len(b) == 69 and a[0] == 0 and b[0] == 0      # sink tile first, then the run of 68
    same = sum(int(x == y) for x, y in zip(a[1:], b[1:]))
    assert same == 64                                                # runs overlap in 64 of 68 tiles


# ------------------------------------------------------------------ register masks of PARTIAL tiles
def reg_offset(r, half):
    return 4 * half + 8 * (r // 4) + r % 4


BIT_CASES = [
    (300, 16, 128, 1, 0), (1000, 64, 192, 64, 8), (1000, 48, 96, 48, 3), (900, 0, 16, 16, 1), (777, 3, 10, 1, 7),
    (2000, 64, 1024, 64, 0), (1500, 32, 64, 32, 3), (600, 8, 24, 8, 5), (500, 4, 6, 2, 2), (640, 0, 192, 64, 64),
    (257, 100, 3, 1, 2), (4100, 64, 1024, 64, 8), (333, 0, 1, 1, 0), (400, 10, 30, 10, 4),
]


@pytest.mark.parametrize("N,sink,window,block,stride", BIT_CASES)
def test_partial_tile_register_masks_match_the_predicate(N, sink, window, block, stride):
    """The closed-form per-lane masks of the bf16 kernels (runs of register bits) against the oracle's
    predicate, bit for bit: every lane position of every 64-wide tile that can be PARTIAL, both orientations
    (lane = query row over a key tile; lane = key over a query-row tile), both halves of the wave."""
    mask = O.mask(N, sink, window, block, stride)
    rng = np.random.default_rng(N + 7 * block + stride)
    fixed_all = np.unique(np.concatenate([np.arange(min(N, 140)), rng.integers(0, N, 120), np.arange(max(0, N - 70), N)]))
    for transposed in (0, 1):
        for f in fixed_all:
            f = int(f)
            # tiles around the diagonal, the window edge, the sink, and a few others (ragged last tile included)
            tiles = {0, 64, (f // 64) * 64, max(0, ((f - window) // 64) * 64), max(0, ((f + window) // 64) * 64),
                     ((N - 1) // 64) * 64, int(rng.integers(0, N)) // 64 * 64, max(0, (f // 64) * 64 - 64)}
            for t0 in sorted(tiles):
                for half in (0, 1):
                    got = lg.lg_debug_partial_tile_bits(N, sink, window, block, stride, transposed, f, t0, half)
                    want = 0
                    for r in range(32):
                        x = t0 + reg_offset(r, half)
                        if x < N and (mask[x, f] if transposed else mask[f, x]):
                            want |= 1 << r
                    assert got == want, (transposed, f, t0, half, bin(got), bin(want))


def test_partial_tile_bits_argument_errors():
    with pytest.raises(lg.LgError):
        lg.lg_debug_partial_tile_bits(100, 0, 8, 1, 0, 0, 100, 0, 0)      # row outside the sequence
    with pytest.raises(lg.LgError):
        lg.lg_debug_partial_tile_bits(100, 0, 8, 1, 0, 0, 5, 0, 2)        # half is 0 or 1


def test_pattern_of_a_packed_sequence_equals_the_pattern_made_for_its_length():
    """The packed different-lengths forward makes one pattern for a length no sequence exceeds and derives each
    sequence's own on the device: the derived fields equal those made directly for the sequence's length, and both
    equal what the mask's definition says (sink, window and strided columns cut to the sequence: values beyond it
    change nothing)."""
    rng = np.random.default_rng(11)
    cases = [(1, 0, 1, 1, 0), (5, 64, 4096, 1, 0), (100, 64, 2048, 64, 64), (4096, 64, 2048, 64, 64), (4097, 64, 2048, 64, 64),
             (63 * 64, 64, 192, 64, 64), (63 * 64 + 1, 64, 192, 64, 64), (1000, 48, 96, 48, 3), (777, 3, 10, 1, 7), (6, 3, 10, 1, 7),
             (7, 3, 10, 1, 7), (130, 0, 16, 16, 1)]
    for _ in range(300):
        b = int(rng.choice([1, 1, 2, 16, 48, 64]))
        cases.append((int(rng.integers(1, 5000)), b * int(rng.integers(0, 6)), b * int(rng.integers(1, 40)), b,
                      int(rng.choice([0, 0, 1, 2, 3, 8, 64]))))
    for n, sink, window, block, stride in cases:
        direct = lg.lg_debug_pattern_fields(n, n, sink, window, block, stride)
        for made_for in (1 << 30, n + 1, 2 * n + 77):
            assert lg.lg_debug_pattern_fields(made_for, n, sink, window, block, stride) == direct, (n, sink, window, block, stride)
        b = max(block, 1)
        nb = -(-n // b)
        sb, wb = min(sink // b, nb), min(window // b, nb)
        st = stride if (stride > 0 and stride - 1 < nb) else 0
        log2 = lambda x: int(np.log2(x)) if x > 0 and (x & (x - 1)) == 0 else -1
        assert direct == [n, sb * b, wb * b, b, st, sb, wb, log2(b), st - 1 if st > 0 and log2(st) >= 0 else -1]
    with pytest.raises(lg.LgError):
        lg.lg_debug_pattern_fields(100, 101, 0, 8, 1, 0)
