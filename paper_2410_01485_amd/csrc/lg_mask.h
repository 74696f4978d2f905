// lg_mask.h — the sparse-attention mask predicate and the block-skipping tile
// scheduler, as integer-only functions compiled for both host and device.
//
// Paper Section 3.1 ("Different KV-Reduced Attention Strategies") defines the
// patterns: sink tokens, local window blocks, strided block columns; Section 3.2
// says the kernel skips key blocks whose mask is zero and keeps the mask in
// compressed-sparse-row form.  Because the mask is static and identical for every
// head, the row lists are produced here in closed form instead of being stored:
// lg_next_ktile walks the live key tiles of a query tile in increasing order, and
// lg_qtile_range gives the (contiguous) live query tiles of a key tile.  The host
// entry point lg_debug_tile_map materialises the same lists as CSR for checking.
//
// Divisions by the block size and remainders by the stride run once per tile inside
// the kernels' main loops, so power-of-two values (the usual case: 64-token blocks,
// strides 8 or 64) take a shift / mask path; other values fall back to division.
#ifndef LG_MASK_H_
#define LG_MASK_H_

#include <stdint.h>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define LG_HD __host__ __device__ __forceinline__
#else
#define LG_HD inline
#endif

struct LgMask {
  int N;       // sequence length (queries = keys)
  int ld;      // rows from one head to the next in the caller's tensors: N in the batch layout, the
               // total number of tokens when sequences of different lengths are packed per head
  int sink;    // tokens
  int window;  // tokens
  int b;       // max(block, 1): pattern granularity in tokens
  int stride;  // in blocks; 0 = no strided columns
  int sb;      // sink / b
  int wb;      // window / b
  int bshift;  // log2(b) when b is a power of two, else -1
  int smask;   // stride - 1 when stride is a power of two, else -1
};

LG_HD int lg_log2_exact(int x) {
  for (int s = 0; s < 31; ++s)
    if ((1 << s) == x) return s;
  return -1;
}

LG_HD LgMask lg_make_mask(int N, int sink, int window, int block, int stride) {
  LgMask m;
  m.N = N;
  m.ld = N;
  m.b = block > 1 ? block : 1;
  // Values beyond the sequence change nothing; clamping them keeps every product
  // below in int range.
  const int nb = (N + m.b - 1) / m.b;  // number of blocks
  m.sb = sink / m.b < nb ? sink / m.b : nb;
  m.wb = window / m.b < nb ? window / m.b : nb;
  m.sink = m.sb * m.b;
  m.window = m.wb * m.b;
  m.stride = (stride > 0 && stride - 1 < nb) ? stride : 0;
  m.bshift = lg_log2_exact(m.b);
  m.smask = (m.stride > 0 && lg_log2_exact(m.stride) >= 0) ? m.stride - 1 : -1;
  return m;
}

// x / b for x >= 0
LG_HD int lg_div_b(const LgMask& m, int x) { return m.bshift >= 0 ? (x >> m.bshift) : x / m.b; }

// The pattern of a sequence of n tokens that shares sink, window, block and stride with t, a mask made
// by lg_make_mask for a length that no sequence exceeds: the same fields lg_make_mask(n, ...) gives
// (it clamps sink, window and stride to the length), ld kept.
LG_HD LgMask lg_mask_for_length(const LgMask& t, int n) {
  LgMask m = t;
  m.N = n;
  const int nb = lg_div_b(t, n + t.b - 1);
  m.sb = t.sb < nb ? t.sb : nb;
  m.wb = t.wb < nb ? t.wb : nb;
  m.sink = m.sb * t.b;
  m.window = m.wb * t.b;
  if (!(t.stride > 0 && t.stride - 1 < nb)) {
    m.stride = 0;
    m.smask = -1;
  }
  return m;
}

// Is block column kb one of the strided columns (kb % stride == stride - 1)?  stride > 0.
LG_HD bool lg_strided(const LgMask& m, int kb) {
  return m.smask >= 0 ? ((kb & m.smask) == m.smask) : (kb % m.stride == m.stride - 1);
}

// First strided block index >= kb (stride > 0).
LG_HD int lg_next_strided_block(const LgMask& m, int kb) {
  return m.smask >= 0 ? (kb | m.smask) : kb + (m.stride - 1 - kb % m.stride);
}

// live(i, j): may query i attend to key j?
LG_HD bool lg_live(const LgMask& m, int i, int j) {
  if (j > i) return false;
  if (m.b == 1 && m.stride == 0) return j < m.sink || i - j < m.window;
  const int qb = lg_div_b(m, i), kb = lg_div_b(m, j);
  if (kb < m.sb || qb - kb < m.wb) return true;
  return m.stride > 0 && lg_strided(m, kb);
}

enum { LG_TILE_DEAD = 0, LG_TILE_PARTIAL = 1, LG_TILE_FULL = 2 };

// Classify the tile of query rows [q0, q1] x keys [k0, k1] (inclusive bounds).
// q0 <= q1 < N and k0 < N are required; k1 may run past N-1 (ragged last tile),
// which makes the tile at most PARTIAL.  FULL: every pair is live.  DEAD: none is.
LG_HD int lg_tile_kind(const LgMask& m, int q0, int q1, int k0, int k1) {
  if (k0 > q1) return LG_TILE_DEAD;
  const int je = k1 < q1 ? k1 : q1;  // largest key any row of the tile can see
  bool live = k0 < m.sink;
  if (!live) {
    const int istar = q0 > je ? q0 : je;  // earliest row that sees key je
    live = lg_div_b(m, istar) - lg_div_b(m, je) < m.wb;
  }
  if (!live && m.stride > 0) live = lg_next_strided_block(m, lg_div_b(m, k0)) <= lg_div_b(m, je);
  if (!live) return LG_TILE_DEAD;
  if (k1 > q0) return LG_TILE_PARTIAL;  // crosses the diagonal (or runs past N-1)
  if (m.stride == 1) return LG_TILE_FULL;
  // smallest key of the tile that is neither sink nor strided must still be inside
  // the window of the last row
  int j = k0;
  for (int it = 0; it < 4 && j <= k1; ++it) {
    const int kb = lg_div_b(m, j);
    if (kb < m.sb) j = m.sink;
    else if (m.stride > 0 && lg_strided(m, kb)) j = (kb + 1) * m.b;
    else break;
  }
  if (j > k1) return LG_TILE_FULL;
  return (lg_div_b(m, q1) - lg_div_b(m, j) < m.wb) ? LG_TILE_FULL : LG_TILE_PARTIAL;
}

// Next live key tile (tile = keys [t*Tk, t*Tk+Tk-1]) after tile `prev` for the query
// rows [q0, q1]; pass prev = -1 to get the first.  Returns -1 when there is none.
// Tk must be a power of two.
LG_HD int lg_next_ktile(const LgMask& m, int q0, int q1, int Tk, int prev) {
  const int t0 = prev + 1;
  const int j0 = t0 * Tk;
  if (j0 > q1) return -1;
  if (j0 < m.sink) return t0;
  // window: live keys of the row range are [jw, q1]
  int jw = (lg_div_b(m, q0) - m.wb + 1) * m.b;
  if (jw < 0) jw = 0;
  int t = (int)((unsigned)jw / (unsigned)Tk);
  if (t < t0) t = t0;
  if (m.stride > 0) {
    const int kb0 = lg_div_b(m, j0);
    const int f = lg_next_strided_block(m, kb0);
    const int ts = (f == kb0) ? t0 : (int)(((unsigned long long)f * (unsigned)m.b) / (unsigned)Tk);
    if (ts < t) t = ts;
  }
  return ((long long)t * Tk <= q1) ? t : -1;
}

// ---------------------------------------------------------------------------------
// Per-query-tile schedule for the kernels' main loops: the same live key tiles and the
// same FULL / PARTIAL classes as lg_next_ktile / lg_tile_kind, but with everything that
// depends only on the query tile computed once, so that one step costs a handful of
// scalar operations.  Key tiles are Tk = 64 keys.
struct LgQSched {
  int tmax;   // last causal key tile: q1 / 64
  int tS;     // key tiles [0, tS) hold sink keys
  int tW;     // first key tile that reaches into the window of some row
  int jfull;  // keys >= jfull are inside the window of every row of the query tile
  int q0;
};

LG_HD LgQSched lg_qsched_init(const LgMask& m, int q0, int q1) {
  LgQSched s;
  s.q0 = q0;
  s.tmax = q1 >> 6;
  s.tS = (m.sink + 63) >> 6;
  int jw = (lg_div_b(m, q0) - m.wb + 1) * m.b;
  s.tW = jw > 0 ? (jw >> 6) : 0;
  const int jf = (lg_div_b(m, q1) - m.wb + 1) * m.b;
  s.jfull = jf > 0 ? jf : 0;
  return s;
}

// Next live key tile after `prev` (-1 for the first), or -1.
LG_HD int lg_qsched_next(const LgMask& m, const LgQSched& s, int prev) {
  int t = prev + 1;
  if (t >= s.tS && t < s.tW) {  // in the gap between the sink tiles and the window tiles
    int ts = s.tW;
    if (m.stride > 0) {
      const int kb0 = lg_div_b(m, t << 6);
      const int f = lg_next_strided_block(m, kb0);
      const int tf = (f == kb0) ? t : (int)(((unsigned long long)f * (unsigned)m.b) >> 6);
      ts = tf < ts ? tf : ts;
    }
    t = ts;
  }
  return t <= s.tmax ? t : -1;
}

// Is live key tile t FULL (every pair live, nothing to mask)?
LG_HD bool lg_qsched_full(const LgMask& m, const LgQSched& s, int t) {
  const int k0 = t << 6, k1 = k0 + 63;
  if (k1 > s.q0) return false;                       // crosses the diagonal or the end
  if (k0 >= s.jfull || k1 < m.sink || s.jfull <= m.sink) return true;
  if (m.stride == 0) return false;
  if (m.stride == 1) return true;
  // the keys below jfull that are not sink keys must all lie in one strided block
  const int lo = k0 > m.sink ? k0 : m.sink;
  const int hi = k1 < s.jfull - 1 ? k1 : s.jfull - 1;
  const int kb = lg_div_b(m, lo);
  return kb == lg_div_b(m, hi) && lg_strided(m, kb);
}

// Walk order for patterns without strided columns (the live key tiles of a query tile are then
// the sink tiles plus ONE contiguous run [tws, tmax]).  The online softmax takes tiles in any
// order, so the run is walked rotated: at step x every query tile is at the key tile of its run
// that is congruent to x modulo the run length.  Query tiles that are computed side by side
// (neighbours, whose runs overlap almost completely) therefore read the SAME key tile at the
// same time and share it in L2, instead of trailing each other by a few tiles.
struct LgQWalk {
  int nsink;   // sink tiles [0, nsink) come first
  int tws;     // first tile of the window run
  int tmax;    // last tile of the window run
  int tstart;  // where the rotated walk of the run starts (-1: the run is empty)
};

LG_HD LgQWalk lg_qwalk_init(const LgQSched& s) {
  LgQWalk w;
  w.tmax = s.tmax;
  w.nsink = s.tS < s.tmax + 1 ? s.tS : s.tmax + 1;
  w.tws = s.tS > s.tW ? s.tS : s.tW;
  const int len = w.tmax - w.tws + 1;
  w.tstart = len > 0 ? w.tws + (len - w.tws % len) % len : -1;
  return w;
}

LG_HD int lg_qwalk_first(const LgQWalk& w) { return w.nsink > 0 ? 0 : w.tstart; }

// Tile after t in the walk, or -1.
LG_HD int lg_qwalk_next(const LgQWalk& w, int t) {
  if (t < w.nsink) return t + 1 < w.nsink ? t + 1 : w.tstart;
  const int n = t == w.tmax ? w.tws : t + 1;
  return n == w.tstart ? -1 : n;
}

// Live query tiles (tile = rows [u*Tq, u*Tq+Tq-1]) of the keys [k0, k1] (k1 <= N-1):
// always one contiguous range [*lo, *hi].
LG_HD void lg_qtile_range(const LgMask& m, int k0, int k1, int Tq, int* lo, int* hi) {
  *lo = k0 / Tq;
  bool always = k0 < m.sink;
  if (!always && m.stride > 0) always = lg_next_strided_block(m, lg_div_b(m, k0)) <= lg_div_b(m, k1);
  long long last = m.N - 1;
  if (!always) {
    const long long w = ((long long)lg_div_b(m, k1) + m.wb) * m.b - 1;  // last row whose window holds k1
    if (w < last) last = w;
  }
  *hi = (int)(last / Tq);
}

// ---------------------------------------------------------------------------------
// Register masks of PARTIAL tiles (bf16 matrix-core kernels).  A lane of a wave holds, of a 64 x 32 (or
// 32 x 64) block of pairs, ONE column and 32 of its entries in two stacked 32 x 32 accumulators: register
// r = 0..31 of lane-half g is the entry at offset 4 g + c(r), c(r) = 8 (r / 4) + r % 4, along the other axis.
// c grows with r, so the entries whose offset lies in [lo, hi) are a run of register bits, and every pattern
// of the predicate decomposes into a few such runs: no per-element evaluation is needed.
// lg_regs_below(x) = number of registers with c(r) < x.
LG_HD int lg_regs_below(int x) {
  x = x < 0 ? 0 : (x > 64 ? 64 : x);
  const int rem = x & 7;
  return 4 * (x >> 3) + (rem < 4 ? rem : 4);
}
LG_HD uint32_t lg_reg_run(int lo, int hi) {
  const int a = lg_regs_below(lo), b = lg_regs_below(hi);
  const uint32_t ma = a >= 32 ? ~0u : (1u << a) - 1u, mb = b >= 32 ? ~0u : (1u << b) - 1u;
  return mb & ~ma;
}
LG_HD int lg_clamp_off(int x) { return x < -1 ? -1 : (x > 64 ? 64 : x); }

// (All of the following is 32-bit arithmetic: the entry points accept sequences of up to 2^30 tokens.)
// Forward / dq layout: the lane owns query row i, register r is key k0 + 4 g + c(r) of the 64-key tile at
// k0.  Bit r of the result: live(i, that key).  The live keys of a row are its window run (keys from the
// first key of block qb - wb + 1 up to i), the sink run (keys below `sink`), and the strided blocks.
LG_HD uint32_t lg_key_bits(const LgMask& m, int i, int k0, int g) {
  const int off = k0 + 4 * g;
  const int hi = lg_clamp_off(i - off + 1);      // causal: offsets below hi
  if (m.stride == 1) return lg_reg_run(-1, hi);  // every block is a strided column
  const int jw = (lg_div_b(m, i) - m.wb + 1) * m.b;
  uint32_t w = lg_reg_run(lg_clamp_off(jw - off), hi);
  if (k0 < m.sink) {
    const int se = lg_clamp_off(m.sink - off);
    w |= lg_reg_run(-1, se < hi ? se : hi);
  }
  if (m.stride > 0) {
    const int kb1 = lg_div_b(m, k0 + 63);
    for (int kb = lg_next_strided_block(m, lg_div_b(m, k0)); kb <= kb1; kb += m.stride) {
      const int s = kb * m.b - off;
      const int e = lg_clamp_off(s + m.b);
      w |= lg_reg_run(lg_clamp_off(s), e < hi ? e : hi);
    }
  }
  return w;
}

// dk/dv layout: the lane owns key j, register r is query row q0 + 4 g + c(r) of the 64-row tile at q0.
// Bit r: that row exists (below N) and live(row, j).  The rows that see a key are ONE run: from j to the
// last row of block kb + wb - 1, or to the end of the sequence for a sink or strided-column key.
LG_HD uint32_t lg_row_bits(const LgMask& m, int j, int q0, int g) {
  const int off = q0 + 4 * g;
  const int kb = lg_div_b(m, j);
  const int nb = lg_div_b(m, m.N - 1) + 1;  // blocks of the sequence
  const bool column = j < m.sink || (m.stride > 0 && lg_strided(m, kb));
  const int qe = kb + m.wb;                 // first block whose rows no longer see the key through the window
  const int end = (column || qe >= nb) ? m.N : qe * m.b;
  return lg_reg_run(lg_clamp_off(j - off), lg_clamp_off(end - off));
}

// ---------------------------------------------------------------------------------
// Reduced KV cache (paper Section 3.2: fixed cache management; Section 4.1: the block-sparse
// variant retains one block per `stride` blocks).  A cache row is
//     [ sink tokens | rolling window of `window` tokens | retained strided blocks ]
// token p sits in slot p (p < sink) or sink + (p - sink) % window, and, when its block
// kb = p / b is a strided column, also in slot sink + window + (kb / stride) * b + p % b.
//
// The keys of a decode step (query = token N-1) are then up to four runs of consecutive
// slots: the sink tokens, the live part of the rolling window (one or two runs: the ring
// wraps, and in block mode the tail of the block that just left the window is still in the
// ring but dead), and the retained blocks older than the window.  Every live key is in
// exactly one run.
struct LgDecSegs {
  int n;         // runs in use
  int start[4];  // first slot of a run
  int pre[5];    // keys before a run; pre[n] = all keys of the step
};

LG_HD void lg_decsegs_push(LgDecSegs& g, int start, int len) {
  if (len <= 0) return;
  if (g.n > 0 && g.start[g.n - 1] + (g.pre[g.n] - g.pre[g.n - 1]) == start) {  // continues the previous run
    g.pre[g.n] += len;
    return;
  }
  g.start[g.n] = start;
  g.pre[g.n + 1] = g.pre[g.n] + len;
  ++g.n;
}

// The pattern for cache geometry: like lg_make_mask but sink and window keep their given
// values (the slot layout depends on them, not on the current context length N).
LG_HD LgMask lg_make_cache_mask(int N, int sink, int window, int block, int stride) {
  LgMask m;
  m.N = N;
  m.ld = N;
  m.b = block > 1 ? block : 1;
  m.sb = sink / m.b;
  m.wb = window / m.b;
  m.sink = m.sb * m.b;
  m.window = m.wb * m.b;
  m.stride = stride > 0 ? stride : 0;
  m.bshift = lg_log2_exact(m.b);
  m.smask = (m.stride > 0 && lg_log2_exact(m.stride) >= 0) ? m.stride - 1 : -1;
  return m;
}

// m: from lg_make_cache_mask, m.N = context length (>= 1), m.window >= 1.
LG_HD LgDecSegs lg_decode_segments(const LgMask& m) {
  LgDecSegs g;
  g.n = 0;
  for (int x = 0; x < 4; ++x) g.start[x] = 0;
  for (int x = 0; x < 5; ++x) g.pre[x] = 0;
  const int t = m.N - 1, qb = lg_div_b(m, t);
  lg_decsegs_push(g, 0, m.N < m.sink ? m.N : m.sink);
  if (m.N > m.sink) {
    const long long w0 = ((long long)qb - m.wb + 1) * m.b;  // first token of the oldest live window block
    const int pl = w0 > m.sink ? (int)w0 : m.sink;          // first token read from the ring
    const int len = t - pl + 1;
    if (len >= m.window) {
      lg_decsegs_push(g, m.sink, m.window);  // the whole ring
    } else {
      const int r0 = (pl - m.sink) % m.window;
      if (r0 + len <= m.window) {
        lg_decsegs_push(g, m.sink + r0, len);
      } else {
        lg_decsegs_push(g, m.sink, r0 + len - m.window);
        lg_decsegs_push(g, m.sink + r0, m.window - r0);
      }
    }
  }
  if (m.stride > 0) {
    const int x_lo = m.sb / m.stride;  // first retained block that is not a sink block
    const int hi_kb = qb - m.wb;       // newest block older than the window
    if (hi_kb >= m.stride - 1) {
      const int x_hi = (hi_kb - (m.stride - 1)) / m.stride;
      if (x_hi >= x_lo) lg_decsegs_push(g, m.sink + m.window + x_lo * m.b, (x_hi - x_lo + 1) * m.b);
    }
  }
  for (int x = g.n + 1; x < 5; ++x) g.pre[x] = 0x7fffffff;  // no key index reaches an unused run
  return g;
}

// Slots a cache row needs for contexts of up to n_max tokens.
LG_HD long long lg_cache_slots(int n_max, const LgMask& m) {
  const long long nb = ((long long)n_max + m.b - 1) / m.b;
  return (long long)m.sink + m.window + (m.stride > 0 ? (nb / m.stride) * m.b : 0);
}

// ---------------------------------------------------------------------------------
// Column keys: sink tokens and the keys of strided block columns are seen by EVERY later
// query, not only by the queries whose window reaches them.  The dk/dv pass treats the two
// parts of a key tile's query range separately (window part: dense, ~window/Tq tiles; column
// part: all later query tiles, but only for the few column keys).

// Does [k0, k1] hold a column key?
LG_HD bool lg_has_column_key(const LgMask& m, int k0, int k1) {
  if (k0 < m.sink) return true;
  return m.stride > 0 && lg_next_strided_block(m, lg_div_b(m, k0)) <= lg_div_b(m, k1);
}

// Last query tile (Tq rows) that the window of key k1 (<= N-1) reaches.
LG_HD int lg_qtile_window_hi(const LgMask& m, int k1, int Tq) {
  long long last = m.N - 1;
  const long long w = ((long long)lg_div_b(m, k1) + m.wb) * m.b - 1;
  if (w < last) last = w;
  return (int)(last / Tq);
}

// Is the 64-key group c a column group: column keys AND query rows beyond the window part of
// the Tk-key tile it belongs to?  (The window part of a tile is the same for all its keys.)
LG_HD bool lg_is_column_group(const LgMask& m, int c, int Tk, int Tq) {
  const int g0 = c * 64, g1 = (g0 + 63 < m.N - 1) ? g0 + 63 : m.N - 1;
  const int t0 = (g0 / Tk) * Tk, t1 = (t0 + Tk - 1 < m.N - 1) ? t0 + Tk - 1 : m.N - 1;
  return lg_has_column_key(m, g0, g1) && lg_qtile_window_hi(m, t1, Tq) < (m.N - 1) / Tq;
}

#endif  // LG_MASK_H_
