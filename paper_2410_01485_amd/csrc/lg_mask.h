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
#ifndef LG_MASK_H_
#define LG_MASK_H_

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define LG_HD __host__ __device__ __forceinline__
#else
#define LG_HD inline
#endif

struct LgMask {
  int N;       // sequence length (queries = keys)
  int sink;    // tokens
  int window;  // tokens
  int b;       // max(block, 1): pattern granularity in tokens
  int stride;  // in blocks; 0 = no strided columns
  int sb;      // sink / b
  int wb;      // window / b
};

LG_HD LgMask lg_make_mask(int N, int sink, int window, int block, int stride) {
  LgMask m;
  m.N = N;
  m.b = block > 1 ? block : 1;
  // Values beyond the sequence change nothing; clamping them keeps every product
  // below in int range.
  const int nb = (N + m.b - 1) / m.b;  // number of blocks
  m.sb = sink / m.b < nb ? sink / m.b : nb;
  m.wb = window / m.b < nb ? window / m.b : nb;
  m.sink = m.sb * m.b;
  m.window = m.wb * m.b;
  m.stride = (stride > 0 && stride - 1 < nb) ? stride : 0;
  return m;
}

// live(i, j): may query i attend to key j?
LG_HD bool lg_live(const LgMask& m, int i, int j) {
  if (j > i) return false;
  if (m.b == 1 && m.stride == 0) return j < m.sink || i - j < m.window;
  const int qb = i / m.b, kb = j / m.b;
  if (kb < m.sb || qb - kb < m.wb) return true;
  return m.stride > 0 && kb % m.stride == m.stride - 1;
}

// Is block column kb kept for every later query (sink or strided column)?
LG_HD bool lg_block_always_on(const LgMask& m, int kb) {
  return kb < m.sb || (m.stride > 0 && kb % m.stride == m.stride - 1);
}

// First strided block index >= kb (stride > 0).
LG_HD int lg_next_strided_block(const LgMask& m, int kb) {
  return kb + (m.stride - 1 - kb % m.stride);
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
    live = istar / m.b - je / m.b < m.wb;
  }
  if (!live && m.stride > 0) live = lg_next_strided_block(m, k0 / m.b) <= je / m.b;
  if (!live) return LG_TILE_DEAD;
  if (k1 > q0) return LG_TILE_PARTIAL;  // crosses the diagonal (or runs past N-1)
  if (m.stride == 1) return LG_TILE_FULL;
  // smallest key of the tile that is neither sink nor strided must still be inside
  // the window of the last row
  int j = k0;
  for (int it = 0; it < 4 && j <= k1; ++it) {
    const int kb = j / m.b;
    if (kb < m.sb) j = m.sink;
    else if (m.stride > 0 && kb % m.stride == m.stride - 1) j = (kb + 1) * m.b;
    else break;
  }
  if (j > k1) return LG_TILE_FULL;
  return (q1 / m.b - j / m.b < m.wb) ? LG_TILE_FULL : LG_TILE_PARTIAL;
}

// Next live key tile (tile = keys [t*Tk, t*Tk+Tk-1]) after tile `prev` for the query
// rows [q0, q1]; pass prev = -1 to get the first.  Returns -1 when there is none.
LG_HD int lg_next_ktile(const LgMask& m, int q0, int q1, int Tk, int prev) {
  const int t0 = prev + 1;
  const int j0 = t0 * Tk;
  if (j0 > q1) return -1;
  if (j0 < m.sink) return t0;
  // window: live keys of the row range are [jw, q1]
  int jw = (q0 / m.b - m.wb + 1) * m.b;
  if (jw < 0) jw = 0;
  int t = jw / Tk;
  if (t < t0) t = t0;
  if (m.stride > 0) {
    const int kb0 = j0 / m.b;
    const int f = lg_next_strided_block(m, kb0);
    const int ts = (f == kb0) ? t0 : (int)(((long long)f * m.b) / Tk);
    if (ts < t) t = ts;
  }
  return ((long long)t * Tk <= q1) ? t : -1;
}

// Live query tiles (tile = rows [u*Tq, u*Tq+Tq-1]) of the keys [k0, k1] (k1 <= N-1):
// always one contiguous range [*lo, *hi].
LG_HD void lg_qtile_range(const LgMask& m, int k0, int k1, int Tq, int* lo, int* hi) {
  *lo = k0 / Tq;
  bool always = k0 < m.sink;
  if (!always && m.stride > 0) always = lg_next_strided_block(m, k0 / m.b) <= k1 / m.b;
  long long last = m.N - 1;
  if (!always) {
    const long long w = ((long long)(k1 / m.b) + m.wb) * m.b - 1;  // last row whose window holds k1
    if (w < last) last = w;
  }
  *hi = (int)(last / Tq);
}

#endif  // LG_MASK_H_
