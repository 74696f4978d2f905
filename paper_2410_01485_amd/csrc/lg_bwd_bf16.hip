// lg_bwd_bf16.hip — bf16 backward on the gfx950 matrix cores (paper Section 3.2: the
// backward step skips masked key blocks just like the forward; Table 1 counts both).
//
// Two kernels (the first one also forms Delta).  Sink + window without GQA uses no atomics and is
// bit-reproducible; strided patterns and GQA add float32 partial dk/dv sums of the column keys
// with atomics (see the dk/dv section).  Tiles travel global -> LDS directly (row-major,
// swizzled; lg_swz.h) and are read both with the contraction over dims (row reads) and with the
// contraction over tile rows (transposing LDS reads), so no tile is ever stored twice.
//
//  dq kernel (query-tile major, same tile walk and 4-stage ring as the forward; 8 waves x
//  32 query rows).  Per live key tile:
//     S^T  = K Q^T,  dP^T = V dO^T      (keys x queries; A = K / V rows from LDS,
//                                        B = Q / dO fragments kept in registers)
//     P^T  = exp2(S^T c - lse_i c'),  dS^T = P^T o (dP^T - Delta_i)   (one query per lane)
//     dQ^T += K^T dS^T                  (dims x queries; A = K through transposing reads,
//                                        B = dS^T straight from the accumulator registers)
//  dk/dv kernel (key-tile major; 8 waves x 32 keys = 256 keys per workgroup; the K fragment
//  of a wave stays in registers, the V rows of the workgroup stay in LDS).  Per live query
//  tile of 64 rows, for every query head of the kv group:
//     S  = Q K^T,  dP = dO V^T          (queries x keys; A = Q / dO rows from LDS)
//     P, dS as above                    (one key per lane; S and dP start from the per-row
//                                        values -lse / scale and -Delta as their addend)
//     dV^T += dO^T P,  dK^T += Q^T dS   (dims x keys; A = dO / Q through transposing reads,
//                                        B = P / dS straight from the accumulators)
// 7 tile products instead of the minimal 5: S and dP are computed in both kernels.
//
// For head dim 128 and windows of 16 or more tiles both kernels have a second form with 64 rows
// (keys) per wave, one wave per SIMD and the accumulators in AGPRs (further down): every operand
// read from LDS then feeds two matrix instructions.
#include "../../include/longgen_attn.h"
#include "lg_kernels.h"
#include "lg_mfma.h"
#include "lg_swz.h"
#include "lg_wide.h"

namespace {

constexpr float LOG2E = 1.44269504088896340736f;

// TOKEN (both kernels): the pattern is token-granular without strided columns (block <= 1,
// stride 0).  The mask fields that are then known let the compiler drop the block / stride
// arithmetic from the per-tile scheduling, and partial tiles are masked with two compares per
// element instead of a per-element evaluation of the general predicate.

// sum over 8 bf16 pairs of x * y, added to s
__device__ __forceinline__ float lg_dot8(uint4 x, uint4 y, float s) {
  const unsigned xw[4] = {x.x, x.y, x.z, x.w}, yw[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    s = fmaf(__uint_as_float(xw[t] << 16), __uint_as_float(yw[t] << 16), s);
    s = fmaf(__uint_as_float(xw[t] & 0xffff0000u), __uint_as_float(yw[t] & 0xffff0000u), s);
  }
  return s;
}

// Both dq kernels also form Delta_i = <dout_i, out_i> of their rows (a lane and its partner in
// the other half of the wave hold the whole row of dout anyway) and leave -Delta and -lse / scale
// in the workspace for the dk/dv kernels, which run after them on the same stream.
// ------------------------------------------------------------------------- dq
template <int D, bool TOKEN>
__global__ __launch_bounds__(512) void dq_bf16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const uint16_t* __restrict__ out, const uint16_t* __restrict__ dout, const float* __restrict__ lse,
    float* __restrict__ ndelta, float* __restrict__ nlse, uint16_t* __restrict__ dq, int Hq, int Hkv, float scale,
    LgMask m_in, int nqt, int total, int per_xcd) {
  LgMask m = m_in;
  if (TOKEN) {
    m.b = 1;
    m.stride = 0;
    m.bshift = 0;
    m.smask = -1;
    m.sb = m.sink;
    m.wb = m.window;
  }
  using T = LgSwzTile<D>;
  constexpr int NT = 512, STAGES = 4;
  using Dma = LgDma<D, NT>;
  constexpr int TQ = LG_BF16_TQ, TK = LG_BF16_TK;
  static_assert(TQ == 256 && TK == 64, "8 waves x 32 query rows, 64-key tiles");
  constexpr int DC = D / 16, DB = D / 32;
  constexpr int STAGE = 2 * T::BYTES;  // K tile + V tile
  constexpr int LPT = 2 * Dma::CH;
  __shared__ __attribute__((aligned(1024))) unsigned char smem[STAGES * STAGE];

  const int L = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (L >= total) return;
  // logical order: (b, kv head) slowest, then query tile (longest rows first), then the query
  // heads of the GQA group: the G workgroups that walk the same K/V tiles run side by side
  const int G = Hq / Hkv;
  const int gq = L % G, rest = L / G;
  const int qt = nqt - 1 - (rest % nqt);
  const int bhk = rest / nqt;
  const int b = bhk / Hkv, hk = bhk % Hkv;
  const int hq = hk * G + gq;
  const int N = m.N;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, g = lane >> 5;
  const int q0 = qt * TQ, q1 = min(q0 + TQ - 1, N - 1);
  const size_t qbase = ((size_t)(b * Hq + hq) * m.ld) * D;
  const uint16_t* kh = k + ((size_t)(b * Hkv + hk) * m.ld) * D;
  const uint16_t* vh = v + ((size_t)(b * Hkv + hk) * m.ld) * D;
  const int i = q0 + wave * 32 + n;
  const int iq = min(i, N - 1);
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const int qw0 = min(q0 + wave_s * 32, N - 1), qw1 = min(q0 + wave_s * 32 + 31, N - 1);  // this wave's rows

  bf16x8_t qf[DC], gf[DC];
  float di = 0.f;
#pragma unroll
  for (int dc = 0; dc < DC; ++dc) {
    const uint4 gw = *reinterpret_cast<const uint4*>(dout + qbase + (size_t)iq * D + dc * 16 + g * 8);
    qf[dc] = lg_as_bf16x8(*reinterpret_cast<const uint4*>(q + qbase + (size_t)iq * D + dc * 16 + g * 8));
    gf[dc] = lg_as_bf16x8(gw);
    di = lg_dot8(gw, *reinterpret_cast<const uint4*>(out + qbase + (size_t)iq * D + dc * 16 + g * 8), di);
  }
  di += lg_other_half(di);  // Delta of row i
  const float sl2 = scale * LOG2E;
  const float lse_i = lse[(size_t)(b * Hq + hq) * m.ld + iq];
  float lse2 = lse_i * LOG2E;
  if (g == 0 && i < N) {
    ndelta[(size_t)(b * Hq + hq) * N + i] = -di;
    nlse[(size_t)(b * Hq + hq) * N + i] = -lse_i / scale;
  }
  // Touch everything loaded so far, so that the compiler's waits for these loads sit here and
  // not inside the tile loop (where they would drain the direct loads kept in flight).
#pragma unroll
  for (int dc = 0; dc < DC; ++dc) asm volatile("" ::"v"(qf[dc]), "v"(gf[dc]));
  asm volatile("" : "+v"(lse2), "+v"(di));

  f32x16_t acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

  Dma dma;
  dma.init(tid);
  LgSwzReader<D> rd;
  rd.init(n, g);
  const uint32_t lds0 = (uint32_t)(uintptr_t)LG_LDS_PTR(unsigned char, smem);
  const LgQSched qs = lg_qsched_init(m, q0, q1);
  auto issue = [&](int t, int stage) {
    const size_t off = (size_t)t * TK * D;
    dma.issue(kh + off, N - t * TK, lds0 + stage * STAGE);
    dma.issue(vh + off, N - t * TK, lds0 + stage * STAGE + T::BYTES);
  };

  // patterns without strided columns walk the window run rotated (L2 sharing between neighbours)
  const LgQWalk qw = lg_qwalk_init(qs);
  auto next_tile = [&](int prev) -> int {
    if (TOKEN || m.stride == 0) return prev < 0 ? lg_qwalk_first(qw) : lg_qwalk_next(qw, prev);
    return lg_qsched_next(m, qs, prev);
  };
  int t = next_tile(-1);
  int t_issue = t;
  int ahead = 0;
  for (; ahead < STAGES - 1 && t_issue >= 0; ++ahead) {
    issue(t_issue, ahead);
    t_issue = next_tile(t_issue);
  }
  int stage = 0;
  while (t >= 0) {
    if (ahead >= 3) LG_WAIT_VMCNT(2 * LPT);
    else if (ahead == 2) LG_WAIT_VMCNT(LPT);
    else LG_WAIT_VMCNT(0);
    __syncthreads();  // tile t landed for everyone; everyone is done with tile t-1
    if (t_issue >= 0) {
      issue(t_issue, (stage + STAGES - 1) % STAGES);
      t_issue = next_tile(t_issue);
      ++ahead;
    }
    const int k0 = t * TK;
    // A tile that is not live throughout for the workgroup's 256 rows is classified again for
    // this wave's 32 rows: most waves then find it wholly live or wholly dead (they sit it out).
    int kind = LG_TILE_FULL;
    if (!lg_qsched_full(m, qs, t)) kind = lg_tile_kind(m, qw0, qw1, k0, k0 + TK - 1);
    const bool full = kind == LG_TILE_FULL;
    const int sk = stage * STAGE, sv = sk + T::BYTES;
    uint32_t bits = 0xffffffffu;
    if (kind == LG_TILE_PARTIAL && !TOKEN) bits = lg_key_bits(m, iq, k0, g);
    // Token mode: row i sees the keys [i - window + 1, i] and the sink keys below
    // min(sink, i + 1).  In tile coordinates (key = k0 + 4g + c, c a compile-time constant):
    const int hi = i - k0 - 4 * g;         // c <= hi           : causal
    const int lo = hi - (m.window - 1);    // c >= lo           : inside the window
    const int se = m.sink - k0 - 4 * g;    // c < se (&& c <= hi): a sink key
    const bool has_sink = k0 < m.sink;     // wave-uniform
    auto dead = [&](int kb, int r) -> bool {
      if (!TOKEN) return !(bits & (1u << (kb * 16 + r)));
      const int c = 32 * kb + lg_crow(r, 0);
      bool live = (unsigned)(c - lo) < (unsigned)m.window;
      if (has_sink) live |= c < se && c <= hi;
      return !live;
    };

    if (kind != LG_TILE_DEAD)
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      f32x16_t sc, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) sc[r] = dp[r] = 0.f;
#pragma unroll
      for (int dc = 0; dc < DC; ++dc) {
        sc = lg_mfma32(rd.read_rows(smem, sk, kb, dc), qf[dc], sc);
        dp = lg_mfma32(rd.read_rows(smem, sv, kb, dc), gf[dc], dp);
      }
      float ds[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float p = __builtin_amdgcn_exp2f(fmaf(sc[r], sl2, -lse2));
        if (!full && dead(kb, r)) p = 0.f;
        ds[r] = p * (dp[r] - di);
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const bf16x8_t bop = lg_pack8(ds + 8 * h);
#pragma unroll
        for (int db = 0; db < DB; ++db) acc[db] = lg_mfma32(rd.read_cols(smem, sk, db, 2 * kb + h), bop, acc[db]);
      }
    }
    --ahead;
    t = next_tile(t);
    stage = (stage + 1) % STAGES;
  }

  if (i < N) {
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        uint2 w;
        w.x = lg_pack_bf16(acc[db][4 * r4 + 0] * scale, acc[db][4 * r4 + 1] * scale);
        w.y = lg_pack_bf16(acc[db][4 * r4 + 2] * scale, acc[db][4 * r4 + 3] * scale);
        *reinterpret_cast<uint2*>(dq + qbase + (size_t)i * D + db * 32 + 8 * r4 + 4 * g) = w;
      }
  }
}

// ---------------------------------------------------------------------- dk, dv
// Column keys (sink tokens, keys of strided block columns) are seen by every later query.
// The query range of a key tile therefore has a dense window part (like every tile) and, if it
// holds column keys, a long column part: all later rows, but only its column keys live.
// With one column group per head (the sink of a sink + window pattern) and no GQA the tile that
// holds it simply runs its whole range and is launched first.  Otherwise (strided patterns, or G
// query heads per kv head, which one workgroup would have to walk one after the other) the column
// parts are split off: the COLUMN instance of the kernel packs the 64-key column groups four at
// a time into virtual 256-key tiles, so that all 8 waves have live keys and a Q / dO tile is
// used by 256 keys again, cuts their query range into chunks of LG_COL_CHUNK tiles that run as
// separate workgroups, and adds float32 partial sums into the workspace with hardware atomics
// (their order is not fixed, so the last bits of dk/dv of column keys can differ from run to
// run).  The main instance then handles the window part of every tile and folds the partial
// sums in before it rounds to bf16.  The table kernel lists the column groups once per call.
constexpr int LG_COL_CHUNK = 64;  // query tiles (64 rows each) per column workgroup

// col_of_group[c] = index of 64-key group c among the column groups, or -1; col_list = inverse.
// One workgroup of 1024 threads, 1024 groups per round: ranks from a ballot per wave plus the
// counts of the waves before it.
__global__ __launch_bounds__(1024) void dkdv_column_table_kernel(int* __restrict__ col_of_group,
                                                                 int* __restrict__ col_list, LgMask m, int ngroups) {
  __shared__ int wcount[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int base = 0;
  for (int c0 = 0; c0 < ngroups; c0 += 1024) {
    const int c = c0 + tid;
    const bool is = c < ngroups && lg_is_column_group(m, c, LG_BF16_BTK, LG_BF16_BTQ);
    const unsigned long long bal = __ballot(is);
    if (lane == 0) wcount[wave] = __popcll(bal);
    __syncthreads();
    int off = base, all = 0;
    for (int w = 0; w < 16; ++w) {
      if (w < wave) off += wcount[w];
      all += wcount[w];
    }
    const int rank = off + __popcll(bal & ((1ull << lane) - 1ull));
    if (c < ngroups) col_of_group[c] = is ? rank : -1;
    if (is) col_list[rank] = c;
    base += all;
    __syncthreads();
  }
}

__global__ void fill_zero_kernel(float4* __restrict__ p, size_t n4) {
  for (size_t x = (size_t)blockIdx.x * blockDim.x + threadIdx.x; x < n4; x += (size_t)gridDim.x * blockDim.x)
    p[x] = make_float4(0.f, 0.f, 0.f, 0.f);
}

// Adds a 32 x 32 accumulator block (lane (n, g), register r <-> row n, column 8 (r / 4) + 4 g + r % 4)
// to dst[row * ld + column], rows below nrows only, with float32 atomics.  The block is turned
// through 4 KB of LDS that belong to the calling wave (16-byte chunks XOR-swizzled by row), so that
// one atomic instruction adds two whole rows of 32 consecutive floats -- two cache lines --
// instead of two floats in each of 32 lines, which is what bounds the column instances otherwise.
template <typename Acc>
__device__ __forceinline__ void lg_atomic_add_block(float* tr, const Acc& acc, float* dst, int ld, int nrows,
                                                    int n, int g) {
#pragma unroll
  for (int r4 = 0; r4 < 4; ++r4)
    *reinterpret_cast<float4*>(tr + n * 32 + 4 * ((2 * r4 + g) ^ (n & 7))) =
        make_float4(acc[4 * r4], acc[4 * r4 + 1], acc[4 * r4 + 2], acc[4 * r4 + 3]);
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // (one wave: its LDS accesses complete in order)
#pragma unroll
  for (int it = 0; it < 16; ++it) {
    const int row = 2 * it + g;
    const float x = tr[row * 32 + 4 * ((n >> 2) ^ (row & 7)) + (n & 3)];
    if (row < nrows) unsafeAtomicAdd(dst + (size_t)row * ld + n, x);  // hardware float add in L2
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
}

// ncol: column groups handled by the COLUMN instance (0: none are split off)
template <int D, bool TOKEN, bool COLUMN>
__global__ __launch_bounds__(512) void dkdv_bf16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const uint16_t* __restrict__ dout, const float* __restrict__ nlse, const float* __restrict__ ndelta,
    uint16_t* __restrict__ dk, uint16_t* __restrict__ dv, int Hq, int Hkv, float scale, LgMask m_in,
    int nkt, int total, int per_xcd, const int* __restrict__ col_of_group, const int* __restrict__ col_list,
    float* __restrict__ part_dk, float* __restrict__ part_dv, int ncol, int nchunk) {
  LgMask m = m_in;
  if (TOKEN) {
    m.b = 1;
    m.stride = 0;
    m.bshift = 0;
    m.smask = -1;
    m.sb = m.sink;
    m.wb = m.window;
  }
  using T = LgSwzTile<D>;
  constexpr int NT = 512;
  using Dma = LgDma<D, NT>;
  constexpr int TQ = LG_BF16_BTQ, TK = LG_BF16_BTK;
  static_assert(TQ == 64 && TK == 256, "64 query rows per step, 8 waves x 32 keys");
  constexpr int DC = D / 16, DB = D / 32;
  constexpr int HALF = 32 * T::ROW_BYTES;
  constexpr int VRES = 4 * T::BYTES;                 // the workgroup's 256 V rows
  constexpr int OFF_G = T::BYTES, OFF_L = 2 * T::BYTES;
  constexpr int STAGE = 2 * T::BYTES + 1024;         // Q tile, dO tile, -lse / scale | -Delta (2 x 64 floats)
  __shared__ __attribute__((aligned(1024))) unsigned char smem[VRES + 2 * STAGE];

  const int G = Hq / Hkv;
  const int N = m.N;
  const float sl2 = scale * LOG2E;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, g = lane >> 5;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  // Work item.
  //   main, no split-off columns: key tile 0 of every (b, kv head) holds the sink keys and runs
  //     ~N/64 steps instead of ~(window+256)/64, so those workgroups take the first block ids
  //     (dealt round-robin over the XCDs: they start at once, spread evenly); the other
  //     (head, key tile) items follow in XCD-contiguous runs, so that neighbouring key tiles
  //     share their Q / dO rows in one XCD's L2.
  //   main, columns split off: all items in XCD-contiguous runs.
  //   COLUMN: blockIdx.x = (chunk * nvt + virtual tile) * (heads) + (b x kv head) * G + query head of
  //     the group: with the heads innermost every XCD gets the same mix of long and short items (and
  //     of those that exit at once: a virtual tile has no rows in the chunks before its column part
  //     starts), and the virtual tiles of one head that walk the same chunk of query rows run on one
  //     XCD at about the same time.
  int bh, kt = 0, vt = 0, chunk = 0, gq = 0;
  if (COLUMN) {
    const int nvt = (ncol + 3) / 4, nh = (total / nkt) * G;
    int x = blockIdx.x;
    const int hd = x % nh;
    x /= nh;
    vt = x % nvt;
    chunk = x / nvt;
    gq = hd % G;
    bh = hd / G;
  } else if (ncol > 0) {
    const int L = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (L >= total) return;
    bh = L / nkt;
    kt = L % nkt;
  } else {
    const int nbh = total / nkt;
    if ((int)blockIdx.x < nbh) {
      bh = blockIdx.x;
      kt = 0;
    } else {
      const int idx = blockIdx.x - nbh;
      const int L = (idx % 8) * per_xcd + idx / 8;
      if (nkt == 1 || L >= total - nbh) return;
      bh = L / (nkt - 1);
      kt = 1 + L % (nkt - 1);
    }
  }
  const int b = bh / Hkv, hk = bh % Hkv;
  const int k0 = kt * TK, k1 = min(k0 + TK - 1, N - 1);
  const size_t kbase = ((size_t)(b * Hkv + hk) * m.ld) * D;
  // this wave's 32 keys: part of the key tile, or half of one of the virtual tile's column groups
  int kw0 = k0 + wave_s * 32;
  int col_gi = 0;        // COLUMN: index of this wave's column group
  bool active = true;    // COLUMN: the virtual tile may have fewer than 4 groups
  int r0_w = 0;          // COLUMN: first row of the wave's column part
  if (COLUMN) {
    col_gi = 4 * vt + (wave_s >> 1);
    active = col_gi < ncol;
    const int grp = col_list[min(col_gi, ncol - 1)];
    kw0 = 64 * grp + 32 * (wave_s & 1);
    const int t1 = min((64 * grp / TK) * TK + TK - 1, N - 1);
    r0_w = (lg_qtile_window_hi(m, t1, TQ) + 1) * TQ;
  }
  const int j = kw0 + n;  // this lane's key
  const int jk = min(j, N - 1);

  bf16x8_t kf[DC];
#pragma unroll
  for (int dc = 0; dc < DC; ++dc)
    kf[dc] = lg_as_bf16x8(*reinterpret_cast<const uint4*>(k + kbase + (size_t)jk * D + dc * 16 + g * 8));
#pragma unroll
  for (int dc = 0; dc < DC; ++dc) asm volatile("" ::"v"(kf[dc]));

  f32x16_t ak[DB], av[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) ak[db][r] = av[db][r] = 0.f;
  // query tiles of this work item
  int lo, hi, hq0 = hk * G, nheads = G;
  if (COLUMN) {
    // the query tiles of chunk number `chunk` (chunks are cut at fixed tile numbers for all virtual
    // tiles, counted from the chunk in which the first column part starts) that come after the
    // window part of the virtual tile's first group
    const int tf = min((64 * col_list[0] / TK) * TK + TK - 1, N - 1);
    const int c_abs = (lg_qtile_window_hi(m, tf, TQ) + 1) / LG_COL_CHUNK + chunk;
    const int grp0 = col_list[4 * vt];
    const int t1 = min((64 * grp0 / TK) * TK + TK - 1, N - 1);
    lo = max(lg_qtile_window_hi(m, t1, TQ) + 1, c_abs * LG_COL_CHUNK);
    hi = min((N - 1) / TQ, c_abs * LG_COL_CHUNK + LG_COL_CHUNK - 1);
    if (lo > hi) return;
    hq0 += gq;
    nheads = 1;
  } else if (ncol > 0) {  // the window part; the column part is the COLUMN instance's
    lo = k0 / TQ;
    hi = lg_qtile_window_hi(m, k1, TQ);
  } else {
    lg_qtile_range(m, k0, k1, TQ, &lo, &hi);
  }
  const int per_head = hi - lo + 1;
  const int steps = per_head * nheads;

  Dma dma;
  dma.init(tid);
  LgSwzReader<D> rd;
  rd.init(n, g);
  const uint32_t lds0 = (uint32_t)(uintptr_t)LG_LDS_PTR(unsigned char, smem);
  // the workgroup's V rows, resident for the whole kernel
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    const int r0 = COLUMN ? 64 * col_list[min(4 * vt + x, ncol - 1)] : k0 + 64 * x;
    const int rc = min(r0, N - 1);  // a tile wholly past the end repeats the last row
    dma.issue(v + kbase + (size_t)rc * D, r0 < N ? N - r0 : 1, lds0 + x * T::BYTES);
  }
  const int voff = (wave >> 1) * T::BYTES + (wave & 1) * HALF;  // this wave's 32 V rows

  // (head, query tile) of a step advance incrementally: no divisions in the loop
  auto issue_step = [&](int hq, int u, int buf) {
    const int q0 = u * TQ;
    const size_t row0 = (size_t)(b * Hq + hq) * N;
    const uint32_t st = lds0 + VRES + buf * STAGE;
    // the small per-row loads go first: anything the compiler makes them wait for must not
    // include the tile loads issued below
    if (wave < 2) {  // wave 0: -lse / scale rows, wave 1: -Delta rows (64 floats each)
      const float* src = (wave == 0 ? nlse : ndelta) + row0 + min(q0 + lane, N - 1);
      lg_dma_f32x64(src, st + OFF_L + wave * 256);
    }
    const size_t urow0 = (size_t)(b * Hq + hq) * m.ld;  // the head's first row in the caller's tensors
    dma.issue(q + (urow0 + q0) * D, N - q0, st);
    dma.issue(dout + (urow0 + q0) * D, N - q0, st + OFF_G);
  };

  // The query tiles [lo, hi] of a head are walked rotated: at step x the tile congruent to x
  // modulo the range length.  Neighbouring key tiles, whose ranges overlap almost completely and
  // which run side by side, then read the same Q / dO tile at the same time and share it in L2.
  const int u0 = lo + (per_head - lo % per_head) % per_head;
  int hq_i = hq0, u_i = u0;      // step being issued
  int u_c = u0;                  // query tile of the step being computed
  int left_i = per_head;         // steps of the head being issued that are not issued yet
  issue_step(hq_i, u_i, 0);
  for (int st = 0; st < steps; ++st) {
    const int buf = st & 1;
    LG_WAIT_VMCNT(0);
    __syncthreads();  // step st landed for everyone; everyone is done with step st-1
    if (st + 1 < steps) {
      u_i = (u_i == hi) ? lo : u_i + 1;
      if (--left_i == 0) {  // next query head of the group: same walk again
        left_i = per_head;
        u_i = u0;
        ++hq_i;
      }
      issue_step(hq_i, u_i, buf ^ 1);
    }
    const int q0 = u_c * TQ;
    u_c = (u_c == hi) ? lo : u_c + 1;
    const int q1 = min(q0 + TQ - 1, N - 1);
    // this wave's 32 keys against the step's 64 queries: a wave with no live pair sits the step
    // out (most waves of the sink key tile do, once the queries are past its window)
    if (COLUMN && (!active || q0 < r0_w)) continue;  // no group, or rows of its window part
    const int kind = lg_tile_kind(m, q0, q1, kw0, kw0 + 31);
    if (kind == LG_TILE_DEAD) continue;
    const bool full = kind == LG_TILE_FULL && q0 + TQ <= N;
    const int sq = VRES + buf * STAGE, sg = sq + OFF_G;
    const float* sL = reinterpret_cast<const float*>(smem + sq + OFF_L);
    uint32_t bits = ~0u;
    if (!full && !TOKEN) bits = lg_row_bits(m, j, q0, g);
    // Token mode: key j is seen by the rows [j, j + window - 1] (by every row >= j if it is a
    // sink key), below N.  In tile coordinates (row = q0 + 4g + c, c a compile-time constant):
    const int lo_c = j - q0 - 4 * g;                                   // c >= lo_c : causal
    const unsigned w_eff = j < m.sink ? 0x7fffffffu : (unsigned)m.window;  // c < lo_c + w_eff
    const int n_c = N - q0 - 4 * g;                                    // c < n_c   : row exists
    auto dead = [&](int qb, int r) -> bool {
      if (!TOKEN) return !((bits >> (qb * 16 + r)) & 1);
      const int c = 32 * qb + lg_crow(r, 0);
      return !((unsigned)(c - lo_c) < w_eff && c < n_c);
    };

    // Per 32-row query block, in an order that keeps few values alive at a time:
    // S -> P -> (dV += dO^T P) -> dP -> dS -> (dK += Q^T dS)
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      float p[16];
      __builtin_amdgcn_sched_barrier(0);  // phases stay apart: bounds the operands held at once
      {
        // the accumulator starts from -lse / scale of its rows (register r <-> row 8 (r / 4) + 4g + r % 4)
        f32x16_t sc;
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const float4 l4 = *reinterpret_cast<const float4*>(sL + qb * 32 + 8 * r4 + 4 * g);
          sc[4 * r4 + 0] = l4.x; sc[4 * r4 + 1] = l4.y; sc[4 * r4 + 2] = l4.z; sc[4 * r4 + 3] = l4.w;
        }
#pragma unroll
        for (int dc = 0; dc < DC; ++dc) sc = lg_mfma32(rd.read_rows(smem, sq, qb, dc), kf[dc], sc);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float pv = __builtin_amdgcn_exp2f(sc[r] * sl2);
          if (!full && dead(qb, r)) pv = 0.f;
          p[r] = pv;
        }
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const bf16x8_t pb = lg_pack8(p + 8 * h);
#pragma unroll
        for (int db = 0; db < DB; ++db) av[db] = lg_mfma32(rd.read_cols(smem, sg, db, 2 * qb + h), pb, av[db]);
      }
      __builtin_amdgcn_sched_barrier(0);
      {
        f32x16_t dp;  // starts from -Delta of its rows
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const float4 d4 = *reinterpret_cast<const float4*>(sL + 64 + qb * 32 + 8 * r4 + 4 * g);
          dp[4 * r4 + 0] = d4.x; dp[4 * r4 + 1] = d4.y; dp[4 * r4 + 2] = d4.z; dp[4 * r4 + 3] = d4.w;
        }
#pragma unroll
        for (int dc = 0; dc < DC; ++dc)
          dp = lg_mfma32(rd.read_rows(smem, sg, qb, dc), rd.read_rows(smem, voff, 0, dc), dp);
#pragma unroll
        for (int r = 0; r < 16; ++r) p[r] *= dp[r];  // p becomes dS
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const bf16x8_t db_ = lg_pack8(p + 8 * h);
#pragma unroll
        for (int db = 0; db < DB; ++db) ak[db] = lg_mfma32(rd.read_cols(smem, sq, db, 2 * qb + h), db_, ak[db]);
      }
    }
  }

  // partial sums of the column parts: [b x kv head][column group][64 keys][D] float32, dk unscaled
  if (COLUMN) {
    // the wave's own V rows (only this wave ever read them) serve as the turning space
    static_assert(HALF >= 4096, "a 32 x 32 float block fits the wave's V rows");
    float* tr = reinterpret_cast<float*>(smem + voff);
    const int nrows = active ? min(max(N - kw0, 0), 32) : 0;
    const size_t prow = (((size_t)bh * ncol + col_gi) * 64 + (wave_s & 1) * 32) * D;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      lg_atomic_add_block(tr, ak[db], part_dk + prow + db * 32, D, nrows, n, g);
      lg_atomic_add_block(tr, av[db], part_dv + prow + db * 32, D, nrows, n, g);
    }
    return;
  }
  const int cid = (ncol > 0 && kw0 < N) ? col_of_group[kw0 >> 6] : -1;
  if (cid >= 0 && j < N) {
    const size_t prow = (((size_t)bh * ncol + cid) * 64 + (wave_s & 1) * 32 + n) * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const float4 pk = *reinterpret_cast<const float4*>(part_dk + prow + db * 32 + 8 * r4 + 4 * g);
        const float4 pv = *reinterpret_cast<const float4*>(part_dv + prow + db * 32 + 8 * r4 + 4 * g);
        ak[db][4 * r4 + 0] += pk.x; ak[db][4 * r4 + 1] += pk.y; ak[db][4 * r4 + 2] += pk.z; ak[db][4 * r4 + 3] += pk.w;
        av[db][4 * r4 + 0] += pv.x; av[db][4 * r4 + 1] += pv.y; av[db][4 * r4 + 2] += pv.z; av[db][4 * r4 + 3] += pv.w;
      }
  }
  if (j < N) {
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        uint2 w;
        w.x = lg_pack_bf16(ak[db][4 * r4 + 0] * scale, ak[db][4 * r4 + 1] * scale);
        w.y = lg_pack_bf16(ak[db][4 * r4 + 2] * scale, ak[db][4 * r4 + 3] * scale);
        *reinterpret_cast<uint2*>(dk + kbase + (size_t)j * D + db * 32 + 8 * r4 + 4 * g) = w;
        w.x = lg_pack_bf16(av[db][4 * r4 + 0], av[db][4 * r4 + 1]);
        w.y = lg_pack_bf16(av[db][4 * r4 + 2], av[db][4 * r4 + 3]);
        *reinterpret_cast<uint2*>(dv + kbase + (size_t)j * D + db * 32 + 8 * r4 + 4 * g) = w;
      }
  }
}

// Work queue of the kernels that keep one workgroup per CU: queue[x] counts the items handed out
// with id % 8 == x (the ids that a grid launch would have placed on XCD x); a workgroup serves its
// own XCD's ids first, then the others'.  Returns the next id, or -1 once all eight counters have
// run out (every wave of every workgroup gets there).  Called by all threads of the workgroup; the
// barriers also separate two items' use of LDS.
__device__ __forceinline__ int lg_queue_take(int* __restrict__ queue, int nitems, int xcd, int* s_item) {
  __syncthreads();  // everyone is done with the previous item: its LDS, and *s_item
  if (threadIdx.x == 0) {
    int id = -1;
    for (int d = 0; d < 8 && id < 0; ++d) {
      const int x = (xcd + d) & 7;
      const int c = atomicAdd(queue + x, 1);
      if (c < (1 << 27) && 8 * c + x < nitems) id = 8 * c + x;
    }
    *s_item = id;
  }
  __syncthreads();
  return __builtin_amdgcn_readfirstlane(*s_item);
}

// ------------------------------------------------- dk, dv: 64 keys per wave (D = 128)
// The main instance for D = 128.  Four waves of 64 keys each: every operand read from LDS (Q / dO
// rows, their transposed blocks) now feeds two matrix instructions, which halves the LDS traffic
// per product, the limit of the 32-keys-per-wave kernel above.  A wave then owns 256 accumulator
// registers (dk and dv of 64 keys x 128 dims); they live in the AGPR half of the register file
// for the whole kernel and only the matrix instructions touch them, while S / dP, which the
// vector unit has to read, use ordinary VGPRs.  The compiler picks one register form for all
// matrix instructions of a function, so the instructions are written out with their register
// classes here; that leaves their dependency waits, which the compiler otherwise provides, to
// this code (see the notes at lg_tie and in the step).
// COLUMN: the instance for the split-off column parts, as in the 8-wave kernel: a virtual tile of
// four 64-key column groups, one group per wave, one chunk of the query range per workgroup,
// float32 atomics into the partial sums.
// bid: the work item, numbered like the block ids of the 8-wave kernel's grid.
template <bool TOKEN, bool COLUMN>
__device__ __forceinline__ void dkdv_wide_item(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const uint16_t* __restrict__ dout, const float* __restrict__ nlse, const float* __restrict__ ndelta,
    uint16_t* __restrict__ dk, uint16_t* __restrict__ dv, int Hq, int Hkv, float scale, LgMask m_in,
    int nkt, int total, int per_xcd, const int* __restrict__ col_of_group, const int* __restrict__ col_list,
    float* __restrict__ part_dk, float* __restrict__ part_dv, int ncol, int nchunk, const int bid) {
  LgMask m = m_in;
  if (TOKEN) {
    m.b = 1;
    m.stride = 0;
    m.bshift = 0;
    m.smask = -1;
    m.sb = m.sink;
    m.wb = m.window;
  }
  constexpr int D = 128;
  using T = LgSwzTile<D>;
  constexpr int NT = 256;
  using Dma = LgDma<D, NT>;
  constexpr int TQ = LG_BF16_BTQ, TK = LG_BF16_BTK;
  static_assert(TQ == 64 && TK == 256, "64 query rows per step, 4 waves x 64 keys");
  constexpr int DC = D / 16, DB = D / 32;
  constexpr int VRES = 4 * T::BYTES;                 // the workgroup's 256 V rows
  constexpr int OFF_G = T::BYTES, OFF_L = 2 * T::BYTES;
  constexpr int STAGE = 2 * T::BYTES + 1024;         // Q tile, dO tile, -lse / scale | -Delta (2 x 64 floats)
  __shared__ __attribute__((aligned(1024))) unsigned char smem[VRES + 2 * STAGE];

  const int G = Hq / Hkv;
  const int N = m.N;
  const float sl2 = scale * LOG2E;
  // (the thread index is made opaque per work item: what derives from it is recomputed for every item
  // instead of being kept in registers, or spilled, across the resident kernel's loop over items)
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, g = lane >> 5;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  // work item: as in the kernel above
  int bh, kt = 0, vt = 0, chunk = 0, gq = 0;
  if (COLUMN) {
    const int nvt = (ncol + 3) / 4;
    // (the results of these divisions are pinned to scalar registers: the global->LDS copies take
    // their base addresses, which derive from them, as scalar operands)
    const int nh = (total / nkt) * G;
    int x = bid;
    const int hd = x % nh;
    x /= nh;
    vt = __builtin_amdgcn_readfirstlane(x % nvt);
    chunk = __builtin_amdgcn_readfirstlane(x / nvt);
    gq = __builtin_amdgcn_readfirstlane(hd % G);
    bh = __builtin_amdgcn_readfirstlane(hd / G);
  } else if (ncol > 0) {
    const int L = (bid % 8) * per_xcd + bid / 8;
    if (L >= total) return;
    bh = L / nkt;
    kt = L % nkt;
  } else {
    const int nbh = total / nkt;
    if (bid < nbh) {
      bh = bid;
      kt = 0;
    } else {
      const int idx = bid - nbh;
      const int L = (idx % 8) * per_xcd + idx / 8;
      if (nkt == 1 || L >= total - nbh) return;
      bh = L / (nkt - 1);
      kt = 1 + L % (nkt - 1);
    }
  }
  const int b = bh / Hkv, hk = bh % Hkv;
  const int k0 = kt * TK, k1 = min(k0 + TK - 1, N - 1);
  const size_t kbase = ((size_t)(b * Hkv + hk) * m.ld) * D;
  // this wave's 64 keys: a quarter of the key tile, or one column group of the virtual tile;
  // lane n holds keys kw0 + n and kw0 + 32 + n
  int kw0 = k0 + wave_s * 64;
  int col_gi = 0;        // COLUMN: index of this wave's column group
  bool active = true;    // COLUMN: the virtual tile may have fewer than 4 groups
  int r0_w = 0;          // COLUMN: first row of the wave's column part
  if (COLUMN) {
    col_gi = 4 * vt + wave_s;
    active = col_gi < ncol;
    const int grp = col_list[min(col_gi, ncol - 1)];
    kw0 = 64 * grp;
    const int t1 = min((64 * grp / TK) * TK + TK - 1, N - 1);
    r0_w = (lg_qtile_window_hi(m, t1, TQ) + 1) * TQ;
  }
  const int j = kw0 + n;

  bf16x8_t kf[2][DC];
#pragma unroll
  for (int kb = 0; kb < 2; ++kb) {
    const int jk = min(j + 32 * kb, N - 1);
#pragma unroll
    for (int dc = 0; dc < DC; ++dc)
      kf[kb][dc] = lg_as_bf16x8(*reinterpret_cast<const uint4*>(k + kbase + (size_t)jk * D + dc * 16 + g * 8));
  }
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int dc = 0; dc < DC; ++dc) asm volatile("" ::"v"(kf[kb][dc]));

  // accumulators: dk of key block kb, dim block db = block kb * 4 + db; dv = block 8 + kb * 4 + db
  bf16x8_t zero8 = lg_as_bf16x8(make_uint4(0u, 0u, 0u, 0u));
  // A matrix instruction must not read a register that a vector instruction wrote just before it
  // (the compiler spaces its own; an inline one that followed the write directly read stale lanes).
  asm volatile("s_nop 15" : "+v"(zero8));
#pragma unroll
  for (int i = 0; i < 16; ++i) lg_acc_zero(i, zero8);

  int lo, hi, hq0 = hk * G, nheads = G;
  if (COLUMN) {
    // the query tiles of chunk number `chunk` (chunks are cut at fixed tile numbers for all virtual
    // tiles, counted from the chunk in which the first column part starts) that come after the
    // window part of the virtual tile's first group
    const int tf = min((64 * col_list[0] / TK) * TK + TK - 1, N - 1);
    const int c_abs = (lg_qtile_window_hi(m, tf, TQ) + 1) / LG_COL_CHUNK + chunk;
    const int grp0 = col_list[4 * vt];
    const int t1 = min((64 * grp0 / TK) * TK + TK - 1, N - 1);
    lo = max(lg_qtile_window_hi(m, t1, TQ) + 1, c_abs * LG_COL_CHUNK);
    hi = min((N - 1) / TQ, c_abs * LG_COL_CHUNK + LG_COL_CHUNK - 1);
    if (lo > hi) return;
    hq0 += gq;
    nheads = 1;
  } else if (ncol > 0) {  // the window part; the column part is the COLUMN instance's
    lo = k0 / TQ;
    hi = lg_qtile_window_hi(m, k1, TQ);
  } else {
    lg_qtile_range(m, k0, k1, TQ, &lo, &hi);
  }
  const int per_head = hi - lo + 1;
  const int steps = per_head * nheads;

  Dma dma;
  dma.init(tid);
  LgSwzReader<D> rd;
  rd.init(n, g);
  const uint32_t lds0 = (uint32_t)(uintptr_t)LG_LDS_PTR(unsigned char, smem);
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    const int r0 = COLUMN ? 64 * col_list[min(4 * vt + x, ncol - 1)] : k0 + 64 * x;
    const int rc = min(r0, N - 1);  // a tile wholly past the end repeats the last row
    dma.issue(v + kbase + (size_t)rc * D, r0 < N ? N - r0 : 1, lds0 + x * T::BYTES);
  }
  const int voff = wave * T::BYTES;  // this wave's 64 V rows

  auto issue_step = [&](int hq, int u, int buf) {
    const int q0 = u * TQ;
    const size_t row0 = (size_t)(b * Hq + hq) * N;
    const uint32_t st = lds0 + VRES + buf * STAGE;
    if (wave < 2) {  // wave 0: -lse / scale rows, wave 1: -Delta rows (64 floats each)
      const float* src = (wave == 0 ? nlse : ndelta) + row0 + min(q0 + lane, N - 1);
      lg_dma_f32x64(src, st + OFF_L + wave * 256);
    }
    const size_t urow0 = (size_t)(b * Hq + hq) * m.ld;  // the head's first row in the caller's tensors
    dma.issue(q + (urow0 + q0) * D, N - q0, st);
    dma.issue(dout + (urow0 + q0) * D, N - q0, st + OFF_G);
  };

  const int u0 = lo + (per_head - lo % per_head) % per_head;  // rotated walk, as above
  int hq_i = hq0, u_i = u0;
  int u_c = u0;
  int left_i = per_head;
  issue_step(hq_i, u_i, 0);
  for (int st = 0; st < steps; ++st) {
    const int buf = st & 1;
    LG_WAIT_VMCNT(0);
    __syncthreads();  // step st landed for everyone; everyone is done with step st-1
    if (st + 1 < steps) {
      u_i = (u_i == hi) ? lo : u_i + 1;
      if (--left_i == 0) {
        left_i = per_head;
        u_i = u0;
        ++hq_i;
      }
      issue_step(hq_i, u_i, buf ^ 1);
    }
    const int q0 = u_c * TQ;
    u_c = (u_c == hi) ? lo : u_c + 1;
    const int q1 = min(q0 + TQ - 1, N - 1);
    if (COLUMN && (!active || q0 < r0_w)) continue;  // no group, or rows of its window part
    const int kind = lg_tile_kind(m, q0, q1, kw0, kw0 + 63);
    if (kind == LG_TILE_DEAD) continue;
    const bool full = kind == LG_TILE_FULL && q0 + TQ <= N;
    const int sq = VRES + buf * STAGE, sg = sq + OFF_G;
    const float* sL = reinterpret_cast<const float*>(smem + sq + OFF_L);
    // bit 16 qb + r of bits[kb]: pair (row of register r of query block qb, key j + 32 kb) is live
    uint32_t bits[2] = {~0u, ~0u};
    if (!full) {
      if (TOKEN) {
        // in tile coordinates (row = q0 + 4g + c): key j + 32 kb is seen by the rows c with
        // lo_c <= c < lo_c + window (no upper end for a sink key), below n_c
        const int n_c = N - q0 - 4 * g;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          const int lo_c = j + 32 * kb - q0 - 4 * g;
          const long long end = j + 32 * kb < m.sink ? (long long)n_c : (long long)lo_c + m.window;
          bits[kb] = lg_reg_run(lo_c, (int)min(end, (long long)n_c));
        }
      } else {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) bits[kb] = lg_row_bits(m, j + 32 * kb, q0, g);
      }
    }
    auto dead = [&](int kb, int qb, int r) -> bool { return !((bits[kb] >> (qb * 16 + r)) & 1); };

    // One step = two 32-row query blocks (q) = 128 matrix instructions m, in pairs (units) that
    // share one operand read from LDS (one instruction for each key block); per block, m - 64 q:
    //    0..15  S  = Q K^T      16..31  dP = dO V^T      32..47  C: dV^T += dO^T P
    //   48..63  D: dK^T += Q^T dS
    // The instructions keep this order.  The LDS operand of unit u + DIST is requested before unit
    // u runs.  The vector work is cut into pieces of two elements (five instructions) and each
    // piece is placed after one matrix instruction, in whose shadow it then executes:
    //   22..29  P of rows h = 0 (both key blocks; S is final six instructions after its last one)
    //   32..39  P of rows h = 1           (C needs P of h = 0 from 32 on, of h = 1 from 40 on)
    //   40..47  dS of rows h = 0          (dP is final from 38 on; D needs dS of h = 0 from 48 on)
    //   48..55  dS of rows h = 1          (all vector work of a block ends before the next block's S)
    // S and dP start from the per-row values -lse / scale and -Delta (16 rows per lane, read from
    // LDS eight instructions before the chain starts), so P = exp2(c S') and dS = P dP'.
    f32x16_t sc[2], dp[2];
    uint32_t wP[2][2][4], wD[2][2][4];  // P / dS rounded to bf16, [key block][h][pair]
    constexpr int DIST = 2, NSL = DIST + 1;
    bf16x8_t ra[NSL], rv0[NSL], rv1[NSL];
    f32x16_t rowinit;
    auto row_init = [&](const float* base, int q) {  // register r <-> row 8 (r / 4) + 4g + r % 4 of block q
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const float4 x = *reinterpret_cast<const float4*>(base + q * 32 + 8 * r4 + 4 * g);
        rowinit[4 * r4 + 0] = x.x; rowinit[4 * r4 + 1] = x.y; rowinit[4 * r4 + 2] = x.z; rowinit[4 * r4 + 3] = x.w;
      }
    };
    auto reads = [&](int u) {  // u = 0..63: unit (m / 2) of the step
      const int sl = u % NSL, c = u & 7, q = u >> 5, ph = (u >> 3) & 3;
      if (ph == 0) {
        ra[sl] = rd.read_rows(smem, sq, q, c);
      } else if (ph == 1) {
        ra[sl] = rd.read_rows(smem, sg, q, c);
        rv0[sl] = rd.read_rows(smem, voff, 0, c);
        rv1[sl] = rd.read_rows(smem, voff, 1, c);
      } else if (ph == 2) {
        ra[sl] = rd.read_cols(smem, sg, c & 3, 2 * q + (c >> 2));  // dO^T, rows 32 q + 16 h ..
      } else {
        ra[sl] = rd.read_cols(smem, sq, c & 3, 2 * q + (c >> 2));  // Q^T
      }
    };
    // piece i (0..3) of (key block kb, half h): elements r = 8 h + 2 i, + 1
    auto sm_piece = [&](bool masked, int q, int kb, int h, int i) {
      const int r = 8 * h + 2 * i;
      float p0 = __builtin_amdgcn_exp2f(sc[kb][r] * sl2);
      float p1 = __builtin_amdgcn_exp2f(sc[kb][r + 1] * sl2);
      if (masked) {
        if (dead(kb, q, r)) p0 = 0.f;
        if (dead(kb, q, r + 1)) p1 = 0.f;
      }
      sc[kb][r] = p0;
      sc[kb][r + 1] = p1;
      wP[kb][h][i] = lg_pack_bf16(p0, p1);
    };
    auto ds_piece = [&](int kb, int h, int i) {
      const int r = 8 * h + 2 * i;
      wD[kb][h][i] = lg_pack_bf16(sc[kb][r] * dp[kb][r], sc[kb][r + 1] * dp[kb][r + 1]);
    };
    auto bop = [&](const uint32_t* w) { return lg_as_bf16x8(make_uint4(w[0], w[1], w[2], w[3])); };

    // two copies of the step: tiles that are live throughout skip the mask tests
    // Instruction numbers inside a 64-instruction block (see the table above): the chains' last
    // instructions, the anchors, and the first instruction after which each group of 8 pieces runs.
    constexpr int S_LAST = 15, DP_LAST = 31, C_FIRST = 32, D_FIRST = 48, NEXT_S = 64;
    constexpr int TIE_S = S_LAST + LG_MFMA_GAP, TIE_DP = DP_LAST + LG_MFMA_GAP;
    constexpr int P0 = 22, P1 = 32, DS0 = 40, DS1 = 48, NP = 8;  // P h0, P h1, dS h0, dS h1: NP pieces each
    static_assert(lg_readable_after(TIE_S, S_LAST) && P0 > TIE_S && P1 > TIE_S, "P reads S too early");
    static_assert(lg_readable_after(TIE_DP, DP_LAST) && DS0 > TIE_DP && DS1 > TIE_DP, "dS reads dP too early");
    static_assert(DS0 >= P0 + NP && DS1 >= P1 + NP, "dS of a half needs its P");
    // piece x of a group serves key block (x / 4) % 2; instruction C_FIRST + 8 h + 2 c' + kb reads the P of
    // (kb, h), D_FIRST + ... the dS: the last piece of key block 0 is number 3, of key block 1 number 7
    static_assert(lg_operand_ready(C_FIRST, P0 + 3) && lg_operand_ready(C_FIRST + 1, P0 + 7), "P (h0) late for dV");
    static_assert(lg_operand_ready(C_FIRST + 8, P1 + 3) && lg_operand_ready(C_FIRST + 9, P1 + 7), "P (h1) late for dV");
    static_assert(lg_operand_ready(D_FIRST, DS0 + 3) && lg_operand_ready(D_FIRST + 1, DS0 + 7), "dS (h0) late for dK");
    static_assert(lg_operand_ready(D_FIRST + 8, DS1 + 3) && lg_operand_ready(D_FIRST + 9, DS1 + 7), "dS (h1) late for dK");
    static_assert(DS1 + NP <= NEXT_S, "the vector work of a block ends before the next block's S overwrites it");
    auto run_step = [&](auto MASKED) {
    constexpr bool masked = decltype(MASKED)::value;
    __builtin_amdgcn_sched_barrier(0);
    row_init(sL, 0);
    lg_static_for<DIST>([&](auto U) { reads(decltype(U)::value); });
    lg_static_for<128>([&](auto M) {
      constexpr int m = decltype(M)::value;
      constexpr int u = m >> 1, kb = m & 1, sl = u % NSL, c = u & 7, q = m >> 6, mm = m & 63, ph = mm >> 4;
      if (kb == 0 && u + DIST < 64) reads(u + DIST);
      if (ph == 0) {
        if (c == 0) lg_mfma_vi(sc[kb], ra[sl], kf[kb][c], rowinit);
        else lg_mfma_v(sc[kb], ra[sl], kf[kb][c]);
      } else if (ph == 1) {
        if (c == 0) lg_mfma_vi(dp[kb], ra[sl], kb ? rv1[sl] : rv0[sl], rowinit);
        else lg_mfma_v(dp[kb], ra[sl], kb ? rv1[sl] : rv0[sl]);
      } else if (ph == 2) {
        lg_acc_fma(8 + 4 * kb + (c & 3), ra[sl], bop(wP[kb][c >> 2]));
      } else {
        lg_acc_fma(4 * kb + (c & 3), ra[sl], bop(wD[kb][c >> 2]));
      }
      if (mm == TIE_S) lg_tie(sc[0], sc[1]);
      if (mm == TIE_DP) lg_tie(dp[0], dp[1]);
      if (mm == 8) row_init(sL + 64, q);             // -Delta rows: dP starts at 16
      if (m == 56) row_init(sL, 1);                  // -lse / scale rows of the second block
      __builtin_amdgcn_sched_barrier(0);  // the piece follows its matrix instruction
      // pieces: P h0 at 22..29, P h1 at 32..39, dS h0 at 40..47, dS h1 at 48..55; key block = bit 2
      if (mm >= P0 && mm < P0 + NP) sm_piece(masked, q, ((mm - P0) >> 2) & 1, 0, (mm - P0) & 3);
      if (mm >= P1 && mm < P1 + NP) sm_piece(masked, q, ((mm - P1) >> 2) & 1, 1, (mm - P1) & 3);
      if (mm >= DS0 && mm < DS0 + NP) ds_piece(((mm - DS0) >> 2) & 1, 0, (mm - DS0) & 3);
      if (mm >= DS1 && mm < DS1 + NP) ds_piece(((mm - DS1) >> 2) & 1, 1, (mm - DS1) & 3);
      __builtin_amdgcn_sched_barrier(0);
    });
    };
    if (full) run_step(std::false_type{});
    else run_step(std::true_type{});
  }

  // the last matrix results must have landed before the blocks are copied out
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  if (COLUMN) {  // partial sums of the column parts, as in the 8-wave kernel
    float* tr = reinterpret_cast<float*>(smem + voff);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const int nrows = active ? min(max(N - kw0 - 32 * kb, 0), 32) : 0;
      const size_t prow = (((size_t)bh * ncol + col_gi) * 64 + kb * 32) * D;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        float akv[16], avv[16];
        lg_acc_get(kb * 4 + db, akv);
        lg_acc_get(8 + kb * 4 + db, avv);
        lg_atomic_add_block(tr, akv, part_dk + prow + db * 32, D, nrows, n, g);
        lg_atomic_add_block(tr, avv, part_dv + prow + db * 32, D, nrows, n, g);
      }
    }
    return;
  }
  const int cid = (ncol > 0 && kw0 < N) ? col_of_group[kw0 >> 6] : -1;
#pragma unroll
  for (int kb = 0; kb < 2; ++kb) {
    const int jj = j + 32 * kb;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      float akv[16], avv[16];
      lg_acc_get(kb * 4 + db, akv);
      lg_acc_get(8 + kb * 4 + db, avv);
      if (jj < N)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        float a4[4], v4[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          a4[t] = akv[4 * r4 + t];
          v4[t] = avv[4 * r4 + t];
        }
        if (cid >= 0) {  // fold in the column part's partial sums
          const size_t prow = (((size_t)bh * ncol + cid) * 64 + kb * 32 + n) * D;
          const float4 pk = *reinterpret_cast<const float4*>(part_dk + prow + db * 32 + 8 * r4 + 4 * g);
          const float4 pv = *reinterpret_cast<const float4*>(part_dv + prow + db * 32 + 8 * r4 + 4 * g);
          a4[0] += pk.x; a4[1] += pk.y; a4[2] += pk.z; a4[3] += pk.w;
          v4[0] += pv.x; v4[1] += pv.y; v4[2] += pv.z; v4[3] += pv.w;
        }
        uint2 w;
        w.x = lg_pack_bf16(a4[0] * scale, a4[1] * scale);
        w.y = lg_pack_bf16(a4[2] * scale, a4[3] * scale);
        *reinterpret_cast<uint2*>(dk + kbase + (size_t)jj * D + db * 32 + 8 * r4 + 4 * g) = w;
        w.x = lg_pack_bf16(v4[0], v4[1]);
        w.y = lg_pack_bf16(v4[2], v4[3]);
        *reinterpret_cast<uint2*>(dv + kbase + (size_t)jj * D + db * 32 + 8 * r4 + 4 * g) = w;
      }
    }
  }
}

// The column instance: one workgroup per work item.
template <bool TOKEN, bool COLUMN>
__global__ __launch_bounds__(256) void dkdv_wide_bf16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const uint16_t* __restrict__ dout, const float* __restrict__ nlse, const float* __restrict__ ndelta,
    uint16_t* __restrict__ dk, uint16_t* __restrict__ dv, int Hq, int Hkv, float scale, LgMask m,
    int nkt, int total, int per_xcd, const int* __restrict__ col_of_group, const int* __restrict__ col_list,
    float* __restrict__ part_dk, float* __restrict__ part_dv, int ncol, int nchunk) {
  dkdv_wide_item<TOKEN, COLUMN>(q, k, v, dout, nlse, ndelta, dk, dv, Hq, Hkv, scale, m, nkt, total, per_xcd,
                                col_of_group, col_list, part_dk, part_dv, ncol, nchunk, (int)blockIdx.x);
}

// The main instance: a workgroup holds a whole CU (4 x 512 registers, 130 KB of LDS), so the launch of
// the next one cannot overlap anything.  One workgroup per CU therefore stays and takes work items
// from a queue (lg_queue_take).
template <bool TOKEN>
__global__ __launch_bounds__(256) void dkdv_wide_bf16_kernel_q(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const uint16_t* __restrict__ dout, const float* __restrict__ nlse, const float* __restrict__ ndelta,
    uint16_t* __restrict__ dk, uint16_t* __restrict__ dv, int Hq, int Hkv, float scale, LgMask m,
    int nkt, int total, int per_xcd, const int* __restrict__ col_of_group, const int* __restrict__ col_list,
    float* __restrict__ part_dk, float* __restrict__ part_dv, int ncol, int nchunk, int* __restrict__ queue,
    int nitems) {
  __shared__ int s_item;
  const int xcd = blockIdx.x & 7;
  for (;;) {
    const int id = lg_queue_take(queue, nitems, xcd, &s_item);
    if (id < 0) return;
    dkdv_wide_item<TOKEN, false>(q, k, v, dout, nlse, ndelta, dk, dv, Hq, Hkv, scale, m, nkt, total, per_xcd,
                                 col_of_group, col_list, part_dk, part_dv, ncol, nchunk, id);
  }
}

// ------------------------------------------------- dq: 64 query rows per wave (D = 128)
// Same idea as the wide dk/dv kernel: four waves of 64 query rows, so that every K / V operand
// read from LDS feeds two matrix instructions; same tile walk as the 8-wave kernel, the 4-stage ring
// used as two pairs of tiles with one barrier per pair.  The AGPR half of the register file holds the dq
// accumulators (blocks 0..7 = a[0:127]: row block rb, dim block db -> block 4 rb + db) and the
// wave's Q and dO fragments (a[128:255], four registers per 32 rows x 16 dims), which the matrix
// instructions read as their second operand straight from there.
// bid: the work item, numbered like the block ids of the 8-wave kernel's grid.
template <bool TOKEN>
__device__ __forceinline__ void dq_wide_item(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const uint16_t* __restrict__ out, const uint16_t* __restrict__ dout, const float* __restrict__ lse,
    float* __restrict__ ndelta, float* __restrict__ nlse, uint16_t* __restrict__ dq, int Hq, int Hkv, float scale,
    LgMask m_in, int nqt, int total, int per_xcd, const int bid) {
  LgMask m = m_in;
  if (TOKEN) {
    m.b = 1;
    m.stride = 0;
    m.bshift = 0;
    m.smask = -1;
    m.sb = m.sink;
    m.wb = m.window;
  }
  constexpr int D = 128;
  using T = LgSwzTile<D>;
  constexpr int NT = 256, STAGES = 4;
  using Dma = LgDma<D, NT>;
  constexpr int TQ = LG_BF16_TQ, TK = LG_BF16_TK;
  static_assert(TQ == 256 && TK == 64, "4 waves x 64 query rows, 64-key tiles");
  constexpr int DC = D / 16, DB = D / 32;
  constexpr int STAGE = 2 * T::BYTES;  // K tile + V tile
  __shared__ __attribute__((aligned(1024))) unsigned char smem[STAGES * STAGE];

  const int L = (bid % 8) * per_xcd + bid / 8;
  if (L >= total) return;
  const int G = Hq / Hkv;
  const int gq = L % G, rest = L / G;
  const int qt = nqt - 1 - (rest % nqt);
  const int bhk = rest / nqt;
  const int b = bhk / Hkv, hk = bhk % Hkv;
  const int hq = hk * G + gq;
  const int N = m.N;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, g = lane >> 5;
  const int q0 = qt * TQ, q1 = min(q0 + TQ - 1, N - 1);
  const size_t qbase = ((size_t)(b * Hq + hq) * m.ld) * D;
  const uint16_t* kh = k + ((size_t)(b * Hkv + hk) * m.ld) * D;
  const uint16_t* vh = v + ((size_t)(b * Hkv + hk) * m.ld) * D;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const int qw0 = min(q0 + wave_s * 64, N - 1), qw1 = min(q0 + wave_s * 64 + 63, N - 1);  // this wave's rows
  const int i0 = q0 + wave * 64 + n;  // this lane's row of row block 0 (block 1: + 32)

  // fragments: Q of (rb, dc) -> fragment 8 rb + dc, dO -> 16 + 8 rb + dc
  float lse2[2], lse_i[2];
  f32x16_t ndl[2];  // -Delta of the lane's row in all 16 registers: the addend dP^T starts from
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    const int iq = min(i0 + 32 * rb, N - 1);
    float di = 0.f;
#pragma unroll
    for (int dc = 0; dc < DC; ++dc) {
      const uint4 gw = *reinterpret_cast<const uint4*>(dout + qbase + (size_t)iq * D + dc * 16 + g * 8);
      lg_frag_set(8 * rb + dc, *reinterpret_cast<const uint4*>(q + qbase + (size_t)iq * D + dc * 16 + g * 8));
      lg_frag_set(16 + 8 * rb + dc, gw);
      di = lg_dot8(gw, *reinterpret_cast<const uint4*>(out + qbase + (size_t)iq * D + dc * 16 + g * 8), di);
    }
    di += lg_other_half(di);  // Delta of the row
    lse_i[rb] = lse[(size_t)(b * Hq + hq) * m.ld + iq];
    lse2[rb] = lse_i[rb] * LOG2E;
#pragma unroll
    for (int r = 0; r < 16; ++r) ndl[rb][r] = -di;
  }
  const float sl2 = scale * LOG2E;
  asm volatile("" : "+v"(lse2[0]), "+v"(lse2[1]), "+v"(ndl[0]), "+v"(ndl[1]));
  {  // The rows' -Delta and -lse / scale for the dk/dv kernels.  Every lane stores, without a branch:
     // the two lanes of a row store the same values, and lanes past the end hold (and store) those
     // of row N - 1, whose data they loaded.
    const float inv_scale = 1.f / scale;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      const size_t row = (size_t)(b * Hq + hq) * N + min(i0 + 32 * rb, N - 1);
      ndelta[row] = ndl[rb][0];
      nlse[row] = -lse_i[rb] * inv_scale;
    }
  }
  bf16x8_t zero8 = lg_as_bf16x8(make_uint4(0u, 0u, 0u, 0u));
  asm volatile("s_nop 15" : "+v"(zero8));  // as in the dk/dv kernel: written well before it is read
#pragma unroll
  for (int x = 0; x < 8; ++x) lg_acc_zero(x, zero8);

  Dma dma;
  dma.init(tid);
  LgSwzReader<D> rd;
  rd.init(n, g);
  const uint32_t lds0 = (uint32_t)(uintptr_t)LG_LDS_PTR(unsigned char, smem);
  const LgQSched qs = lg_qsched_init(m, q0, q1);
  auto issue = [&](int t, int stage) {
    const size_t off = (size_t)t * TK * D;
    dma.issue(kh + off, N - t * TK, lds0 + stage * STAGE);
    dma.issue(vh + off, N - t * TK, lds0 + stage * STAGE + T::BYTES);
  };
  const LgQWalk qw = lg_qwalk_init(qs);
  auto next_tile = [&](int prev) -> int {
    if (TOKEN || m.stride == 0) return prev < 0 ? lg_qwalk_first(qw) : lg_qwalk_next(qw, prev);
    return lg_qsched_next(m, qs, prev);
  };
  // Tiles are handled in pairs: one barrier per two tiles (with one wave per SIMD nothing hides the
  // wait for the slowest wave, so fewer barriers matter more than a deeper ring).  Pair p lives in
  // stages 2 (p % 2), + 1; at its start the loads of pair p + 1 go into the other two stages.
  int t = next_tile(-1);
  int t_issue = t;
  for (int x = 0; x < 2 && t_issue >= 0; ++x) {
    issue(t_issue, x);
    t_issue = next_tile(t_issue);
  }
  int stage = 0;
  while (t >= 0) {
    if ((stage & 1) == 0) {
      LG_WAIT_VMCNT(0);
      __syncthreads();  // this pair landed for everyone; everyone is done with the previous pair
#pragma unroll
      for (int x = 0; x < 2; ++x)
        if (t_issue >= 0) {
          issue(t_issue, (stage + 2 + x) % STAGES);
          t_issue = next_tile(t_issue);
        }
    }
    const int k0 = t * TK;
    int kind = LG_TILE_FULL;
    if (!lg_qsched_full(m, qs, t)) kind = lg_tile_kind(m, qw0, qw1, k0, k0 + TK - 1);
    const int sk = stage * STAGE, sv = sk + T::BYTES;
    t = next_tile(t);
    stage = (stage + 1) % STAGES;
    if (kind == LG_TILE_DEAD) continue;
    // bit 16 kb + r of bits[rb]: pair (row i0 + 32 rb, key of register r of key block kb) is live
    uint32_t bits[2] = {~0u, ~0u};
    if (kind == LG_TILE_PARTIAL) {
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) {
        const int i = i0 + 32 * rb;
        uint32_t w = 0;
        if (TOKEN) {
          // key = k0 + 4g + c: live if inside the window of row i, or a sink key not after i
          const int hi = i - k0 - 4 * g, lo = hi - (m.window - 1), se = m.sink - k0 - 4 * g;
          w = lg_reg_run(lo, hi + 1) | lg_reg_run(-1, min(se, hi + 1));
        } else {
          w = lg_key_bits(m, min(i, N - 1), k0, g);
        }
        bits[rb] = w;
      }
    }
    auto dead = [&](int rb, int kb, int r) -> bool { return !((bits[rb] >> (kb * 16 + r)) & 1); };

    // One tile = 96 matrix instructions mi, in pairs (units) that share one operand read from LDS
    // (one instruction for each 32-row block rb):
    //    0..15  S^T(0) = K Q^T    16..31  dP^T(0) = V dO^T    32..47  S^T(1)    48..63  dP^T(1)
    //   64..79  E(0): dQ^T += K^T dS^T(0)                     80..95  E(1)
    // (0), (1): key block of the tile.  S / dP of the two key blocks use separate registers, so the
    // vector work of key block 0 runs under the instructions of key block 1, two elements after
    // each instruction:  P(0) 22..37,  dS(0) 38..53,  P(1) 54..69,  dS(1) 70..85 (rows h = 0 of
    // both row blocks first: E(1) needs them from 80 on, h = 1 from 88 on).
    f32x16_t sc[2][2], dp[2][2];   // [key block][row block]
    uint32_t wD[2][2][2][4];       // dS rounded to bf16: [key block][row block][h][pair]
    constexpr int DIST = 2, NSL = DIST + 1;
    bf16x8_t ra[NSL];
    auto reads = [&](int u) {  // u = 0..47: unit (mi / 2) of the tile
      const int sl = u % NSL, c = u & 7, ph = u >> 3;
      if (ph == 0 || ph == 2) ra[sl] = rd.read_rows(smem, sk, ph >> 1, c);
      else if (ph == 1 || ph == 3) ra[sl] = rd.read_rows(smem, sv, ph >> 1, c);
      else ra[sl] = rd.read_cols(smem, sk, c & 3, 2 * (ph - 4) + (c >> 2));
    };
    // piece x (0..15) of key block kb: row block (x / 4) % 2, h = x / 8, elements 8 h + 2 (x % 4), + 1
    auto p_piece = [&](bool masked, int kb, int x) {
      const int rb = (x >> 2) & 1, r = 8 * (x >> 3) + 2 * (x & 3);
      float p0 = __builtin_amdgcn_exp2f(fmaf(sc[kb][rb][r], sl2, -lse2[rb]));
      float p1 = __builtin_amdgcn_exp2f(fmaf(sc[kb][rb][r + 1], sl2, -lse2[rb]));
      if (masked) {
        if (dead(rb, kb, r)) p0 = 0.f;
        if (dead(rb, kb, r + 1)) p1 = 0.f;
      }
      sc[kb][rb][r] = p0;
      sc[kb][rb][r + 1] = p1;
    };
    auto ds_piece = [&](int kb, int x) {
      const int rb = (x >> 2) & 1, h = x >> 3, r = 8 * h + 2 * (x & 3);
      wD[kb][rb][h][x & 3] = lg_pack_bf16(sc[kb][rb][r] * dp[kb][rb][r], sc[kb][rb][r + 1] * dp[kb][rb][r + 1]);
    };
    auto bop = [&](const uint32_t* w) { return lg_as_bf16x8(make_uint4(w[0], w[1], w[2], w[3])); };

    // Instruction numbers of the tile (see the table above): last instruction of each chain, anchors, first
    // instruction after which each group of 16 pieces runs.
    constexpr int S0_LAST = 15, DP0_LAST = 31, S1_LAST = 47, DP1_LAST = 63, E0_FIRST = 64, E1_FIRST = 80;
    constexpr int TIE_S0 = S0_LAST + LG_MFMA_GAP, TIE_DP0 = DP0_LAST + LG_MFMA_GAP, TIE_S1 = S1_LAST + LG_MFMA_GAP,
                  TIE_DP1 = DP1_LAST + LG_MFMA_GAP;
    constexpr int PP0 = 22, DSS0 = 38, PP1 = 54, DSS1 = 70, NPC = 16;
    static_assert(lg_readable_after(TIE_S0, S0_LAST) && PP0 > TIE_S0, "P(0) reads S too early");
    static_assert(lg_readable_after(TIE_DP0, DP0_LAST) && DSS0 > TIE_DP0 && DSS0 >= PP0 + NPC, "dS(0) too early");
    static_assert(lg_readable_after(TIE_S1, S1_LAST) && PP1 > TIE_S1, "P(1) reads S too early");
    static_assert(lg_readable_after(TIE_DP1, DP1_LAST) && DSS1 > TIE_DP1 && DSS1 >= PP1 + NPC, "dS(1) too early");
    // pieces 0..7 of a dS group are h = 0 (both row blocks), 8..15 are h = 1; E(kb) reads h = 0 in its first
    // eight instructions and h = 1 in its last eight
    static_assert(lg_operand_ready(E0_FIRST, DSS0 + 7) && lg_operand_ready(E0_FIRST + 8, DSS0 + 15), "dS(0) late for dQ");
    static_assert(lg_operand_ready(E1_FIRST, DSS1 + 7) && lg_operand_ready(E1_FIRST + 8, DSS1 + 15), "dS(1) late for dQ");
    auto run_tile = [&](auto MASKED) {
      constexpr bool masked = decltype(MASKED)::value;
      __builtin_amdgcn_sched_barrier(0);
      lg_static_for<DIST>([&](auto U) { reads(decltype(U)::value); });
      lg_static_for<96>([&](auto M) {
        constexpr int mi = decltype(M)::value;
        constexpr int u = mi >> 1, rb = mi & 1, sl = u % NSL, c = u & 7, ph = u >> 3;
        if (rb == 0 && u + DIST < 48) reads(u + DIST);
        constexpr int kb = ph < 4 ? ph >> 1 : ph - 4;  // key block of the unit
        if (ph == 0 || ph == 2) lg_frag_mfma(8 * rb + c, c == 0, sc[kb][rb], ra[sl]);
        else if ((ph == 1 || ph == 3) && c == 0) lg_frag_mfma_init(16 + 8 * rb, dp[kb][rb], ra[sl], ndl[rb]);
        else if (ph == 1 || ph == 3) lg_frag_mfma(16 + 8 * rb + c, false, dp[kb][rb], ra[sl]);
        else lg_acc_fma(4 * rb + (c & 3), ra[sl], bop(wD[kb][rb][c >> 2]));
        // S / dP are final six matrix instructions after their last one
        if (mi == TIE_S0) lg_tie(sc[0][0], sc[0][1]);
        if (mi == TIE_DP0) lg_tie(dp[0][0], dp[0][1]);
        if (mi == TIE_S1) lg_tie(sc[1][0], sc[1][1]);
        if (mi == TIE_DP1) lg_tie(dp[1][0], dp[1][1]);
        __builtin_amdgcn_sched_barrier(0);  // the piece follows its matrix instruction
        if (mi >= PP0 && mi < PP0 + NPC) p_piece(masked, 0, mi - PP0);
        if (mi >= DSS0 && mi < DSS0 + NPC) ds_piece(0, mi - DSS0);
        if (mi >= PP1 && mi < PP1 + NPC) p_piece(masked, 1, mi - PP1);
        if (mi >= DSS1 && mi < DSS1 + NPC) ds_piece(1, mi - DSS1);
        __builtin_amdgcn_sched_barrier(0);
      });
    };
    if (kind == LG_TILE_FULL) run_tile(std::false_type{});
    else run_tile(std::true_type{});
  }

  // the last matrix results must have landed before the blocks are copied out
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    const int i = i0 + 32 * rb;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      float a[16];
      lg_acc_get(4 * rb + db, a);
      if (i < N)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          uint2 w;
          w.x = lg_pack_bf16(a[4 * r4 + 0] * scale, a[4 * r4 + 1] * scale);
          w.y = lg_pack_bf16(a[4 * r4 + 2] * scale, a[4 * r4 + 3] * scale);
          *reinterpret_cast<uint2*>(dq + qbase + (size_t)i * D + db * 32 + 8 * r4 + 4 * g) = w;
        }
    }
  }
}

// One resident workgroup per CU that takes its work items from a queue, as the dk/dv kernel above.
template <bool TOKEN>
__global__ __launch_bounds__(256) void dq_wide_bf16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const uint16_t* __restrict__ out, const uint16_t* __restrict__ dout, const float* __restrict__ lse,
    float* __restrict__ ndelta, float* __restrict__ nlse, uint16_t* __restrict__ dq, int Hq, int Hkv, float scale,
    LgMask m, int nqt, int total, int per_xcd, int* __restrict__ queue, int nitems) {
  __shared__ int s_item;
  const int xcd = blockIdx.x & 7;
  for (;;) {
    const int id = lg_queue_take(queue, nitems, xcd, &s_item);
    if (id < 0) return;
    dq_wide_item<TOKEN>(q, k, v, out, dout, lse, ndelta, nlse, dq, Hq, Hkv, scale, m, nqt, total, per_xcd, id);
  }
}

}  // namespace

// Workspace of the bf16 backward after Delta: two int tables of nkt entries, then the float32
// partial sums of the column tiles (dk, then dv).
namespace {
struct ColumnLayout {
  int nkt, ngroups, ncol, nchunk;  // ncol = 0: no column parts are split off
  size_t tab_off, pdk_off, pdv_off, queue_off, end;
};
ColumnLayout column_layout(const LgShape& sh, const LgMask& m, size_t head_bytes) {
  ColumnLayout c;
  c.nkt = (sh.N + LG_BF16_BTK - 1) / LG_BF16_BTK;
  c.ngroups = (sh.N + 63) / 64;
  c.ncol = 0;
  int first = -1;
  for (int grp = 0; grp < c.ngroups; ++grp)
    if (lg_is_column_group(m, grp, LG_BF16_BTK, LG_BF16_BTQ)) {
      if (first < 0) first = grp;
      ++c.ncol;
    }
  // a lone group (the sink) of a head without GQA stays with its key tile, which is launched first;
  // with G query heads per kv head that workgroup would run G times as long as everything else
  if (c.ncol < 2 && sh.Hq == sh.Hkv) c.ncol = 0;
  c.nchunk = 0;
  if (c.ncol > 0) {  // the first group has the longest column part
    const int t0 = (first * 64 / LG_BF16_BTK) * LG_BF16_BTK;
    const int t1 = (t0 + LG_BF16_BTK - 1 < sh.N - 1) ? t0 + LG_BF16_BTK - 1 : sh.N - 1;
    const int first_tile = lg_qtile_window_hi(m, t1, LG_BF16_BTQ) + 1, last_tile = (sh.N - 1) / LG_BF16_BTQ;
    c.nchunk = last_tile / LG_COL_CHUNK - first_tile / LG_COL_CHUNK + 1;  // chunks are cut at fixed tile numbers
  }
  c.tab_off = head_bytes;  // after the per-row arrays (-Delta, -lse / scale)
  const size_t tab = (((size_t)2 * c.ngroups * sizeof(int)) + 255) & ~(size_t)255;
  const size_t part = (size_t)sh.B * sh.Hkv * c.ncol * 64 * sh.D * sizeof(float);
  c.pdk_off = c.tab_off + (c.ncol > 0 ? tab : 0);
  c.pdv_off = c.pdk_off + part;
  c.queue_off = (c.pdv_off + part + 255) & ~(size_t)255;  // the work queue's counters (8 ints)
  c.end = c.queue_off + 256;
  return c;
}
}  // namespace

size_t lg_bwd_bf16_workspace_bytes(const LgShape& sh, const LgMask& m, size_t head_bytes) {
  return column_layout(sh, m, head_bytes).end;
}

hipError_t lg_launch_bwd_bf16(const void* q, const void* k, const void* v, const void* out,
                              const float* lse, const void* dout, void* dq, void* dk, void* dv,
                              void* ws, const LgShape& sh, const LgMask& m, hipStream_t s,
                              hipEvent_t* ev) {
  // workspace: -Delta | -lse / scale | column tables and partial sums.  In this form the dk/dv
  // kernels start the S and dP accumulators from them: S - lse / scale needs one multiply before
  // exp2, and dP - Delta comes out of the matrix pipe directly.
  const size_t row_bytes = (((size_t)sh.B * sh.Hq * sh.N * sizeof(float)) + 255) & ~(size_t)255;
  float* ndelta = (float*)ws;
  float* nlse = (float*)((char*)ws + row_bytes);
  // (no separate pre-pass on this path: the dq kernel forms Delta and writes both arrays; the first
  // bracket of the timing aid holds only the kernel that clears the work-queue counters)
  if (ev) (void)hipEventRecord(ev[0], s);
  hipError_t e = hipSuccess;
  const uint16_t* uo = (const uint16_t*)out;
  const uint16_t* uq = (const uint16_t*)q;
  const uint16_t* uk = (const uint16_t*)k;
  const uint16_t* uv = (const uint16_t*)v;
  const uint16_t* ug = (const uint16_t*)dout;
  const bool token = m.b == 1 && m.stride == 0;
  const ColumnLayout cl = column_layout(sh, m, 2 * row_bytes);
  // the work queues of the kernels that keep one workgroup per CU: 8 counters each, cleared per call
  int* queue = (int*)((char*)ws + cl.queue_off);
  int cus = 0;
  {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
      return hipErrorInvalidDevice;
    fill_zero_kernel<<<1, 64, 0, s>>>((float4*)queue, 4);
    if (ev) (void)hipEventRecord(ev[1], s);
  }
  {
    const int nqt = (sh.N + LG_BF16_TQ - 1) / LG_BF16_TQ;
    const long long tl = (long long)nqt * sh.Hq * sh.B;
    if (tl > 0x7fffffffLL - 8) return hipErrorInvalidValue;
    const int total = (int)tl, per_xcd = (total + 7) / 8;
    const dim3 grid(per_xcd * 8);
    // key tiles of an average query tile: its window, plus the strided columns below it
    const int col_tiles = m.stride > 0 ? (sh.N / 2) / (m.b * m.stride) * ((m.b + LG_BF16_TK - 1) / LG_BF16_TK) : 0;
    const int key_tiles = (m.wb * m.b + LG_BF16_TQ) / LG_BF16_TK + col_tiles;
#define LG_DQ_LAUNCH(DD, TT)                                                                        \
  dq_bf16_kernel<DD, TT><<<grid, 512, 0, s>>>(uq, uk, uv, uo, ug, lse, ndelta, nlse, (uint16_t*)dq, sh.Hq, \
                                              sh.Hkv, sh.scale, m, nqt, total, per_xcd)
    if (sh.D == 64) {
      if (token) LG_DQ_LAUNCH(64, true);
      else LG_DQ_LAUNCH(64, false);
    } else if (key_tiles < 16) {
      // few key tiles per query tile: the 8-wave kernel starts up and drains faster
      if (token) LG_DQ_LAUNCH(128, true);
      else LG_DQ_LAUNCH(128, false);
    } else {
      const int nitems = (int)grid.x;
      const dim3 grid_q((unsigned)(nitems < cus ? nitems : cus));
      if (token)
        dq_wide_bf16_kernel<true><<<grid_q, 256, 0, s>>>(uq, uk, uv, uo, ug, lse, ndelta, nlse, (uint16_t*)dq, sh.Hq,
                                                         sh.Hkv, sh.scale, m, nqt, total, per_xcd, queue, nitems);
      else
        dq_wide_bf16_kernel<false><<<grid_q, 256, 0, s>>>(uq, uk, uv, uo, ug, lse, ndelta, nlse, (uint16_t*)dq, sh.Hq,
                                                          sh.Hkv, sh.scale, m, nqt, total, per_xcd, queue, nitems);
    }
#undef LG_DQ_LAUNCH
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (ev) (void)hipEventRecord(ev[2], s);
  }
  {
    const int nkt = cl.nkt;
    const long long tl = (long long)nkt * sh.Hkv * sh.B;
    if (tl > 0x7fffffffLL - 8) return hipErrorInvalidValue;
    const int total = (int)tl, nbh = sh.Hkv * sh.B;
    const int per_xcd = (total + 7) / 8;
    int* col_of_group = (int*)((char*)ws + cl.tab_off);
    int* col_list = col_of_group + cl.ngroups;
    float* pdk = (float*)((char*)ws + cl.pdk_off);
    float* pdv = (float*)((char*)ws + cl.pdv_off);
#define LG_DKDV_LAUNCH(DD, TT, CC, GRID)                                                                  \
  dkdv_bf16_kernel<DD, TT, CC><<<GRID, 512, 0, s>>>(uq, uk, uv, ug, nlse, ndelta, (uint16_t*)dk,             \
                                                    (uint16_t*)dv, sh.Hq, sh.Hkv, sh.scale, m, nkt, total,  \
                                                    per_xcd, col_of_group, col_list, pdk, pdv, cl.ncol,     \
                                                    cl.nchunk)
#define LG_DKDV_BOTH(CC, GRID)                          \
  do {                                                  \
    if (sh.D == 64) {                                   \
      if (token) LG_DKDV_LAUNCH(64, true, CC, GRID);    \
      else LG_DKDV_LAUNCH(64, false, CC, GRID);         \
    } else {                                            \
      if (token) LG_DKDV_LAUNCH(128, true, CC, GRID);   \
      else LG_DKDV_LAUNCH(128, false, CC, GRID);        \
    }                                                   \
  } while (0)
    // the 64-keys-per-wave kernel pays off once a key tile has a dozen or more query tiles
    const bool wide = sh.D == 128 && (m.wb * m.b + LG_BF16_BTK) / LG_BF16_BTQ >= 16;
    if (cl.ncol > 0) {
      // list the column groups, clear their partial sums, run the column parts
      const long long ncolwg = (long long)((cl.ncol + 3) / 4) * cl.nchunk * sh.Hq * sh.B;
      if (ncolwg > 0x7fffffffLL) return hipErrorInvalidValue;
      dkdv_column_table_kernel<<<1, 1024, 0, s>>>(col_of_group, col_list, m, cl.ngroups);
      const size_t n4 = (cl.end - cl.pdk_off) / sizeof(float4);
      fill_zero_kernel<<<dim3((unsigned)((n4 + 255) / 256 < 2048 ? (n4 + 255) / 256 : 2048)), 256, 0, s>>>(
          (float4*)pdk, n4);
      const dim3 grid_col((unsigned)ncolwg);
      // column parts are long whatever the window is: the 64-keys form whenever it exists (its
      // general-predicate instance serves token-granular patterns too)
      if (sh.D == 128)
        dkdv_wide_bf16_kernel<false, true><<<grid_col, 256, 0, s>>>(
            uq, uk, uv, ug, nlse, ndelta, (uint16_t*)dk, (uint16_t*)dv, sh.Hq, sh.Hkv, sh.scale, m, nkt, total,
            per_xcd, col_of_group, col_list, pdk, pdv, cl.ncol, cl.nchunk);
      else
        LG_DKDV_BOTH(true, grid_col);
      e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
    // main instance: all items in XCD-contiguous runs, or (no split-off columns) the sink tiles first
    const int per_xcd_main = cl.ncol > 0 ? per_xcd : (total - nbh + 7) / 8;
    const dim3 grid_main(cl.ncol > 0 ? per_xcd * 8 : nbh + per_xcd_main * 8);
    {
      const int per_xcd = per_xcd_main;  // the value the kernel's mapping expects
      if (wide) {
        // one resident workgroup per CU, work items (the ids of grid_main) from the second queue
        const int nitems = (int)grid_main.x;
        const dim3 grid_q((unsigned)(nitems < cus ? nitems : cus));
        if (token)
          dkdv_wide_bf16_kernel_q<true><<<grid_q, 256, 0, s>>>(
              uq, uk, uv, ug, nlse, ndelta, (uint16_t*)dk, (uint16_t*)dv, sh.Hq, sh.Hkv, sh.scale, m, nkt, total,
              per_xcd, col_of_group, col_list, pdk, pdv, cl.ncol, cl.nchunk, queue + 8, nitems);
        else
          dkdv_wide_bf16_kernel_q<false><<<grid_q, 256, 0, s>>>(
              uq, uk, uv, ug, nlse, ndelta, (uint16_t*)dk, (uint16_t*)dv, sh.Hq, sh.Hkv, sh.scale, m, nkt, total,
              per_xcd, col_of_group, col_list, pdk, pdv, cl.ncol, cl.nchunk, queue + 8, nitems);
      } else {
        LG_DKDV_BOTH(false, grid_main);
      }
    }
#undef LG_DKDV_BOTH
#undef LG_DKDV_LAUNCH
    e = hipGetLastError();
    if (ev) (void)hipEventRecord(ev[3], s);
  }
  return e;
}
