// lg_fwd_bf16.hip — bf16 prefill forward on the gfx950 matrix cores (paper Section
// 3.2: fused online-softmax attention that never loads key tiles whose mask is zero).
//
// Workgroup = 8 wavefronts = 256 query rows of one (b, hq); wave w owns 32 rows.
// Two waves share each SIMD, so one wave's softmax (vector ALU) overlaps the other's
// matrix work.  Per live key tile (64 keys, from the closed-form scheduler in lg_mask.h):
//   S^T = K Q^T     (keys x queries): A = K rows from LDS, B = Q kept in registers
//   online softmax  on S^T: a lane holds 32 keys of ONE query, so row max / row sum
//                   are in-lane reductions plus one exchange with lane^32
//   O^T += V^T P^T  (dims x queries): A = V read from LDS through the transposing
//                   LDS load, B = P^T straight from the S^T accumulator registers
// K and V tiles travel global -> LDS directly (no registers) into a 4-stage ring;
// tiles t+1..t+3 are in flight while tile t is computed, one barrier per tile.
// Masking is applied only on PARTIAL tiles.
#include "lg_kernels.h"
#include "lg_mfma.h"
#include "lg_swz.h"

namespace {

constexpr int TK = LG_BF16_TK;  // 64 keys per step
constexpr int TQ = LG_BF16_TQ;  // 256 query rows per workgroup
constexpr int NT = TQ * 2;      // threads: one wave per 32 rows
constexpr int STAGES = 4;
static_assert(TQ == 256 && TK == 64, "8 waves x 32 rows, 64-key tiles");

// TOKEN: the pattern is token-granular without strided columns (block <= 1, stride 0).  The
// mask fields that are then known let the compiler drop the block / stride arithmetic from
// the per-tile scheduler, and partial tiles are masked with two compares per element.
// PackT: LgNoPack for the batch layout (every (b, head) has nqt query tiles of one length), LgPack for
// sequences of different lengths side by side in each head (nqt = all their query tiles; B = 1).
struct LgNoPack {};
template <int D, bool TOKEN, typename PackT>
__global__ __launch_bounds__(NT) void fwd_bf16_kernel(const uint16_t* __restrict__ q,
                                                      const uint16_t* __restrict__ k,
                                                      const uint16_t* __restrict__ v,
                                                      uint16_t* __restrict__ out,
                                                      float* __restrict__ lse, int Hq, int Hkv,
                                                      float scale_log2e, LgMask m_in, int nqt,
                                                      int total, int per_xcd, PackT pack) {
  constexpr bool PACK = !__is_same(PackT, LgNoPack);
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
  using Dma = LgDma<D, NT>;
  constexpr int DC = D / 16;            // 16-wide contraction chunks of the head dim
  constexpr int DB = D / 32;            // 32-row blocks of O^T
  constexpr int STAGE = 2 * T::BYTES;   // K tile + V tile
  constexpr int LPT = 2 * Dma::CH;      // direct loads per thread per tile
  __shared__ __attribute__((aligned(1024))) unsigned char smem[STAGES * STAGE];

  // XCD-aware order: workgroup ids are dealt round-robin to the 8 XCDs, so give
  // each XCD one contiguous run of the logical (head, query tile) sequence; its L2
  // then sees neighbouring query tiles, whose key windows overlap.
  const int L = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (L >= total) return;
  // logical order: (b, kv head) slowest, then query tile (longest rows first), then the query
  // heads of the GQA group: the G workgroups that walk the same K/V tiles run side by side
  const int G = Hq / Hkv;
  const int gq = L % G, rest = L / G;
  int qt = nqt - 1 - (rest % nqt);
  const int bhk = rest / nqt;
  const int b = bhk / Hkv, hk = bhk % Hkv;
  const int hq = hk * G + gq;
  int seq_row0 = 0;  // first row of the sequence inside its head
  if constexpr (PACK) {
    // the sequence that owns query tile qt of the launch: the last one whose first tile is <= qt
    int lo = 0, hi = pack.n;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (pack.tile0[mid] <= qt) lo = mid;
      else hi = mid;
    }
    qt -= pack.tile0[lo];
    seq_row0 = pack.row0[lo];
    m = lg_mask_for_length(m, pack.row0[lo + 1] - seq_row0);
  }
  const int N = m.N;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, g = lane >> 5;
  const int q0 = qt * TQ;
  const int q1 = min(q0 + TQ - 1, N - 1);
  const size_t qbase = ((size_t)(b * Hq + hq) * m.ld + seq_row0) * D;
  const uint16_t* kh = k + ((size_t)(b * Hkv + hk) * m.ld + seq_row0) * D;
  const uint16_t* vh = v + ((size_t)(b * Hkv + hk) * m.ld + seq_row0) * D;
  const int i = q0 + wave * 32 + n;  // this lane's query row
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const int qw0 = min(q0 + wave_s * 32, N - 1), qw1 = min(q0 + wave_s * 32 + 31, N - 1);  // this wave's rows

  // Q fragments (B operand): lane (n, g) holds dims 16*dc + 8g .. +7 of its row.
  bf16x8_t qf[DC];
  {
    const uint16_t* qr = q + qbase + (size_t)min(i, N - 1) * D + g * 8;
#pragma unroll
    for (int dc = 0; dc < DC; ++dc) qf[dc] = lg_as_bf16x8(*reinterpret_cast<const uint4*>(qr + dc * 16));
    // Touch the fragments here so that the compiler's own wait for these loads sits before
    // the tile ring starts: a wait placed inside the loop would also drain the direct loads
    // that are meant to stay in flight.
#pragma unroll
    for (int dc = 0; dc < DC; ++dc) asm volatile("" ::"v"(qf[dc]));
  }

  f32x16_t oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float mrow = -INFINITY, mref = -INFINITY, lrow = 0.f;

  Dma dma;
  dma.init(tid);
  LgSwzReader<D> rd;
  rd.init(n, g);
  const uint32_t lds0 = (uint32_t)(uintptr_t)LG_LDS_PTR(unsigned char, smem);
  const bf16x2_t ones = {(__bf16)1.0f, (__bf16)1.0f};

  auto issue = [&](int t, int stage) {
    const size_t off = (size_t)t * TK * D;
    dma.issue(kh + off, N - t * TK, lds0 + stage * STAGE);
    dma.issue(vh + off, N - t * TK, lds0 + stage * STAGE + T::BYTES);
  };

  // ring: tiles are issued up to 3 ahead of the one being computed
  const LgQSched qs = lg_qsched_init(m, q0, q1);
  // patterns without strided columns walk the window run rotated (L2 sharing between neighbours)
  const LgQWalk qw = lg_qwalk_init(qs);
  auto next_tile = [&](int prev) -> int {
    if (TOKEN || m.stride == 0) return prev < 0 ? lg_qwalk_first(qw) : lg_qwalk_next(qw, prev);
    return lg_qsched_next(m, qs, prev);
  };
  int t = next_tile(-1);  // tile to compute next
  int t_issue = t;                           // tile to issue next
  int ahead = 0;                             // tiles issued and not yet computed
  for (; ahead < STAGES - 1 && t_issue >= 0; ++ahead) {
    issue(t_issue, ahead);
    t_issue = next_tile(t_issue);
  }

  int stage = 0;  // ring position of tile t
  while (t >= 0) {
    // this wave's loads of tile t have landed once at most (ahead-1) newer tiles are pending
    if (ahead >= 3) LG_WAIT_VMCNT(2 * LPT);
    else if (ahead == 2) LG_WAIT_VMCNT(LPT);
    else LG_WAIT_VMCNT(0);
    __syncthreads();  // everyone's loads of tile t landed; everyone is done with tile t-1
    if (t_issue >= 0) {
      issue(t_issue, (stage + STAGES - 1) % STAGES);  // into the stage tile t-1 just left
      t_issue = next_tile(t_issue);
      ++ahead;
    }

    const int k0 = t * TK;
    // A tile that is not live throughout for the workgroup's 256 rows is classified again for
    // this wave's 32 rows: most waves then find it wholly live or wholly dead (they sit it out).
    int kind = LG_TILE_FULL;
    if (!lg_qsched_full(m, qs, t)) kind = lg_tile_kind(m, qw0, qw1, k0, k0 + TK - 1);
    const bool full = kind == LG_TILE_FULL;
    const int sk = stage * STAGE;   // byte offsets of the K and V tiles inside smem
    const int sv = sk + T::BYTES;
    if (kind != LG_TILE_DEAD) {

    // ---- S^T = K Q^T ----
    f32x16_t sacc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[kb][r] = 0.f;
    // The K rows are requested half a product ahead of the matrix instructions that use them (the compiler
    // on its own asks for each operand just before its use, which leaves the LDS latency in the wave's
    // critical path eight times per tile).
    {
      constexpr int HC = DC / 2;
      bf16x8_t ka[2][HC], kn[2][HC];
#pragma unroll
      for (int dc = 0; dc < HC; ++dc)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) ka[kb][dc] = rd.read_rows(smem, sk, kb, dc);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int dc = 0; dc < HC; ++dc) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) kn[kb][dc] = rd.read_rows(smem, sk, kb, HC + dc);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) sacc[kb] = lg_mfma32(ka[kb][dc], qf[dc], sacc[kb]);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int dc = 0; dc < HC; ++dc)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) sacc[kb] = lg_mfma32(kn[kb][dc], qf[HC + dc], sacc[kb]);
    }

    // ---- online softmax (log2 domain) ----
    if (!full && TOKEN) {
      // Row i sees the keys [i - window + 1, i] and the sink keys below min(sink, i + 1).  In
      // tile coordinates (key = k0 + 4g + c, c a compile-time constant per register):
      const int hi = i - k0 - 4 * g;           // c <= hi          : causal
      const int lo = hi - (m.window - 1);      // c >= lo          : inside the window
      const int se = m.sink - k0 - 4 * g;      // c < se (&& c <= hi): a sink key
      const bool has_sink = k0 < m.sink;       // wave-uniform
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int c = 32 * kb + lg_crow(r, 0);
          bool live = (unsigned)(c - lo) < (unsigned)m.window;
          if (has_sink) live |= c < se && c <= hi;
          if (!live) sacc[kb][r] = -INFINITY;
        }
    } else if (!full) {
      const uint32_t bits = lg_key_bits(m, min(i, N - 1), k0, g);  // a few runs of registers, in closed form
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (!(bits & (1u << (kb * 16 + r)))) sacc[kb][r] = -INFINITY;
    }
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; r += 2) mx = fmaxf(fmaxf(sacc[kb][r], sacc[kb][r + 1]), mx);
    mx = fmaxf(mx, lg_other_half(mx));
    // Lazy rescaling: the exponent is taken relative to a reference maximum mref that only
    // moves when the running maximum has grown by more than 2^8 (in the log2 domain), so
    // P stays below 2^8 (fine for bf16 / float32 accumulation) and the accumulator rescale is
    // skipped on almost every tile.  lse = mref*c + log2(l) holds for any reference.
    const float mnew = fmaxf(mrow, mx);
    mrow = mnew;
    const bool grow = (mnew - mref) * scale_log2e > 8.0f;  // first live tile: mref = -inf -> true
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {
      asm volatile("; rescale accumulators" ::: "memory");  // keep this a real branch
      const float alpha = (mnew == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f((mref - mnew) * scale_log2e);
      mref = mnew;
      lrow *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    }
    const float moff = (mref == -INFINITY) ? 0.f : mref * scale_log2e;
    float psum = 0.f;
    bf16x8_t pf[4];  // P^T as bf16, B operand of the second product, per 16-key group
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        uint32_t w[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          const float p0 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][8 * h + 2 * x], scale_log2e, -moff));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][8 * h + 2 * x + 1], scale_log2e, -moff));
          w[x] = lg_pack_bf16(p0, p1);
          // row sum of the ROUNDED probabilities: the same values the second product uses
          psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w[x]), ones, psum, false);
        }
        pf[2 * kb + h] = lg_as_bf16x8(make_uint4(w[0], w[1], w[2], w[3]));
      }
    lrow += psum;

    // ---- O^T += V^T P^T ----
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int db = 0; db < DB; ++db) oacc[db] = lg_mfma32(rd.read_cols(smem, sv, db, c), pf[c], oacc[db]);
    }  // kind != dead

    --ahead;
    t = next_tile(t);
    stage = (stage + 1) % STAGES;
  }

  // ---- epilogue: normalise, write O (bf16) and LSE (natural log) ----
  const float l = lrow + lg_other_half(lrow);
  const float inv = 1.f / l;
  if (i < N) {
    uint16_t* orow = out + qbase + (size_t)i * D + 4 * g;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        uint2 w;
        w.x = lg_pack_bf16(oacc[db][4 * r4 + 0] * inv, oacc[db][4 * r4 + 1] * inv);
        w.y = lg_pack_bf16(oacc[db][4 * r4 + 2] * inv, oacc[db][4 * r4 + 3] * inv);
        *reinterpret_cast<uint2*>(orow + db * 32 + 8 * r4) = w;
      }
    if (lse != nullptr && g == 0)
      lse[(size_t)(b * Hq + hq) * m.ld + seq_row0 + i] = (mref * scale_log2e + log2f(l)) * 0.69314718055994530942f;
  }
}

}  // namespace

hipError_t lg_launch_fwd_bf16(const void* q, const void* k, const void* v, void* out, float* lse,
                              const LgShape& sh, const LgMask& m, hipStream_t s) {
  const int nqt = (sh.N + TQ - 1) / TQ;
  const long long total_ll = (long long)nqt * sh.Hq * sh.B;
  if (total_ll > 0x7fffffffLL - 8) return hipErrorInvalidValue;
  const int total = (int)total_ll;
  const int per_xcd = (total + 7) / 8;
  const float sl2 = sh.scale * 1.44269504088896340736f;
  const dim3 grid(per_xcd * 8);
  const bool token = m.b == 1 && m.stride == 0;
#define LG_FWD_LAUNCH(DD, TT)                                                                            \
  fwd_bf16_kernel<DD, TT, LgNoPack><<<grid, NT, 0, s>>>((const uint16_t*)q, (const uint16_t*)k,          \
                                                        (const uint16_t*)v, (uint16_t*)out, lse, sh.Hq,  \
                                                        sh.Hkv, sl2, m, nqt, total, per_xcd, LgNoPack{})
  if (sh.D == 64) {
    if (token) LG_FWD_LAUNCH(64, true);
    else LG_FWD_LAUNCH(64, false);
  } else {
    if (token) LG_FWD_LAUNCH(128, true);
    else LG_FWD_LAUNCH(128, false);
  }
#undef LG_FWD_LAUNCH
  return hipGetLastError();
}

long long lg_fwd_bf16_pack_tiles(LgPack* pack) {
  long long t = 0;
  for (int x = 0; x < pack->n; ++x) {
    pack->tile0[x] = (int)t;
    t += (pack->row0[x + 1] - pack->row0[x] + TQ - 1) / TQ;
    if (t > 0x7fffffffLL) return -1;
  }
  pack->tile0[pack->n] = (int)t;
  return t;
}

hipError_t lg_launch_fwd_bf16_pack(const void* q, const void* k, const void* v, void* out, float* lse,
                                   const LgShape& sh, const LgMask& tmpl, const LgPack& pack, hipStream_t s) {
  const int nqt = pack.tile0[pack.n];
  const long long total_ll = (long long)nqt * sh.Hq;
  if (nqt < 1 || total_ll > 0x7fffffffLL - 8) return hipErrorInvalidValue;
  const int total = (int)total_ll;
  const int per_xcd = (total + 7) / 8;
  const float sl2 = sh.scale * 1.44269504088896340736f;
  const dim3 grid(per_xcd * 8);
  const bool token = tmpl.b == 1 && tmpl.stride == 0;
#define LG_FWD_LAUNCH(DD, TT)                                                                          \
  fwd_bf16_kernel<DD, TT, LgPack><<<grid, NT, 0, s>>>((const uint16_t*)q, (const uint16_t*)k,          \
                                                      (const uint16_t*)v, (uint16_t*)out, lse, sh.Hq,  \
                                                      sh.Hkv, sl2, tmpl, nqt, total, per_xcd, pack)
  if (sh.D == 64) {
    if (token) LG_FWD_LAUNCH(64, true);
    else LG_FWD_LAUNCH(64, false);
  } else {
    if (token) LG_FWD_LAUNCH(128, true);
    else LG_FWD_LAUNCH(128, false);
  }
#undef LG_FWD_LAUNCH
  return hipGetLastError();
}
