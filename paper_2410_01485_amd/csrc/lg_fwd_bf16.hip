// lg_fwd_bf16.hip — bf16 prefill forward on the gfx950 matrix cores (paper Section
// 3.2: fused online-softmax attention that never loads key tiles whose mask is zero).
//
// Workgroup = 4 wavefronts = TQ query rows of one (b, hq); wave w owns 32*QB rows.
// Per live key tile (64 keys, taken from the closed-form scheduler in lg_mask.h):
//   S^T = K Q^T     (keys x queries): A = K tile from LDS, B = Q kept in registers
//   online softmax  on S^T: a lane holds 32 keys of ONE query, so row max / row sum
//                   are in-lane reductions plus one exchange with lane^32
//   O^T += V^T P^T  (dims x queries): A = V^T from LDS, B = P^T straight from the
//                   S^T accumulator registers (no shuffle: the key order of the
//                   contraction slots is chosen to match the accumulator layout and
//                   V^T is stored in LDS in that same order)
// K and V tiles are double-buffered in LDS: the global loads of tile t+1 are issued
// before the matrix work of tile t and written to the other buffer afterwards.
// Masking is applied only on PARTIAL tiles.
#include "lg_kernels.h"
#include "lg_mfma.h"
#include "lg_stage.h"

namespace {

constexpr int TK = LG_BF16_TK;           // 64 keys per step (= LgTile::ROWS)
constexpr int QB = LG_BF16_TQ / 128;     // 32-row query blocks per wave
constexpr int TQ = LG_BF16_TQ;

template <int D>
__global__ __launch_bounds__(256, 2) void fwd_bf16_kernel(const uint16_t* __restrict__ q,
                                                       const uint16_t* __restrict__ k,
                                                       const uint16_t* __restrict__ v,
                                                       uint16_t* __restrict__ out,
                                                       float* __restrict__ lse, int Hq, int Hkv,
                                                       float scale_log2e, LgMask m, int nqt,
                                                       int total, int per_xcd) {
  using T = LgTile<D>;
  constexpr int DC = D / 16;  // 16-wide contraction chunks of the head dim
  constexpr int DB = D / 32;  // 32-row blocks of O^T
  constexpr int STAGE = T::RM_BYTES + T::T_BYTES;  // K row-major + V transposed
  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * STAGE];

  // XCD-aware order: workgroup ids are dealt round-robin to the 8 XCDs, so give
  // each XCD one contiguous run of the logical (head, query tile) sequence; its L2
  // then sees neighbouring query tiles, whose key windows overlap.
  const int L = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (L >= total) return;
  const int bh = L / nqt;
  const int qt = nqt - 1 - (L % nqt);  // longest rows first
  const int b = bh / Hq, hq = bh % Hq;
  const int hk = hq / (Hq / Hkv);
  const int N = m.N;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, g = lane >> 5;
  const int q0 = qt * TQ;
  const int q1 = min(q0 + TQ - 1, N - 1);
  const size_t qbase = ((size_t)(b * Hq + hq) * N) * D;
  const size_t kbase = ((size_t)(b * Hkv + hk) * N) * D;

  // Q fragments (B operand): lane (n, g) holds dims 16*dc + 8g .. +7 of its row.
  bf16x8_t qf[QB][DC];
  int qrow[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    qrow[qb] = q0 + (wave * QB + qb) * 32 + n;
    const int rq = min(qrow[qb], N - 1);
#pragma unroll
    for (int dc = 0; dc < DC; ++dc)
      qf[qb][dc] = lg_as_bf16x8(*reinterpret_cast<const uint4*>(q + qbase + (size_t)rq * D + dc * 16 + g * 8));
  }

  f32x16_t oacc[QB][DB];
  float mrow[QB], lrow[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    mrow[qb] = -INFINITY;
    lrow[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[qb][db][r] = 0.f;
  }

  // global -> register -> LDS staging of one K/V tile
  LgStager<D> kst, vst;
  kst.init(tid);
  vst.init(tid);
  const uint16_t* kh = k + kbase;
  const uint16_t* vh = v + kbase;
  auto load_tile = [&](int t) {
    kst.load(kh, t * TK, N);
    vst.load(vh, t * TK, N);
  };
  auto store_tile = [&](int buf) {
    kst.store_rm(smem + buf * STAGE);
    vst.store_t(smem + buf * STAGE + T::RM_BYTES);
  };

  int t = lg_next_ktile(m, q0, q1, TK, -1);
  load_tile(t);
  store_tile(0);
  __syncthreads();
  int buf = 0;

  while (t >= 0) {
    const int tn = lg_next_ktile(m, q0, q1, TK, t);
    if (tn >= 0) load_tile(tn);

    const int k0 = t * TK;
    const bool full = lg_tile_kind(m, q0, q1, k0, k0 + TK - 1) == LG_TILE_FULL;
    const unsigned char* sk = smem + buf * STAGE;
    const unsigned char* sv = sk + T::RM_BYTES;

    // ---- S^T = K Q^T ----
    f32x16_t sacc[2][QB];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[kb][qb][r] = 0.f;
#pragma unroll
    for (int dc = 0; dc < DC; ++dc) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const bf16x8_t a = lg_read_rm<D>(sk, kb, n, g, dc);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) sacc[kb][qb] = lg_mfma32(a, qf[qb][dc], sacc[kb][qb]);
      }
    }

    // ---- online softmax (log2 domain) ----
    bf16x8_t pf[QB][4];  // P^T as bf16, B operand of the second product, per 16-key chunk
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      if (!full) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int j = k0 + kb * 32 + lg_crow(r, g);
            if (!lg_live(m, qrow[qb], j)) sacc[kb][qb][r] = -INFINITY;
          }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kb][qb][r]);
      mx = fmaxf(mx, lg_other_half(mx));
      const float mnew = fmaxf(mrow[qb], mx);
      const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
      const float alpha = __builtin_amdgcn_exp2f((mrow[qb] - msafe) * scale_log2e);
      const float moff = msafe * scale_log2e;
      mrow[qb] = mnew;
      float psum = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          p[r] = __builtin_amdgcn_exp2f(fmaf(sacc[kb][qb][r], scale_log2e, -moff));
          psum += p[r];
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) pf[qb][2 * kb + h] = lg_pack_acc(p + 8 * h);
      }
      lrow[qb] = lrow[qb] * alpha + psum;
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[qb][db][r] *= alpha;
      }
    }

    // ---- O^T += V^T P^T ----
#pragma unroll
    for (int c = 0; c < 4; ++c) {
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const bf16x8_t a = lg_read_t(sv, db, n, g, c);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
          oacc[qb][db] = lg_mfma32(a, pf[qb][c], oacc[qb][db]);
      }
    }

    if (tn >= 0) store_tile(buf ^ 1);
    __syncthreads();
    buf ^= 1;
    t = tn;
  }

  // ---- epilogue: normalise, write O (bf16) and LSE (natural log) ----
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float l = lrow[qb] + lg_other_half(lrow[qb]);
    const float inv = 1.f / l;
    const int i = qrow[qb];
    if (i < N) {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          uint2 w;
          w.x = lg_pack_bf16(oacc[qb][db][4 * r4 + 0] * inv, oacc[qb][db][4 * r4 + 1] * inv);
          w.y = lg_pack_bf16(oacc[qb][db][4 * r4 + 2] * inv, oacc[qb][db][4 * r4 + 3] * inv);
          const int d = db * 32 + 8 * r4 + 4 * g;
          *reinterpret_cast<uint2*>(out + qbase + (size_t)i * D + d) = w;
        }
      if (lse != nullptr && g == 0)
        lse[(size_t)(b * Hq + hq) * N + i] =
            (mrow[qb] * scale_log2e + log2f(l)) * 0.69314718055994530942f;
    }
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
  if (sh.D == 64)
    fwd_bf16_kernel<64><<<grid, 256, 0, s>>>((const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v,
                                             (uint16_t*)out, lse, sh.Hq, sh.Hkv, sl2, m, nqt, total, per_xcd);
  else
    fwd_bf16_kernel<128><<<grid, 256, 0, s>>>((const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v,
                                              (uint16_t*)out, lse, sh.Hq, sh.Hkv, sl2, m, nqt, total, per_xcd);
  return hipGetLastError();
}
