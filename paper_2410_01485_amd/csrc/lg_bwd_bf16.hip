// lg_bwd_bf16.hip — bf16 backward on the gfx950 matrix cores (paper Section 3.2: the
// backward step skips masked key blocks just like the forward; Table 1 counts both).
//
// Two kernels after the Delta pre-pass, both free of atomics and deterministic:
//
//  dq kernel (query-tile major, same tile walk as the forward).  Per live key tile:
//     S^T  = K Q^T,  dP^T = V dO^T      (keys x queries; A = K / V row-major from LDS,
//                                        B = Q / dO fragments kept in registers)
//     P^T  = exp2(S^T c - lse_i c'),  dS^T = P^T o (dP^T - Delta_i)   (one query per lane)
//     dQ^T += K^T dS^T                  (dims x queries; A = K transposed from LDS,
//                                        B = dS^T straight from the accumulator registers)
//  dk/dv kernel (key-tile major; a wave owns 32 keys, K / V fragments in registers).
//  Per live query tile of 64 rows, for every query head of the kv group:
//     S  = Q K^T,  dP = dO V^T          (queries x keys; A = Q / dO row-major from LDS)
//     P, dS as above                    (one key per lane; lse / Delta read per row)
//     dV^T += dO^T P,  dK^T += Q^T dS   (dims x keys; A = dO / Q transposed from LDS,
//                                        B = P / dS straight from the accumulators)
// 7 tile products instead of the minimal 5: S and dP are computed in both kernels.
#include "../../include/longgen_attn.h"
#include "lg_kernels.h"
#include "lg_mfma.h"
#include "lg_stage.h"

namespace {

constexpr float LOG2E = 1.44269504088896340736f;

// ------------------------------------------------------------------------- dq
// 8 waves x 32 query rows; threads 0..255 stage K (row-major and transposed), threads
// 256..511 stage V (row-major); tiles double-buffered in LDS.
template <int D>
__global__ __launch_bounds__(512) void dq_bf16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const uint16_t* __restrict__ dout, const float* __restrict__ lse, const float* __restrict__ delta,
    uint16_t* __restrict__ dq, int Hq, int Hkv, float scale, LgMask m, int nqt, int total, int per_xcd) {
  using T = LgTile<D>;
  constexpr int TQ = LG_BF16_TQ, TK = LG_BF16_TK;
  static_assert(TQ == 256, "8 waves x 32 query rows");
  constexpr int DC = D / 16, DB = D / 32;
  constexpr int OFF_KT = T::RM_BYTES, OFF_V = T::RM_BYTES + T::T_BYTES;
  constexpr int STAGE = 2 * T::RM_BYTES + T::T_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * STAGE];

  const int L = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (L >= total) return;
  const int bh = L / nqt;
  const int qt = nqt - 1 - (L % nqt);
  const int b = bh / Hq, hq = bh % Hq;
  const int hk = hq / (Hq / Hkv);
  const int N = m.N;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, g = lane >> 5;
  const int q0 = qt * TQ, q1 = min(q0 + TQ - 1, N - 1);
  const size_t qbase = ((size_t)(b * Hq + hq) * N) * D;
  const uint16_t* kh = k + ((size_t)(b * Hkv + hk) * N) * D;
  const uint16_t* vh = v + ((size_t)(b * Hkv + hk) * N) * D;
  const int i = q0 + wave * 32 + n;
  const int iq = min(i, N - 1);

  bf16x8_t qf[DC], gf[DC];
#pragma unroll
  for (int dc = 0; dc < DC; ++dc) {
    qf[dc] = lg_as_bf16x8(*reinterpret_cast<const uint4*>(q + qbase + (size_t)iq * D + dc * 16 + g * 8));
    gf[dc] = lg_as_bf16x8(*reinterpret_cast<const uint4*>(dout + qbase + (size_t)iq * D + dc * 16 + g * 8));
  }
  const float sl2 = scale * LOG2E;
  const float lse2 = lse[(size_t)(b * Hq + hq) * N + iq] * LOG2E;
  const float di = delta[(size_t)(b * Hq + hq) * N + iq];

  f32x16_t acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

  const bool is_k = tid < 256;
  LgStager<D> st;
  st.init(tid & 255, is_k);
  LgReader<D> rd;
  rd.init(n, g);
  const uint16_t* src = is_k ? kh : vh;
  auto load_tile = [&](int t) { st.load(src + (size_t)t * TK * D, N - t * TK); };
  auto store_tile = [&](int buf) {
    unsigned char* s = smem + buf * STAGE;
    if (is_k) {
      st.store_rm(s);
      st.store_t(s + OFF_KT);
    } else {
      st.store_rm(s + OFF_V);
    }
  };

  const LgQSched qs = lg_qsched_init(m, q0, q1);
  int t = lg_qsched_next(m, qs, -1);
  load_tile(t);
  store_tile(0);
  __syncthreads();
  int buf = 0;
  while (t >= 0) {
    const int tn = lg_qsched_next(m, qs, t);
    if (tn >= 0) load_tile(tn);
    const int k0 = t * TK;
    const bool full = lg_qsched_full(m, qs, t);
    const unsigned char* s = smem + buf * STAGE;
    uint32_t bits = 0xffffffffu;
    if (!full) bits = lg_live_bits_q(m, i, k0, g);

#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      f32x16_t sc, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) sc[r] = dp[r] = 0.f;
#pragma unroll
      for (int dc = 0; dc < DC; ++dc) {
        sc = lg_mfma32(rd.read_rm(s, kb, dc), qf[dc], sc);
        dp = lg_mfma32(rd.read_rm(s + OFF_V, kb, dc), gf[dc], dp);
      }
      float ds[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float p = __builtin_amdgcn_exp2f(fmaf(sc[r], sl2, -lse2));
        if (!full && !(bits & (1u << (kb * 16 + r)))) p = 0.f;
        ds[r] = p * (dp[r] - di);
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const bf16x8_t bop = lg_pack_acc(ds + 8 * h);
#pragma unroll
        for (int db = 0; db < DB; ++db)
          acc[db] = lg_mfma32(rd.read_t(s + OFF_KT, db, 2 * kb + h), bop, acc[db]);
      }
    }
    if (tn >= 0) store_tile(buf ^ 1);
    __syncthreads();
    buf ^= 1;
    t = tn;
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
template <int D>
__global__ __launch_bounds__(256) void dkdv_bf16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const uint16_t* __restrict__ dout, const float* __restrict__ lse, const float* __restrict__ delta,
    uint16_t* __restrict__ dk, uint16_t* __restrict__ dv, int Hq, int Hkv, float scale, LgMask m,
    int nkt, int total, int per_xcd) {
  using T = LgTile<D>;
  constexpr int TQ = LG_BF16_BTQ, TK = LG_BF16_BTK;
  static_assert(TQ == 64 && TK == 128, "64 query rows per step, 32 keys per wave");
  constexpr int DC = D / 16, DB = D / 32;
  constexpr int OFF_G = T::RM_BYTES, OFF_QT = 2 * T::RM_BYTES, OFF_GT = 2 * T::RM_BYTES + T::T_BYTES;
  constexpr int OFF_L = 2 * T::RM_BYTES + 2 * T::T_BYTES;
  constexpr int STAGE = OFF_L + 2 * TQ * 4;
  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * STAGE];

  const int L = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (L >= total) return;
  const int bh = L / nkt, kt = L % nkt;  // key tile 0 (sink: longest query range) first
  const int b = bh / Hkv, hk = bh % Hkv;
  const int G = Hq / Hkv;
  const int N = m.N;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, g = lane >> 5;
  const int k0 = kt * TK, k1 = min(k0 + TK - 1, N - 1);
  const size_t kbase = ((size_t)(b * Hkv + hk) * N) * D;
  const int j = k0 + wave * 32 + n;  // this lane's key
  const int jk = min(j, N - 1);

  bf16x8_t kf[DC], vf[DC];
#pragma unroll
  for (int dc = 0; dc < DC; ++dc) {
    kf[dc] = lg_as_bf16x8(*reinterpret_cast<const uint4*>(k + kbase + (size_t)jk * D + dc * 16 + g * 8));
    vf[dc] = lg_as_bf16x8(*reinterpret_cast<const uint4*>(v + kbase + (size_t)jk * D + dc * 16 + g * 8));
  }
  f32x16_t ak[DB], av[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) ak[db][r] = av[db][r] = 0.f;
  const float sl2 = scale * LOG2E;

  int lo, hi;
  lg_qtile_range(m, k0, k1, TQ, &lo, &hi);
  const int per_head = hi - lo + 1;
  const int steps = per_head * G;

  LgStager<D> qst, gst;
  qst.init(tid, true);
  gst.init(tid, true);
  LgReader<D> rd;
  rd.init(n, g);
  float lreg = 0.f;  // threads 0..63 stage lse, 64..127 stage Delta
  auto load_step = [&](int s) {
    const int hq = hk * G + s / per_head;
    const int q0 = (lo + s % per_head) * TQ;
    const size_t qbase = ((size_t)(b * Hq + hq) * N + q0) * D;
    qst.load(q + qbase, N - q0);
    gst.load(dout + qbase, N - q0);
    if (tid < 2 * TQ) {
      const int row = min(q0 + (tid & (TQ - 1)), N - 1);
      const float* src = tid < TQ ? lse : delta;
      lreg = src[(size_t)(b * Hq + hq) * N + row];
    }
  };
  auto store_step = [&](int buf) {
    unsigned char* s = smem + buf * STAGE;
    qst.store_rm(s);
    gst.store_rm(s + OFF_G);
    qst.store_t(s + OFF_QT);
    gst.store_t(s + OFF_GT);
    if (tid < 2 * TQ) reinterpret_cast<float*>(s + OFF_L)[tid] = tid < TQ ? lreg * LOG2E : lreg;
  };

  load_step(0);
  store_step(0);
  __syncthreads();
  int buf = 0;
  for (int st = 0; st < steps; ++st) {
    if (st + 1 < steps) load_step(st + 1);
    const int q0 = (lo + st % per_head) * TQ;
    const int q1 = min(q0 + TQ - 1, N - 1);
    const bool full = lg_tile_kind(m, q0, q1, k0, k0 + TK - 1) == LG_TILE_FULL && q0 + TQ <= N;
    const unsigned char* s = smem + buf * STAGE;
    const float* sL = reinterpret_cast<const float*>(s + OFF_L);
    uint32_t bits = 0xffffffffu;
    if (!full) {
      bits = 0;
#pragma unroll 1
      for (int r = 0; r < 32; ++r) {
        const int i = q0 + (r >> 4) * 32 + lg_crow(r & 15, g);
        bits |= (uint32_t)(i < N && lg_live(m, i, j)) << r;
      }
    }

#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      f32x16_t sc, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) sc[r] = dp[r] = 0.f;
#pragma unroll
      for (int dc = 0; dc < DC; ++dc) {
        sc = lg_mfma32(rd.read_rm(s, qb, dc), kf[dc], sc);
        dp = lg_mfma32(rd.read_rm(s + OFF_G, qb, dc), vf[dc], dp);
      }
      float p[16], ds[16];
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        // rows 8*r4 + 4g .. +3 of this 32-row block: lse*log2e and Delta, 16 bytes each
        const float4 l4 = *reinterpret_cast<const float4*>(sL + qb * 32 + 8 * r4 + 4 * g);
        const float4 d4 = *reinterpret_cast<const float4*>(sL + TQ + qb * 32 + 8 * r4 + 4 * g);
        const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int r = 4 * r4 + t;
          float pv = __builtin_amdgcn_exp2f(fmaf(sc[r], sl2, -lv[t]));
          if (!full && !(bits & (1u << (qb * 16 + r)))) pv = 0.f;
          p[r] = pv;
          ds[r] = pv * (dp[r] - dv4[t]);
        }
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const bf16x8_t pb = lg_pack_acc(p + 8 * h);
        const bf16x8_t db_ = lg_pack_acc(ds + 8 * h);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          av[db] = lg_mfma32(rd.read_t(s + OFF_GT, db, 2 * qb + h), pb, av[db]);
          ak[db] = lg_mfma32(rd.read_t(s + OFF_QT, db, 2 * qb + h), db_, ak[db]);
        }
      }
    }
    if (st + 1 < steps) store_step(buf ^ 1);
    __syncthreads();
    buf ^= 1;
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

}  // namespace

hipError_t lg_launch_bwd_bf16(const void* q, const void* k, const void* v, const void* out,
                              const float* lse, const void* dout, void* dq, void* dk, void* dv,
                              void* ws, const LgShape& sh, const LgMask& m, hipStream_t s,
                              hipEvent_t* ev) {
  float* delta = (float*)ws;
  if (ev) hipEventRecord(ev[0], s);
  hipError_t e = lg_launch_delta(dout, out, delta, (long long)sh.B * sh.Hq * sh.N, sh.D, LG_BF16, s);
  if (e != hipSuccess) return e;
  if (ev) hipEventRecord(ev[1], s);
  const uint16_t* uq = (const uint16_t*)q;
  const uint16_t* uk = (const uint16_t*)k;
  const uint16_t* uv = (const uint16_t*)v;
  const uint16_t* ug = (const uint16_t*)dout;
  {
    const int nqt = (sh.N + LG_BF16_TQ - 1) / LG_BF16_TQ;
    const long long tl = (long long)nqt * sh.Hq * sh.B;
    if (tl > 0x7fffffffLL - 8) return hipErrorInvalidValue;
    const int total = (int)tl, per_xcd = (total + 7) / 8;
    if (sh.D == 64)
      dq_bf16_kernel<64><<<dim3(per_xcd * 8), 512, 0, s>>>(uq, uk, uv, ug, lse, delta, (uint16_t*)dq, sh.Hq,
                                                          sh.Hkv, sh.scale, m, nqt, total, per_xcd);
    else
      dq_bf16_kernel<128><<<dim3(per_xcd * 8), 512, 0, s>>>(uq, uk, uv, ug, lse, delta, (uint16_t*)dq, sh.Hq,
                                                           sh.Hkv, sh.scale, m, nqt, total, per_xcd);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (ev) hipEventRecord(ev[2], s);
  }
  {
    const int nkt = (sh.N + LG_BF16_BTK - 1) / LG_BF16_BTK;
    const long long tl = (long long)nkt * sh.Hkv * sh.B;
    const int total = (int)tl, per_xcd = (total + 7) / 8;
    if (sh.D == 64)
      dkdv_bf16_kernel<64><<<dim3(per_xcd * 8), 256, 0, s>>>(uq, uk, uv, ug, lse, delta, (uint16_t*)dk,
                                                            (uint16_t*)dv, sh.Hq, sh.Hkv, sh.scale, m, nkt,
                                                            total, per_xcd);
    else
      dkdv_bf16_kernel<128><<<dim3(per_xcd * 8), 256, 0, s>>>(uq, uk, uv, ug, lse, delta, (uint16_t*)dk,
                                                             (uint16_t*)dv, sh.Hq, sh.Hkv, sh.scale, m, nkt,
                                                             total, per_xcd);
    e = hipGetLastError();
    if (ev) hipEventRecord(ev[3], s);
  }
  return e;
}
