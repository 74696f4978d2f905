// lg_bwd_f32.hip — float32 backward (paper Section 3.2: masked key blocks are skipped
// in the backward step as well), plus the Delta pre-pass shared with the bf16 path.
//
//   Delta_i = <dout_i, out_i>
//   P_ij = exp(scale <q_i,k_j> - lse_i),  dP_ij = <dout_i, v_j>,  dS_ij = P_ij (dP_ij - Delta_i)
//   dq_i = scale sum_j dS_ij k_j        (query-tile major, same tile walk as the forward)
//   dk_j = scale sum_i dS_ij q_i,  dv_j = sum_i P_ij dout_i   (key-tile major over the
//          contiguous range of live query tiles, summed over the query heads of the group)
// Precision path for float32 data: plain FMA, no matrix cores.  4 lanes share a row
// (query row in the dq kernel, key row in the dk/dv kernel), each owning D/4 dims.
#include <hip/hip_bf16.h>

#include "../../include/longgen_attn.h"
#include "lg_kernels.h"

namespace {

constexpr int SUB = 8;

__device__ __forceinline__ float quad_sum(float a) {
  a += __shfl_xor(a, 1);
  a += __shfl_xor(a, 2);
  return a;
}

// ---------------------------------------------------------------- Delta pre-pass
__device__ __forceinline__ float dot16(const float* a, const float* b) {
  const float4 x = *reinterpret_cast<const float4*>(a), y = *reinterpret_cast<const float4*>(b);
  return x.x * y.x + x.y * y.y + x.z * y.z + x.w * y.w;
}
__device__ __forceinline__ float dot16(const __hip_bfloat16* a, const __hip_bfloat16* b) {
  const uint4 x = *reinterpret_cast<const uint4*>(a), y = *reinterpret_cast<const uint4*>(b);
  const unsigned xw[4] = {x.x, x.y, x.z, x.w}, yw[4] = {y.x, y.y, y.z, y.w};
  float s = 0.f;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    s = fmaf(__uint_as_float(xw[t] << 16), __uint_as_float(yw[t] << 16), s);
    s = fmaf(__uint_as_float(xw[t] & 0xffff0000u), __uint_as_float(yw[t] & 0xffff0000u), s);
  }
  return s;
}

// One row per LPR = D*sizeof(T)/16 lanes; rows = B*Hq*N.  delta = dsign * <dout, out>;
// lse2 (optional) = lse * lscale.  delta and lse2 are dense [B*Hq, N]; in dout, out and lse one head
// follows the other after ld rows.
template <typename T, int D>
__global__ __launch_bounds__(256) void delta_kernel(const T* __restrict__ dout, const T* __restrict__ out,
                                                    float* __restrict__ delta, const float* __restrict__ lse,
                                                    float* __restrict__ lse2, float dsign, float lscale,
                                                    long long rows, int N, int ld) {
  constexpr int E = 16 / sizeof(T);
  constexpr int LPR = D / E;
  const long long row = (long long)blockIdx.x * (256 / LPR) + threadIdx.x / LPR;
  const int c = threadIdx.x % LPR;
  long long rr = row < rows ? row : rows - 1;
  if (ld != N) rr = (rr / N) * ld + rr % N;
  float s = dot16(dout + rr * D + c * E, out + rr * D + c * E);
#pragma unroll
  for (int x = 1; x < LPR; x <<= 1) s += __shfl_xor(s, x);
  if (c == 0 && row < rows) {
    delta[row] = dsign * s;
    if (lse2) lse2[row] = lse[rr] * lscale;
  }
}

// ---------------------------------------------------------------- dq
template <int D>
__global__ __launch_bounds__(256) void dq_f32_kernel(const float* __restrict__ q, const float* __restrict__ k,
                                                     const float* __restrict__ v, const float* __restrict__ dout,
                                                     const float* __restrict__ lse,
                                                     const float* __restrict__ delta, float* __restrict__ dq,
                                                     int Hq, int Hkv, float scale, LgMask m) {
  constexpr int TQ = LG_F32_TQ, TK = LG_F32_TK, DS = D / 4;
  __shared__ float sK[TK * D];
  __shared__ float sV[TK * D];
  const int N = m.N;
  const int tid = threadIdx.x, r = tid >> 2, c = tid & 3;
  const int qt = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
  const int hk = hq / (Hq / Hkv);
  const int q0 = qt * TQ, q1 = min(q0 + TQ - 1, N - 1);
  const int i = q0 + r, iq = min(i, N - 1);
  const size_t qbase = ((size_t)(b * Hq + hq) * m.ld) * D;
  const size_t kbase = ((size_t)(b * Hkv + hk) * m.ld) * D;
  const size_t rbase = (size_t)(b * Hq + hq) * N;     // Delta (workspace, dense)
  const size_t lbase = (size_t)(b * Hq + hq) * m.ld;  // lse (caller's)

  float qr[DS], gr[DS], acc[DS];
#pragma unroll
  for (int d = 0; d < DS; ++d) {
    qr[d] = q[qbase + (size_t)iq * D + c * DS + d];
    gr[d] = dout[qbase + (size_t)iq * D + c * DS + d];
    acc[d] = 0.f;
  }
  const float li = lse[lbase + iq], di = delta[rbase + iq];

  const LgQSched qs = lg_qsched_init(m, q0, q1);
  for (int t = lg_qsched_next(m, qs, -1); t >= 0; t = lg_qsched_next(m, qs, t)) {
    const int k0 = t * TK;
    const bool full = lg_qsched_full(m, qs, t);
    __syncthreads();
    for (int e = tid * 4; e < TK * D; e += 256 * 4) {
      const int row = e / D, col = e % D;
      const int j = min(k0 + row, N - 1);
      *reinterpret_cast<float4*>(&sK[e]) = *reinterpret_cast<const float4*>(&k[kbase + (size_t)j * D + col]);
      *reinterpret_cast<float4*>(&sV[e]) = *reinterpret_cast<const float4*>(&v[kbase + (size_t)j * D + col]);
    }
    __syncthreads();
#pragma unroll 1
    for (int c0 = 0; c0 < TK; c0 += SUB) {
#pragma unroll
      for (int jj = 0; jj < SUB; ++jj) {
        const float* kr = &sK[(c0 + jj) * D + c * DS];
        const float* vr = &sV[(c0 + jj) * D + c * DS];
        float s = 0.f, dp = 0.f;
#pragma unroll
        for (int d = 0; d < DS; ++d) {
          s = fmaf(qr[d], kr[d], s);
          dp = fmaf(gr[d], vr[d], dp);
        }
        s = quad_sum(s) * scale;
        dp = quad_sum(dp);
        const bool ok = full || lg_live(m, i, k0 + c0 + jj);
        const float p = ok ? expf(s - li) : 0.f;
        const float ds = p * (dp - di);
#pragma unroll
        for (int d = 0; d < DS; ++d) acc[d] = fmaf(ds, kr[d], acc[d]);
      }
    }
  }
  if (i < N) {
#pragma unroll
    for (int d = 0; d < DS; ++d) dq[qbase + (size_t)i * D + c * DS + d] = acc[d] * scale;
  }
}

// ---------------------------------------------------------------- dk, dv
template <int D>
__global__ __launch_bounds__(256) void dkdv_f32_kernel(const float* __restrict__ q, const float* __restrict__ k,
                                                       const float* __restrict__ v,
                                                       const float* __restrict__ dout,
                                                       const float* __restrict__ lse,
                                                       const float* __restrict__ delta, float* __restrict__ dk,
                                                       float* __restrict__ dv, int Hq, int Hkv, float scale,
                                                       LgMask m) {
  constexpr int TQ = LG_F32_BTQ, TK = LG_F32_BTK, DS = D / 4;
  __shared__ float sQ[TQ * D];
  __shared__ float sG[TQ * D];
  __shared__ float sL[TQ], sD[TQ];
  const int N = m.N;
  const int tid = threadIdx.x, r = tid >> 2, c = tid & 3;
  const int kt = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
  const int G = Hq / Hkv;
  const int k0 = kt * TK, k1 = min(k0 + TK - 1, N - 1);
  const int j = k0 + r, jk = min(j, N - 1);
  const size_t kbase = ((size_t)(b * Hkv + hk) * m.ld) * D;

  float kr[DS], vr[DS], ak[DS], av[DS];
#pragma unroll
  for (int d = 0; d < DS; ++d) {
    kr[d] = k[kbase + (size_t)jk * D + c * DS + d];
    vr[d] = v[kbase + (size_t)jk * D + c * DS + d];
    ak[d] = av[d] = 0.f;
  }
  int lo, hi;
  lg_qtile_range(m, k0, k1, TQ, &lo, &hi);

  for (int gq = 0; gq < G; ++gq) {
    const int hq = hk * G + gq;
    const size_t qbase = ((size_t)(b * Hq + hq) * m.ld) * D;
    const size_t rbase = (size_t)(b * Hq + hq) * N;     // Delta (workspace, dense)
    const size_t lbase = (size_t)(b * Hq + hq) * m.ld;  // lse (caller's)
    for (int u = lo; u <= hi; ++u) {
      const int q0 = u * TQ, q1 = min(q0 + TQ - 1, N - 1);
      const bool full = lg_tile_kind(m, q0, q1, k0, k0 + TK - 1) == LG_TILE_FULL && q0 + TQ <= N;
      __syncthreads();
      for (int e = tid * 4; e < TQ * D; e += 256 * 4) {
        const int row = e / D, col = e % D;
        const int i = min(q0 + row, N - 1);
        *reinterpret_cast<float4*>(&sQ[e]) = *reinterpret_cast<const float4*>(&q[qbase + (size_t)i * D + col]);
        *reinterpret_cast<float4*>(&sG[e]) = *reinterpret_cast<const float4*>(&dout[qbase + (size_t)i * D + col]);
      }
      if (tid < TQ) {
        const int i = min(q0 + tid, N - 1);
        sL[tid] = lse[lbase + i];
        sD[tid] = delta[rbase + i];
      }
      __syncthreads();
#pragma unroll 1
      for (int c0 = 0; c0 < TQ; c0 += SUB) {
#pragma unroll
        for (int ii = 0; ii < SUB; ++ii) {
          const float* qr = &sQ[(c0 + ii) * D + c * DS];
          const float* gr = &sG[(c0 + ii) * D + c * DS];
          float s = 0.f, dp = 0.f;
#pragma unroll
          for (int d = 0; d < DS; ++d) {
            s = fmaf(qr[d], kr[d], s);
            dp = fmaf(gr[d], vr[d], dp);
          }
          s = quad_sum(s) * scale;
          dp = quad_sum(dp);
          const int i = q0 + c0 + ii;
          const bool ok = full || (i < N && lg_live(m, i, j));
          const float p = ok ? expf(s - sL[c0 + ii]) : 0.f;
          const float ds = p * (dp - sD[c0 + ii]);
#pragma unroll
          for (int d = 0; d < DS; ++d) {
            ak[d] = fmaf(ds, qr[d], ak[d]);
            av[d] = fmaf(p, gr[d], av[d]);
          }
        }
      }
    }
  }
  if (j < N) {
#pragma unroll
    for (int d = 0; d < DS; ++d) {
      dk[kbase + (size_t)j * D + c * DS + d] = ak[d] * scale;
      dv[kbase + (size_t)j * D + c * DS + d] = av[d];
    }
  }
}

template <typename T>
hipError_t launch_delta_t(const void* dout, const void* out, float* delta, const float* lse, float* lse2,
                          float dsign, float lscale, long long rows, int N, int ld, int D, hipStream_t s) {
  const int lpr = D * (int)sizeof(T) / 16;
  const int rpb = 256 / lpr;
  const unsigned grid = (unsigned)((rows + rpb - 1) / rpb);
  if (D == 64)
    delta_kernel<T, 64><<<grid, 256, 0, s>>>((const T*)dout, (const T*)out, delta, lse, lse2, dsign, lscale, rows, N, ld);
  else
    delta_kernel<T, 128><<<grid, 256, 0, s>>>((const T*)dout, (const T*)out, delta, lse, lse2, dsign, lscale, rows, N, ld);
  return hipGetLastError();
}

}  // namespace

// Delta pre-pass for either dtype (used by both backward paths).
hipError_t lg_launch_delta(const void* dout, const void* out, float* delta, const float* lse, float* lse2,
                           float dsign, float lscale, long long rows, int N, int ld, int D, int dtype,
                           hipStream_t s) {
  return dtype == LG_F32
             ? launch_delta_t<float>(dout, out, delta, lse, lse2, dsign, lscale, rows, N, ld, D, s)
             : launch_delta_t<__hip_bfloat16>(dout, out, delta, lse, lse2, dsign, lscale, rows, N, ld, D, s);
}

size_t lg_bwd_workspace_bytes(const LgShape& sh, const LgMask& m, int dtype) {
  // Delta [B, Hq, N] float32, rounded up to 256 bytes; the bf16 path adds a scaled copy of lse in the
  // same shape and its column-tile area
  const size_t n = (((size_t)sh.B * sh.Hq * sh.N * sizeof(float)) + 255) & ~(size_t)255;
  return dtype == LG_BF16 ? lg_bwd_bf16_workspace_bytes(sh, m, 2 * n) : n;
}

hipError_t lg_launch_bwd_f32(const float* q, const float* k, const float* v, const float* out,
                             const float* lse, const float* dout, float* dq, float* dk, float* dv,
                             void* ws, const LgShape& sh, const LgMask& m, hipStream_t s,
                             hipEvent_t* ev) {
  float* delta = (float*)ws;
  if (ev) (void)hipEventRecord(ev[0], s);
  hipError_t e = lg_launch_delta(dout, out, delta, nullptr, nullptr, 1.f, 0.f, (long long)sh.B * sh.Hq * sh.N, sh.N, m.ld, sh.D,
                                 LG_F32, s);
  if (e != hipSuccess) return e;
  if (ev) (void)hipEventRecord(ev[1], s);
  const dim3 gq((sh.N + LG_F32_TQ - 1) / LG_F32_TQ, sh.Hq, sh.B);
  const dim3 gk((sh.N + LG_F32_BTK - 1) / LG_F32_BTK, sh.Hkv, sh.B);
  if (sh.D == 64)
    dq_f32_kernel<64><<<gq, 256, 0, s>>>(q, k, v, dout, lse, delta, dq, sh.Hq, sh.Hkv, sh.scale, m);
  else
    dq_f32_kernel<128><<<gq, 256, 0, s>>>(q, k, v, dout, lse, delta, dq, sh.Hq, sh.Hkv, sh.scale, m);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (ev) (void)hipEventRecord(ev[2], s);
  if (sh.D == 64)
    dkdv_f32_kernel<64><<<gk, 256, 0, s>>>(q, k, v, dout, lse, delta, dk, dv, sh.Hq, sh.Hkv, sh.scale, m);
  else
    dkdv_f32_kernel<128><<<gk, 256, 0, s>>>(q, k, v, dout, lse, delta, dk, dv, sh.Hq, sh.Hkv, sh.scale, m);
  e = hipGetLastError();
  if (ev) (void)hipEventRecord(ev[3], s);
  return e;
}
