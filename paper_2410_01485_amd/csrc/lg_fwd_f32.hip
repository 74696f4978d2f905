// lg_fwd_f32.hip — float32 prefill forward (paper Section 3.2: fused online-softmax
// attention that only visits key tiles the mask leaves live).
//
// Precision path: float32 inputs, float32 FMA dot products, float32 softmax.  The
// bf16 MFMA path cannot meet a 1e-4 bound, so float32 data takes this kernel.
// One workgroup = 64 query rows; 4 lanes share a row, each owning D/4 of the head
// dimension (partial dot products are combined with two lane exchanges).
#include "lg_kernels.h"

namespace {

constexpr int TQ = LG_F32_TQ;
constexpr int TK = LG_F32_TK;
constexpr int SUB = 8;  // keys per online-softmax step

template <int D>
__global__ __launch_bounds__(256) void fwd_f32_kernel(const float* __restrict__ q,
                                                      const float* __restrict__ k,
                                                      const float* __restrict__ v,
                                                      float* __restrict__ out, float* __restrict__ lse,
                                                      int Hq, int Hkv, float scale, LgMask m) {
  constexpr int DS = D / 4;  // head-dim slice per lane
  __shared__ float sK[TK * D];
  __shared__ float sV[TK * D];

  const int N = m.N;
  const int tid = threadIdx.x;
  const int r = tid >> 2, c = tid & 3;
  const int qt = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
  const int hk = hq / (Hq / Hkv);
  const int q0 = qt * TQ;
  const int q1 = min(q0 + TQ - 1, N - 1);
  const int i = q0 + r;             // this lane's query row
  const int iq = min(i, N - 1);     // clamped for loads
  const size_t qbase = ((size_t)(b * Hq + hq) * m.ld) * D;
  const size_t kbase = ((size_t)(b * Hkv + hk) * m.ld) * D;

  float qr[DS], o[DS];
#pragma unroll
  for (int d = 0; d < DS; ++d) {
    qr[d] = q[qbase + (size_t)iq * D + c * DS + d];
    o[d] = 0.f;
  }
  float mrow = -INFINITY, lrow = 0.f;

  const LgQSched qs = lg_qsched_init(m, q0, q1);
  for (int t = lg_qsched_next(m, qs, -1); t >= 0; t = lg_qsched_next(m, qs, t)) {
    const int k0 = t * TK;
    const bool full = lg_qsched_full(m, qs, t);
    __syncthreads();  // previous tile fully consumed
    for (int e = tid * 4; e < TK * D; e += 256 * 4) {
      const int row = e / D, col = e % D;
      const int j = min(k0 + row, N - 1);
      *reinterpret_cast<float4*>(&sK[e]) = *reinterpret_cast<const float4*>(&k[kbase + (size_t)j * D + col]);
      *reinterpret_cast<float4*>(&sV[e]) = *reinterpret_cast<const float4*>(&v[kbase + (size_t)j * D + col]);
    }
    __syncthreads();

    // the tile is consumed in sub-chunks of SUB keys, each one online-softmax step
#pragma unroll 1
    for (int c0 = 0; c0 < TK; c0 += SUB) {
      float s[SUB];
      float mt = -INFINITY;
#pragma unroll
      for (int jj = 0; jj < SUB; ++jj) {
        float a = 0.f;
#pragma unroll
        for (int d = 0; d < DS; ++d) a = fmaf(qr[d], sK[(c0 + jj) * D + c * DS + d], a);
        a += __shfl_xor(a, 1);
        a += __shfl_xor(a, 2);
        a *= scale;
        if (!full && !lg_live(m, i, k0 + c0 + jj)) a = -INFINITY;
        s[jj] = a;
        mt = fmaxf(mt, a);
      }
      const float mnew = fmaxf(mrow, mt);
      const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
      const float alpha = expf(mrow - msafe);  // mrow = -inf -> 0
      lrow *= alpha;
#pragma unroll
      for (int d = 0; d < DS; ++d) o[d] *= alpha;
#pragma unroll
      for (int jj = 0; jj < SUB; ++jj) {
        const float p = expf(s[jj] - msafe);
        lrow += p;
#pragma unroll
        for (int d = 0; d < DS; ++d) o[d] = fmaf(p, sV[(c0 + jj) * D + c * DS + d], o[d]);
      }
      mrow = mnew;
    }
  }

  if (i < N) {
    const float inv = 1.f / lrow;
#pragma unroll
    for (int d = 0; d < DS; ++d) out[qbase + (size_t)i * D + c * DS + d] = o[d] * inv;
    if (lse != nullptr && c == 0) lse[(size_t)(b * Hq + hq) * m.ld + i] = mrow + logf(lrow);
  }
}

}  // namespace

hipError_t lg_launch_fwd_f32(const float* q, const float* k, const float* v, float* out, float* lse,
                             const LgShape& sh, const LgMask& m, hipStream_t s) {
  dim3 grid((sh.N + TQ - 1) / TQ, sh.Hq, sh.B);
  if (sh.D == 64)
    fwd_f32_kernel<64><<<grid, 256, 0, s>>>(q, k, v, out, lse, sh.Hq, sh.Hkv, sh.scale, m);
  else
    fwd_f32_kernel<128><<<grid, 256, 0, s>>>(q, k, v, out, lse, sh.Hq, sh.Hkv, sh.scale, m);
  return hipGetLastError();
}
