// lg_decode.hip — decode over the sink + rolling-window KV cache (paper Section 3.2,
// second paragraph: at inference the bottleneck is loading the KV cache as fast as
// possible; the attention-sink variant keeps the window in a rolling buffer).
//
// One query per (b, hq); every valid cache slot is read exactly once.  The work is
// pure HBM streaming (about one flop per byte), so it runs on vector ALUs with
// 16-byte coalesced loads: LPR consecutive lanes read one key row, a wave reads
// 64/LPR consecutive rows per load, and U loads of K and of V are in flight per
// lane.  The slots of one (b, hkv) are split over `splits` workgroups so the chip
// is filled even for small batches; a second tiny kernel merges the partial
// (max, sum, accumulator) triples.  All query heads of a kv head are served by the
// same pass over K/V (GQA).
//
// The keys of a step are up to four runs of consecutive slots (LgDecSegs: sink tokens,
// live part of the rolling window, retained strided blocks); the kernel walks their
// concatenation.  The common case, one run starting at slot 0, has its own instance
// without the index translation.  A third instance serves paged caches with per-sequence
// context lengths: the runs are computed per sequence on the device and a slot goes through
// the sequence's page table.
//
// lg_kv_append_kernel stores new tokens into the cache rows by the same layout rule.
#include <hip/hip_bf16.h>

#include "../../include/longgen_attn.h"
#include "lg_kernels.h"
#include "lg_mask.h"

namespace {

constexpr int WAVES = 4;
#ifndef LG_DEC_U
#define LG_DEC_U 8
#endif
#ifndef LG_DEC_TARGET
#define LG_DEC_TARGET 512
#endif
constexpr int U = LG_DEC_U;  // key rows per lane group per iteration

template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}

// Sum over a group of LPR consecutive lanes (LPR in {8,16,32}); every lane of the
// group receives the total.
template <int LPR>
__device__ __forceinline__ float group_sum(float x) {
  x += dpp_f<0xB1>(x);  // quad_perm [1,0,3,2]
  x += dpp_f<0x4E>(x);  // quad_perm [2,3,0,1]
  if constexpr (LPR == 8) {
    x += dpp_f<0x141>(x);  // row_half_mirror: the other quad of the 8
  } else {
    x += dpp_f<0x124>(x);  // row_ror:4
    x += dpp_f<0x128>(x);  // row_ror:8
    if constexpr (LPR == 32) x += __shfl_xor(x, 16);
  }
  return x;
}

// E elements of T loaded as one 16-byte vector, widened to float.  The loads are marked
// non-temporal: every cache byte is used exactly once per call, so keeping it in L2 / the
// memory-side cache only evicts something else (measured: 181 -> 164 us at B16 x 32 heads x
// 4160 slots).
typedef unsigned lg_u32x4 __attribute__((ext_vector_type(4)));
typedef float lg_f32x4 __attribute__((ext_vector_type(4)));
template <typename T, int E>
struct Frag;
template <>
struct Frag<float, 4> {
  __device__ static void load(const void* p, float* f) {
    const lg_f32x4 x = __builtin_nontemporal_load(reinterpret_cast<const lg_f32x4*>(p));
    f[0] = x.x; f[1] = x.y; f[2] = x.z; f[3] = x.w;
  }
};
template <>
struct Frag<__hip_bfloat16, 8> {
  __device__ static void load(const void* p, float* f) {
    const lg_u32x4 x = __builtin_nontemporal_load(reinterpret_cast<const lg_u32x4*>(p));
    const unsigned w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      f[2 * t] = __uint_as_float(w[t] << 16);
      f[2 * t + 1] = __uint_as_float(w[t] & 0xffff0000u);
    }
  }
};

__device__ __forceinline__ void store_out(float* p, float x) { *p = x; }
__device__ __forceinline__ void store_out(__hip_bfloat16* p, float x) { *p = __float2bfloat16(x); }

// Partial record in the workspace, per (b, hq, split): D accumulators, max, sum
// (max and running values are in the log2 domain: score * scale * log2(e)).
// What a paged launch adds to the arguments.
struct LgPaged {
  const int* page_table;  // [B, pages_per_seq]
  const int* seq_lens;    // [B]
  int pages_per_seq, page_shift, n_max, num_pages;
  LgMask cm;              // cache geometry (lg_make_cache_mask), N filled in per sequence
};

enum { LG_DEC_PLAIN = 0, LG_DEC_SEGS = 1, LG_DEC_PAGED = 2 };

template <typename T, int D, int GT, int MODE>
__global__ __launch_bounds__(WAVES * 64) void decode_kernel(const T* __restrict__ q,
                                                            const T* __restrict__ kc,
                                                            const T* __restrict__ vc,
                                                            T* __restrict__ out, float* __restrict__ lse,
                                                            float* __restrict__ ws, int Hq, int Hkv,
                                                            int C, int valid, int chunk, int splits,
                                                            float scale_log2e, LgDecSegs segs, LgPaged pg) {
  constexpr int E = 16 / sizeof(T);      // elements per 16-byte lane load
  constexpr int LPR = D / E;             // lanes per key row
  constexpr int KPW = 64 / LPR;          // key rows per wave per load
  constexpr int GROUPS = WAVES * KPW;    // lane groups per workgroup
  __shared__ float sM[WAVES][GT], sL[WAVES][GT];
  __shared__ float sO[WAVES][GT][D];

  const int G = Hq / Hkv;
  const int ngc = (G + GT - 1) / GT;  // chunks of GT query heads per kv head
  const int split = blockIdx.x;
  const int hk = blockIdx.y / ngc, gc = blockIdx.y % ngc;
  const int b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int grp = wave * KPW + lane / LPR;
  const int dl = (lane % LPR) * E;  // first head-dim element of this lane
  if (MODE == LG_DEC_PAGED) {  // this sequence's own context length, key runs and share of the keys
    LgMask cm = pg.cm;
    cm.N = min(max(pg.seq_lens[b], 1), pg.n_max);
    segs = lg_decode_segments(cm);
    valid = segs.pre[segs.n];
    chunk = (valid + splits - 1) / splits;
  }
  const int s0 = split * chunk;
  const int s1 = min(valid, s0 + chunk);

  float qf[GT][E], o[GT][E], mrun[GT], lrun[GT];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    const int hq = min(hk * G + gc * GT + g, Hq - 1);
    Frag<T, E>::load(q + ((size_t)b * Hq + hq) * D + dl, qf[g]);
    mrun[g] = -INFINITY;
    lrun[g] = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      qf[g][e] *= scale_log2e;
      o[g][e] = 0.f;
    }
  }

  const T* kbase = kc + (MODE == LG_DEC_PAGED ? 0 : ((size_t)b * Hkv + hk) * C * D) + dl;
  const T* vbase = vc + (MODE == LG_DEC_PAGED ? 0 : ((size_t)b * Hkv + hk) * C * D) + dl;
  for (int base = s0; base < s1; base += GROUPS * U) {
    float kf[U][E], vf[U][E];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int key = base + u * GROUPS + grp;  // index into the concatenated runs
      ok[u] = key < s1;
      int slot = ok[u] ? key : s1 - 1;
      if (MODE != LG_DEC_PLAIN) {
        int shift = segs.start[0];
        if (slot >= segs.pre[1]) shift = segs.start[1] - segs.pre[1];
        if (slot >= segs.pre[2]) shift = segs.start[2] - segs.pre[2];
        if (slot >= segs.pre[3]) shift = segs.start[3] - segs.pre[3];
        slot += shift;
      }
      size_t off = (size_t)slot * D;
      if (MODE == LG_DEC_PAGED) {
        // (a table entry outside the pool is clamped into it: a wrong result, never a stray read)
        const int page = min(max(pg.page_table[(size_t)b * pg.pages_per_seq + (slot >> pg.page_shift)], 0),
                             pg.num_pages - 1);
        off = ((((size_t)page * Hkv + hk) << pg.page_shift) + (slot & ((1 << pg.page_shift) - 1))) * D;
      }
      Frag<T, E>::load(kbase + off, kf[u]);
      Frag<T, E>::load(vbase + off, vf[u]);
    }
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      float s[U];
      float mb = -INFINITY;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float a = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) a = fmaf(qf[g][e], kf[u][e], a);
        a = group_sum<LPR>(a);
        s[u] = ok[u] ? a : -INFINITY;
        mb = fmaxf(mb, s[u]);
      }
      const float mnew = fmaxf(mrun[g], mb);
      const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
      const float alpha = exp2f(mrun[g] - msafe);
      mrun[g] = mnew;
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < E; ++e) o[g][e] *= alpha;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float p = exp2f(s[u] - msafe);
        psum += p;
#pragma unroll
        for (int e = 0; e < E; ++e) o[g][e] = fmaf(p, vf[u][e], o[g][e]);
      }
      lrun[g] = lrun[g] * alpha + psum;
    }
  }

  // merge the KPW lane groups of the wave (lanes LPR apart hold the same dims)
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    float mall = mrun[g];
#pragma unroll
    for (int x = LPR; x < 64; x <<= 1) mall = fmaxf(mall, __shfl_xor(mall, x));
    const float msafe = (mall == -INFINITY) ? 0.f : mall;
    const float w = exp2f(mrun[g] - msafe);
    float l = lrun[g] * w;
#pragma unroll
    for (int x = LPR; x < 64; x <<= 1) l += __shfl_xor(l, x);
#pragma unroll
    for (int e = 0; e < E; ++e) {
      float a = o[g][e] * w;
#pragma unroll
      for (int x = LPR; x < 64; x <<= 1) a += __shfl_xor(a, x);
      o[g][e] = a;
    }
    if (lane < LPR) {
#pragma unroll
      for (int e = 0; e < E; ++e) sO[wave][g][dl + e] = o[g][e];
      if (lane == 0) {
        sM[wave][g] = mall;
        sL[wave][g] = l;
      }
    }
  }
  __syncthreads();

  // merge the waves; GT*D outputs spread over the workgroup
  for (int idx = threadIdx.x; idx < GT * D; idx += WAVES * 64) {
    const int g = idx / D, d = idx % D;
    const int hq = hk * G + gc * GT + g;
    if (gc * GT + g >= G) continue;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) M = fmaxf(M, sM[w][g]);
    const float Ms = (M == -INFINITY) ? 0.f : M;  // a split without keys (paged, short sequence)
    float L = 0.f, acc = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      const float f = exp2f(sM[w][g] - Ms);
      L += sL[w][g] * f;
      acc += sO[w][g][d] * f;
    }
    const size_t row = (size_t)b * Hq + hq;
    if (splits == 1) {
      store_out(out + row * D + d, acc / L);
      if (lse != nullptr && d == 0) lse[row] = (M + log2f(L)) * 0.69314718055994530942f;
    } else {
      float* rec = ws + (row * splits + split) * (D + 2);
      rec[d] = acc;
      if (d == 0) {
        rec[D] = M;
        rec[D + 1] = L;
      }
    }
  }
}

template <typename T, int D>
__global__ __launch_bounds__(D) void decode_merge_kernel(const float* __restrict__ ws,
                                                         T* __restrict__ out, float* __restrict__ lse,
                                                         int splits) {
  const size_t row = blockIdx.x;
  const int d = threadIdx.x;
  const float* rec = ws + row * splits * (D + 2);
  float M = -INFINITY;
  for (int s = 0; s < splits; ++s) M = fmaxf(M, rec[s * (D + 2) + D]);
  float L = 0.f, acc = 0.f;
  for (int s = 0; s < splits; ++s) {
    const float f = exp2f(rec[s * (D + 2) + D] - M);
    L += rec[s * (D + 2) + D + 1] * f;
    acc += rec[s * (D + 2) + d] * f;
  }
  store_out(out + row * D + d, acc / L);
  if (lse != nullptr && d == 0) lse[row] = (M + log2f(L)) * 0.69314718055994530942f;
}

// One thread per 16 bytes of a new token row (K and V): the token goes to its sink or ring
// slot unless a later token of the same call lands on that ring slot, and to its retained-block
// slot when its block is a strided column.  No two threads write the same bytes.
template <int LPR>
__global__ __launch_bounds__(256) void lg_kv_append_kernel(const uint4* __restrict__ kn,
                                                           const uint4* __restrict__ vn,
                                                           uint4* __restrict__ kc, uint4* __restrict__ vc,
                                                           int T, int pos, int slots, LgMask m) {
  const int ti = blockIdx.x * (256 / LPR) + threadIdx.x / LPR;
  if (ti >= T) return;
  const int c = threadIdx.x % LPR;
  const size_t head = (size_t)blockIdx.z * gridDim.y + blockIdx.y;
  const size_t src = (head * T + ti) * LPR + c;
  const uint4 kx = kn[src], vx = vn[src];
  const int p = pos + ti, last = pos + T - 1;
  const size_t row0 = head * slots;
  if (p < m.sink || (long long)p + m.window > last) {
    const int slot = p < m.sink ? p : m.sink + (p - m.sink) % m.window;
    kc[(row0 + slot) * LPR + c] = kx;
    vc[(row0 + slot) * LPR + c] = vx;
  }
  if (m.stride > 0) {
    const int kb = lg_div_b(m, p);
    if (lg_strided(m, kb)) {
      const int slot = m.sink + m.window + (kb / m.stride) * m.b + (p - kb * m.b);
      kc[(row0 + slot) * LPR + c] = kx;
      vc[(row0 + slot) * LPR + c] = vx;
    }
  }
}

// The same for a paged cache: per-sequence start positions, slots go through the page table.
template <int LPR>
__global__ __launch_bounds__(256) void lg_kv_paged_append_kernel(const uint4* __restrict__ kn,
                                                                 const uint4* __restrict__ vn,
                                                                 uint4* __restrict__ kp, uint4* __restrict__ vp,
                                                                 const int* __restrict__ page_table,
                                                                 const int* __restrict__ positions, int T,
                                                                 int pages_per_seq, int page_shift, int num_pages,
                                                                 LgMask m) {
  const int ti = blockIdx.x * (256 / LPR) + threadIdx.x / LPR;
  if (ti >= T) return;
  const int c = threadIdx.x % LPR;
  const int Hkv = gridDim.y, hk = blockIdx.y, b = blockIdx.z;
  const size_t src = (((size_t)b * Hkv + hk) * T + ti) * LPR + c;
  const uint4 kx = kn[src], vx = vn[src];
  const int pos = max(positions[b], 0);
  const int p = pos + ti, last = pos + T - 1;
  auto put = [&](int slot) {
    // (a table entry outside the pool is clamped into it: a misplaced row, never a stray write)
    const int page = min(max(page_table[(size_t)b * pages_per_seq + (slot >> page_shift)], 0), num_pages - 1);
    const size_t row = (((size_t)page * Hkv + hk) << page_shift) + (slot & ((1 << page_shift) - 1));
    kp[row * LPR + c] = kx;
    vp[row * LPR + c] = vx;
  };
  if (p < m.sink || (long long)p + m.window > last) put(p < m.sink ? p : m.sink + (p - m.sink) % m.window);
  if (m.stride > 0) {
    const int kb = lg_div_b(m, p);
    if (lg_strided(m, kb)) {
      const int slot = m.sink + m.window + (kb / m.stride) * m.b + (p - kb * m.b);
      if ((slot >> page_shift) < pages_per_seq) put(slot);  // positions beyond the table's reach are dropped
    }
  }
}

// ---------------------------------------------------------------- measurement aid
// The paper's decode design splits the LOADING OF THE HEAD DIMENSION across thread blocks instead
// of the cache slots (Section 3.2, second paragraph).  Read here as: block s of S loads dims
// [s*D/S, (s+1)*D/S) of every K row and produces partial scores; a second pass sums the S partial
// scores of a slot, runs the softmax and multiplies with its own dim slice of V.  K and V are
// still read once; the partial scores (S * slots floats per head) travel through the workspace.
// Kept as an A/B against the split over slots above, not used by any product entry point.
template <typename T, int D, int S>
__global__ __launch_bounds__(256) void decode_sd_scores_kernel(const T* __restrict__ q, const T* __restrict__ kc,
                                                               float* __restrict__ part, int Hq, int Hkv, int C,
                                                               int valid, float scale_log2e) {
  constexpr int E = 16 / sizeof(T), DS = D / S, LPR = DS / E, RPB = 256 / LPR;
  const int G = Hq / Hkv;
  const int s = blockIdx.y, bh = blockIdx.z, b = bh / Hkv, hk = bh % Hkv;
  const int slot = blockIdx.x * RPB + threadIdx.x / LPR;
  const int c = threadIdx.x % LPR;
  const int sl = min(slot, valid - 1);
  float kf[E];
  Frag<T, E>::load(kc + (((size_t)b * Hkv + hk) * C + sl) * D + s * DS + c * E, kf);
  for (int g = 0; g < G; ++g) {
    const int hq = hk * G + g;
    float qf[E];
    Frag<T, E>::load(q + ((size_t)b * Hq + hq) * D + s * DS + c * E, qf);
    float a = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) a = fmaf(qf[e], kf[e], a);
#pragma unroll
    for (int x = 1; x < LPR; x <<= 1) a += __shfl_xor(a, x);
    if (c == 0 && slot < valid) part[(((size_t)b * Hq + hq) * S + s) * C + slot] = a * scale_log2e;
  }
}

template <typename T, int D, int S>
__global__ __launch_bounds__(256) void decode_sd_out_kernel(const float* __restrict__ part, const T* __restrict__ vc,
                                                            T* __restrict__ out, float* __restrict__ lse, int Hq,
                                                            int Hkv, int C, int valid) {
  constexpr int E = 16 / sizeof(T), DS = D / S, LPR = DS / E, RPB = 256 / LPR;
  __shared__ float sM[RPB], sL[RPB], sO[RPB][DS];
  const int G = Hq / Hkv;
  const int s = blockIdx.x, row = blockIdx.y, b = row / Hq, hq = row % Hq, hk = hq / G;
  const int r = threadIdx.x / LPR, c = threadIdx.x % LPR;
  const float* pr = part + (size_t)row * S * C;
  const T* vb = vc + (((size_t)b * Hkv + hk) * C) * D + s * DS + c * E;
  float m = -INFINITY, l = 0.f, o[E];
#pragma unroll
  for (int e = 0; e < E; ++e) o[e] = 0.f;
  for (int slot = r; slot < valid; slot += RPB) {
    float sc = 0.f;
#pragma unroll
    for (int x = 0; x < S; ++x) sc += pr[(size_t)x * C + slot];
    float vf[E];
    Frag<T, E>::load(vb + (size_t)slot * D, vf);
    const float mn = fmaxf(m, sc);
    const float alpha = exp2f(m - mn), p = exp2f(sc - mn);
    m = mn;
    l = l * alpha + p;
#pragma unroll
    for (int e = 0; e < E; ++e) o[e] = fmaf(p, vf[e], o[e] * alpha);
  }
  if (c == 0) {
    sM[r] = m;
    sL[r] = l;
  }
#pragma unroll
  for (int e = 0; e < E; ++e) sO[r][c * E + e] = o[e];
  __syncthreads();
  for (int d = threadIdx.x; d < DS; d += 256) {
    float M = -INFINITY;
    for (int x = 0; x < RPB; ++x) M = fmaxf(M, sM[x]);
    float L = 0.f, acc = 0.f;
    for (int x = 0; x < RPB; ++x) {
      const float f = (sM[x] == -INFINITY) ? 0.f : exp2f(sM[x] - M);
      L += sL[x] * f;
      acc += sO[x][d] * f;
    }
    store_out(out + (size_t)row * D + s * DS + d, acc / L);
    if (lse != nullptr && s == 0 && d == 0) lse[row] = (M + log2f(L)) * 0.69314718055994530942f;
  }
}

template <typename T, int D>
hipError_t launch_split_headdim(const void* q, const void* kc, const void* vc, void* out, float* lse, void* ws,
                                int B, int Hq, int Hkv, int C, int valid, float scale, hipStream_t s) {
  constexpr int S = 2, E = 16 / sizeof(T), RPB = 256 / ((D / S) / E);
  const float sl2 = scale * 1.44269504088896340736f;
  decode_sd_scores_kernel<T, D, S><<<dim3((valid + RPB - 1) / RPB, S, B * Hkv), 256, 0, s>>>(
      (const T*)q, (const T*)kc, (float*)ws, Hq, Hkv, C, valid, sl2);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  decode_sd_out_kernel<T, D, S><<<dim3(S, B * Hq), 256, 0, s>>>((const float*)ws, (const T*)vc, (T*)out, lse, Hq,
                                                                Hkv, C, valid);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_typed(const void* q, const void* kc, const void* vc, void* out, float* lse, void* ws,
                        int B, int Hq, int Hkv, int C, const LgDecSegs& segs, float scale, hipStream_t s,
                        const LgPaged* paged) {
  const int valid = segs.pre[segs.n];  // paged: of the longest admissible context (sizes the split)
  const bool plain = segs.n == 1 && segs.start[0] == 0;
  LgPaged pg = {};
  if (paged) pg = *paged;
  const int G = Hq / Hkv;
  const int splits = lg_decode_splits(B, Hkv, valid);
  const int chunk = (valid + splits - 1) / splits;
  const float sl2 = scale * 1.44269504088896340736f;
  const T* tq = (const T*)q;
  const T* tk = (const T*)kc;
  const T* tv = (const T*)vc;
  T* to = (T*)out;
  float* fws = (float*)ws;
#define LG_DECODE_LAUNCH(GT)                                                                          \
  do {                                                                                                \
    const dim3 grid(splits, Hkv*((G + GT - 1) / GT), B);                                              \
    if (paged)                                                                                        \
      decode_kernel<T, D, GT, LG_DEC_PAGED><<<grid, WAVES * 64, 0, s>>>(                              \
          tq, tk, tv, to, lse, fws, Hq, Hkv, C, valid, chunk, splits, sl2, segs, pg);                 \
    else if (plain)                                                                                   \
      decode_kernel<T, D, GT, LG_DEC_PLAIN><<<grid, WAVES * 64, 0, s>>>(                              \
          tq, tk, tv, to, lse, fws, Hq, Hkv, C, valid, chunk, splits, sl2, segs, pg);                 \
    else                                                                                              \
      decode_kernel<T, D, GT, LG_DEC_SEGS><<<grid, WAVES * 64, 0, s>>>(                               \
          tq, tk, tv, to, lse, fws, Hq, Hkv, C, valid, chunk, splits, sl2, segs, pg);                 \
  } while (0)
  if (G == 1) LG_DECODE_LAUNCH(1);
  else if (G == 2) LG_DECODE_LAUNCH(2);
  else if (G <= 4) LG_DECODE_LAUNCH(4);
  else LG_DECODE_LAUNCH(8);
#undef LG_DECODE_LAUNCH
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || splits == 1) return e;
  decode_merge_kernel<T, D><<<dim3(B * Hq), D, 0, s>>>(fws, to, lse, splits);
  return hipGetLastError();
}

}  // namespace

// About two workgroups per CU (measured best at the 16 x 32 x 4160-slot workload: one
// workgroup per (b, kv head), no merge pass), at least 256 slots each
// and never an empty split.
int lg_decode_splits(int B, int Hkv, int valid) {
  const long long pairs = (long long)B * Hkv;
  long long want = (LG_DEC_TARGET + pairs - 1) / pairs;
  const long long cap = (valid + 255) / 256;
  if (want > cap) want = cap;
  if (want < 1) want = 1;
  const int chunk = (int)((valid + want - 1) / want);
  return (valid + chunk - 1) / chunk;
}

size_t lg_decode_workspace_bytes(int B, int Hq, int Hkv, int D, int valid) {
  const int splits = lg_decode_splits(B, Hkv, valid);
  if (splits == 1) return 0;
  return (size_t)B * Hq * splits * (D + 2) * sizeof(float);
}

// paged: NULL for a contiguous cache [B, Hkv, C, D]; else page table, lengths and geometry of a
// paged cache [pages, Hkv, page size, D] (C unused), segs = the runs of the longest context.
hipError_t lg_launch_decode(const void* q, const void* kc, const void* vc, void* out, float* lse,
                            void* ws, int B, int Hq, int Hkv, int C, const LgDecSegs& segs, int D,
                            int dtype, float scale, hipStream_t s, const int* page_table, const int* seq_lens,
                            int pages_per_seq, int page_shift, int n_max, const LgMask* cache_mask,
                            int num_pages) {
  LgPaged pg = {};
  const LgPaged* pp = nullptr;
  if (page_table) {
    pg.page_table = page_table;
    pg.seq_lens = seq_lens;
    pg.pages_per_seq = pages_per_seq;
    pg.page_shift = page_shift;
    pg.n_max = n_max;
    pg.num_pages = num_pages;
    pg.cm = *cache_mask;
    pp = &pg;
  }
  if (dtype == LG_F32) {
    return D == 64 ? launch_typed<float, 64>(q, kc, vc, out, lse, ws, B, Hq, Hkv, C, segs, scale, s, pp)
                   : launch_typed<float, 128>(q, kc, vc, out, lse, ws, B, Hq, Hkv, C, segs, scale, s, pp);
  }
  return D == 64
      ? launch_typed<__hip_bfloat16, 64>(q, kc, vc, out, lse, ws, B, Hq, Hkv, C, segs, scale, s, pp)
      : launch_typed<__hip_bfloat16, 128>(q, kc, vc, out, lse, ws, B, Hq, Hkv, C, segs, scale, s, pp);
}

// Workspace: S = 2 partial score rows of C floats per (b, hq).
size_t lg_decode_split_headdim_workspace_bytes(int B, int Hq, int C) { return (size_t)B * Hq * 2 * C * sizeof(float); }

hipError_t lg_launch_decode_split_headdim(const void* q, const void* kc, const void* vc, void* out, float* lse,
                                          void* ws, int B, int Hq, int Hkv, int C, int valid, int D, int dtype,
                                          float scale, hipStream_t s) {
  if (dtype == LG_F32) {
    return D == 64 ? launch_split_headdim<float, 64>(q, kc, vc, out, lse, ws, B, Hq, Hkv, C, valid, scale, s)
                   : launch_split_headdim<float, 128>(q, kc, vc, out, lse, ws, B, Hq, Hkv, C, valid, scale, s);
  }
  return D == 64
      ? launch_split_headdim<__hip_bfloat16, 64>(q, kc, vc, out, lse, ws, B, Hq, Hkv, C, valid, scale, s)
      : launch_split_headdim<__hip_bfloat16, 128>(q, kc, vc, out, lse, ws, B, Hq, Hkv, C, valid, scale, s);
}

hipError_t lg_launch_kv_paged_append(const void* k_new, const void* v_new, void* k_pages, void* v_pages,
                                     const int* page_table, const int* positions, int B, int Hkv,
                                     int row_bytes, int T, int pages_per_seq, int page_shift, int num_pages,
                                     const LgMask& m, hipStream_t s) {
  const int lpr = row_bytes / 16;
  const dim3 grid((T + 256 / lpr - 1) / (256 / lpr), Hkv, B);
  const uint4* kn = (const uint4*)k_new;
  const uint4* vn = (const uint4*)v_new;
  uint4* kp = (uint4*)k_pages;
  uint4* vp = (uint4*)v_pages;
#define LG_PA(L) lg_kv_paged_append_kernel<L><<<grid, 256, 0, s>>>(kn, vn, kp, vp, page_table, positions, T, \
                                                                   pages_per_seq, page_shift, num_pages, m)
  if (lpr == 8) LG_PA(8);
  else if (lpr == 16) LG_PA(16);
  else LG_PA(32);
#undef LG_PA
  return hipGetLastError();
}

hipError_t lg_launch_kv_append(const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                               int B, int Hkv, int row_bytes, int T, int pos, int slots,
                               const LgMask& m, hipStream_t s) {
  const int lpr = row_bytes / 16;  // 8, 16 or 32 lanes per token row
  const dim3 grid((T + 256 / lpr - 1) / (256 / lpr), Hkv, B);
  const uint4* kn = (const uint4*)k_new;
  const uint4* vn = (const uint4*)v_new;
  uint4* kc = (uint4*)k_cache;
  uint4* vc = (uint4*)v_cache;
  if (lpr == 8) lg_kv_append_kernel<8><<<grid, 256, 0, s>>>(kn, vn, kc, vc, T, pos, slots, m);
  else if (lpr == 16) lg_kv_append_kernel<16><<<grid, 256, 0, s>>>(kn, vn, kc, vc, T, pos, slots, m);
  else lg_kv_append_kernel<32><<<grid, 256, 0, s>>>(kn, vn, kc, vc, T, pos, slots, m);
  return hipGetLastError();
}
