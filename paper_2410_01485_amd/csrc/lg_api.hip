// lg_api.hip — the extern "C" boundary of liblonggen_attn.so: argument checks
// (all before the first HIP call), dtype dispatch, and the host view of the tile
// scheduler.  See include/longgen_attn.h for the contract of every entry point.
#include <math.h>

#include <mutex>

#include "../../include/longgen_attn.h"
#include "lg_kernels.h"

// Scratch memory of the allocation-free decode call: one copy per GPU that loads the library, held
// until the process ends.  In host code this name is only a handle for hipGetSymbolAddress; the
// kernels receive the device address it returns, like any other workspace pointer.
static __device__ __align__(256) unsigned char lg_static_scratch[LG_DECODE_STATIC_SCRATCH_BYTES];

namespace {

// Device address of lg_static_scratch on the current device (looked up once per device, under a lock),
// or nullptr if the runtime refuses.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices];
void* static_scratch_ptr() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(lg_static_scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_common(int B, int Hq, int Hkv, int N, int D, int sink, int window, int block, int stride,
                 int dtype) {
  if (B < 1 || Hq < 1 || Hkv < 1 || N < 1 || N > (1 << 30)) return LG_ERR_INVALID_ARG;
  if (Hq % Hkv != 0) return LG_ERR_INVALID_ARG;
  if (sink < 0 || window < 1 || block < 0 || stride < 0) return LG_ERR_INVALID_ARG;
  if (block > 1 && (sink % block != 0 || window % block != 0)) return LG_ERR_INVALID_ARG;
  if (D < 1) return LG_ERR_INVALID_ARG;
  const double elems = (double)B * (double)Hq * (double)N * (double)D;
  if (elems > 1099511627776.0) return LG_ERR_INVALID_ARG;  // 2^40
  if (D != 64 && D != 128) return LG_ERR_UNSUPPORTED;
  if (dtype != LG_F32 && dtype != LG_BF16) return LG_ERR_UNSUPPORTED;
  return LG_OK;
}

LgShape make_shape(int B, int Hq, int Hkv, int N, int D, float scale) {
  LgShape sh;
  sh.B = B;
  sh.Hq = Hq;
  sh.Hkv = Hkv;
  sh.N = N;
  sh.D = D;
  sh.scale = scale > 0.0f ? scale : 1.0f / sqrtf((float)D);
  return sh;
}

}  // namespace

extern "C" {

const char* lg_status_str(int status) {
  switch (status) {
    case LG_OK: return "ok";
    case LG_ERR_NULL: return "a required pointer is NULL";
    case LG_ERR_INVALID_ARG: return "invalid argument";
    case LG_ERR_UNSUPPORTED: return "unsupported head dimension, dtype or pattern";
    case LG_ERR_WORKSPACE: return "workspace missing or too small";
    case LG_ERR_LAUNCH: return "HIP launch failed";
    default: return "unknown status";
  }
}

int lg_sparse_attn_fwd(const void* q, const void* k, const void* v, void* out, float* lse,
                       int B, int Hq, int Hkv, int N, int D,
                       int sink, int window, int block, int stride,
                       int dtype, float scale, void* hip_stream) {
  if (!q || !k || !v || !out) return LG_ERR_NULL;
  int st = check_common(B, Hq, Hkv, N, D, sink, window, block, stride, dtype);
  if (st != LG_OK) return st;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(lse))
    return LG_ERR_INVALID_ARG;
  const LgShape sh = make_shape(B, Hq, Hkv, N, D, scale);
  const LgMask m = lg_make_mask(N, sink, window, block, stride);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e = (dtype == LG_F32)
      ? lg_launch_fwd_f32((const float*)q, (const float*)k, (const float*)v, (float*)out, lse, sh, m, s)
      : lg_launch_fwd_bf16(q, k, v, out, lse, sh, m, s);
  return e == hipSuccess ? LG_OK : LG_ERR_LAUNCH;
}

size_t lg_sparse_attn_bwd_workspace_bytes(int B, int Hq, int Hkv, int N, int D,
                                          int sink, int window, int block, int stride, int dtype) {
  if (check_common(B, Hq, Hkv, N, D, sink, window, block, stride, dtype) != LG_OK) return 0;
  return lg_bwd_workspace_bytes(make_shape(B, Hq, Hkv, N, D, 0.0f),
                                lg_make_mask(N, sink, window, block, stride), dtype);
}

static int bwd_impl(const void* q, const void* k, const void* v, const void* out, const float* lse,
                    const void* dout, void* dq, void* dk, void* dv,
                    void* workspace, size_t workspace_bytes,
                    int B, int Hq, int Hkv, int N, int D,
                    int sink, int window, int block, int stride,
                    int dtype, float scale, void* hip_stream, float* kernel_ms) {
  if (!q || !k || !v || !out || !lse || !dout || !dq || !dk || !dv) return LG_ERR_NULL;
  int st = check_common(B, Hq, Hkv, N, D, sink, window, block, stride, dtype);
  if (st != LG_OK) return st;
  const void* ptrs[] = {q, k, v, out, lse, dout, dq, dk, dv, workspace};
  for (const void* p : ptrs)
    if (!aligned16(p)) return LG_ERR_INVALID_ARG;
  const LgShape sh = make_shape(B, Hq, Hkv, N, D, scale);
  const LgMask m = lg_make_mask(N, sink, window, block, stride);
  if (!workspace || workspace_bytes < lg_bwd_workspace_bytes(sh, m, dtype)) return LG_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipEvent_t evs[4];
  hipEvent_t* ev = nullptr;
  if (kernel_ms) {
    for (int x = 0; x < 4; ++x)
      if (hipEventCreate(&evs[x]) != hipSuccess) {
        while (x > 0) (void)hipEventDestroy(evs[--x]);  // the ones created so far
        return LG_ERR_LAUNCH;
      }
    ev = evs;
  }
  hipError_t e = (dtype == LG_F32)
      ? lg_launch_bwd_f32((const float*)q, (const float*)k, (const float*)v, (const float*)out, lse,
                          (const float*)dout, (float*)dq, (float*)dk, (float*)dv, workspace, sh, m, s, ev)
      : lg_launch_bwd_bf16(q, k, v, out, lse, dout, dq, dk, dv, workspace, sh, m, s, ev);
  if (kernel_ms) {
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    for (int x = 0; x < 3 && e == hipSuccess; ++x) e = hipEventElapsedTime(&kernel_ms[x], evs[x], evs[x + 1]);
    for (int x = 0; x < 4; ++x) (void)hipEventDestroy(evs[x]);
  }
  return e == hipSuccess ? LG_OK : LG_ERR_LAUNCH;
}

int lg_sparse_attn_bwd(const void* q, const void* k, const void* v, const void* out, const float* lse,
                       const void* dout, void* dq, void* dk, void* dv,
                       void* workspace, size_t workspace_bytes,
                       int B, int Hq, int Hkv, int N, int D,
                       int sink, int window, int block, int stride,
                       int dtype, float scale, void* hip_stream) {
  return bwd_impl(q, k, v, out, lse, dout, dq, dk, dv, workspace, workspace_bytes, B, Hq, Hkv, N, D, sink,
                  window, block, stride, dtype, scale, hip_stream, nullptr);
}

int lg_debug_bwd_kernel_ms(const void* q, const void* k, const void* v, const void* out, const float* lse,
                           const void* dout, void* dq, void* dk, void* dv,
                           void* workspace, size_t workspace_bytes,
                           int B, int Hq, int Hkv, int N, int D,
                           int sink, int window, int block, int stride,
                           int dtype, float scale, void* hip_stream, float* kernel_ms) {
  if (!kernel_ms) return LG_ERR_NULL;
  return bwd_impl(q, k, v, out, lse, dout, dq, dk, dv, workspace, workspace_bytes, B, Hq, Hkv, N, D, sink,
                  window, block, stride, dtype, scale, hip_stream, kernel_ms);
}

// Packed sequences of different lengths: validates cu_seqlens (host; num_seqs + 1 non-decreasing offsets
// from 0) and the common arguments for the longest sequence; *total = cu_seqlens[num_seqs], *longest =
// the longest sequence (0 when every sequence is empty).
static int check_varlen(const int* cu_seqlens, int num_seqs, int Hq, int Hkv, int D, int sink, int window,
                        int block, int stride, int dtype, int* total, int* longest) {
  if (!cu_seqlens) return LG_ERR_NULL;
  if (num_seqs < 1 || cu_seqlens[0] != 0) return LG_ERR_INVALID_ARG;
  int mx = 0;
  for (int x = 0; x < num_seqs; ++x) {
    if (cu_seqlens[x + 1] < cu_seqlens[x]) return LG_ERR_INVALID_ARG;
    const int n = cu_seqlens[x + 1] - cu_seqlens[x];
    mx = n > mx ? n : mx;
  }
  *total = cu_seqlens[num_seqs];
  *longest = mx;
  int st = check_common(1, Hq, Hkv, mx > 0 ? mx : 1, D, sink, window, block, stride, dtype);
  if (st != LG_OK) return st;
  return (double)Hq * (double)*total * (double)D > 1099511627776.0 ? LG_ERR_INVALID_ARG : LG_OK;
}

int lg_sparse_attn_fwd_varlen(const void* q, const void* k, const void* v, void* out, float* lse,
                              const int* cu_seqlens, int num_seqs, int Hq, int Hkv, int D,
                              int sink, int window, int block, int stride,
                              int dtype, float scale, void* hip_stream) {
  if (!q || !k || !v || !out) return LG_ERR_NULL;
  int T = 0, longest = 0;
  int st = check_varlen(cu_seqlens, num_seqs, Hq, Hkv, D, sink, window, block, stride, dtype, &T, &longest);
  if (st != LG_OK) return st;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(lse))
    return LG_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (dtype == LG_BF16) {
    // one launch per LG_PACK_MAX sequences: every (sequence, head, query tile) is a workgroup of the same
    // grid, so short sequences fill the GPU together
    const LgShape sh = make_shape(1, Hq, Hkv, longest > 0 ? longest : 1, D, scale);
    LgMask tmpl = lg_make_mask(1 << 30, sink, window, block, stride);  // nothing clamped to a length yet
    tmpl.ld = T;  // a head's rows of all sequences lie side by side
    int x = 0;
    while (x < num_seqs) {
      LgPack pack;
      pack.n = 0;
      for (; x < num_seqs && pack.n < LG_PACK_MAX; ++x) {
        if (cu_seqlens[x + 1] == cu_seqlens[x]) continue;
        pack.row0[pack.n] = cu_seqlens[x];
        pack.row0[pack.n + 1] = cu_seqlens[x + 1];  // the next sequence starts here unless empty ones intervene
        ++pack.n;
      }
      if (pack.n == 0) break;
      if (lg_fwd_bf16_pack_tiles(&pack) < 1) return LG_ERR_INVALID_ARG;
      if (lg_launch_fwd_bf16_pack(q, k, v, out, lse, sh, tmpl, pack, s) != hipSuccess) return LG_ERR_LAUNCH;
    }
    return LG_OK;
  }
  const size_t es = dtype == LG_F32 ? 4 : 2;
  for (int x = 0; x < num_seqs; ++x) {
    const int n = cu_seqlens[x + 1] - cu_seqlens[x];
    if (n == 0) continue;
    const LgShape sh = make_shape(1, Hq, Hkv, n, D, scale);
    LgMask m = lg_make_mask(n, sink, window, block, stride);
    m.ld = T;  // a head's rows of all sequences lie side by side
    const size_t off = (size_t)cu_seqlens[x] * D * es;
    const char* qs = (const char*)q + off;
    const char* ks = (const char*)k + off;
    const char* vs = (const char*)v + off;
    char* os = (char*)out + off;
    float* ls = lse ? lse + cu_seqlens[x] : nullptr;
    const hipError_t e = (dtype == LG_F32)
        ? lg_launch_fwd_f32((const float*)qs, (const float*)ks, (const float*)vs, (float*)os, ls, sh, m, s)
        : lg_launch_fwd_bf16(qs, ks, vs, os, ls, sh, m, s);
    if (e != hipSuccess) return LG_ERR_LAUNCH;
  }
  return LG_OK;
}

size_t lg_sparse_attn_bwd_varlen_workspace_bytes(const int* cu_seqlens, int num_seqs, int Hq, int Hkv, int D,
                                                 int sink, int window, int block, int stride, int dtype) {
  int T = 0, longest = 0;
  if (check_varlen(cu_seqlens, num_seqs, Hq, Hkv, D, sink, window, block, stride, dtype, &T, &longest) != LG_OK)
    return 0;
  size_t need = 256;  // never 0 for valid arguments: 0 is the error value
  for (int x = 0; x < num_seqs; ++x) {
    const int n = cu_seqlens[x + 1] - cu_seqlens[x];
    if (n == 0) continue;
    const size_t b = lg_bwd_workspace_bytes(make_shape(1, Hq, Hkv, n, D, 0.0f),
                                            lg_make_mask(n, sink, window, block, stride), dtype);
    need = b > need ? b : need;
  }
  return need;
}

int lg_sparse_attn_bwd_varlen(const void* q, const void* k, const void* v, const void* out, const float* lse,
                              const void* dout, void* dq, void* dk, void* dv,
                              void* workspace, size_t workspace_bytes,
                              const int* cu_seqlens, int num_seqs, int Hq, int Hkv, int D,
                              int sink, int window, int block, int stride,
                              int dtype, float scale, void* hip_stream) {
  if (!q || !k || !v || !out || !lse || !dout || !dq || !dk || !dv) return LG_ERR_NULL;
  int T = 0, longest = 0;
  int st = check_varlen(cu_seqlens, num_seqs, Hq, Hkv, D, sink, window, block, stride, dtype, &T, &longest);
  if (st != LG_OK) return st;
  const void* ptrs[] = {q, k, v, out, lse, dout, dq, dk, dv, workspace};
  for (const void* p : ptrs)
    if (!aligned16(p)) return LG_ERR_INVALID_ARG;
  if (!workspace || workspace_bytes < lg_sparse_attn_bwd_varlen_workspace_bytes(
                                          cu_seqlens, num_seqs, Hq, Hkv, D, sink, window, block, stride, dtype))
    return LG_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const size_t es = dtype == LG_F32 ? 4 : 2;
  for (int x = 0; x < num_seqs; ++x) {
    const int n = cu_seqlens[x + 1] - cu_seqlens[x];
    if (n == 0) continue;
    const LgShape sh = make_shape(1, Hq, Hkv, n, D, scale);
    LgMask m = lg_make_mask(n, sink, window, block, stride);
    m.ld = T;
    const size_t off = (size_t)cu_seqlens[x] * D * es;
    const char *qs = (const char*)q + off, *ks = (const char*)k + off, *vs = (const char*)v + off;
    const char *os = (const char*)out + off, *gs = (const char*)dout + off;
    char *dqs = (char*)dq + off, *dks = (char*)dk + off, *dvs = (char*)dv + off;
    const float* ls = lse + cu_seqlens[x];
    // the launches of one sequence follow those of the one before on the stream, so all of them
    // use the same workspace, each with the layout of its own length
    const hipError_t e = (dtype == LG_F32)
        ? lg_launch_bwd_f32((const float*)qs, (const float*)ks, (const float*)vs, (const float*)os, ls,
                            (const float*)gs, (float*)dqs, (float*)dks, (float*)dvs, workspace, sh, m, s, nullptr)
        : lg_launch_bwd_bf16(qs, ks, vs, os, ls, gs, dqs, dks, dvs, workspace, sh, m, s, nullptr);
    if (e != hipSuccess) return LG_ERR_LAUNCH;
  }
  return LG_OK;
}

static int check_decode(int B, int Hq, int Hkv, int N, int D, int sink, int window, int block,
                        int stride, int dtype) {
  int st = check_common(B, Hq, Hkv, N, D, sink, window, block, stride, dtype);
  if (st != LG_OK) return st;
  if (Hq / Hkv > 16) return LG_ERR_UNSUPPORTED;
  if ((double)sink + (double)window > 1073741824.0) return LG_ERR_INVALID_ARG;
  return LG_OK;
}

size_t lg_kv_cache_slots(int n_max, int sink, int window, int block, int stride) {
  if (check_common(1, 1, 1, n_max, 64, sink, window, block, stride, LG_F32) != LG_OK) return 0;
  if ((double)sink + (double)window > 1073741824.0) return 0;
  const long long c = lg_cache_slots(n_max, lg_make_cache_mask(n_max, sink, window, block, stride));
  return c > 0x7fffffffLL ? 0 : (size_t)c;
}

int lg_kv_ring_append(const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                      int B, int Hkv, int D, int T, int pos, int cache_slots,
                      int sink, int window, int block, int stride, int dtype, void* hip_stream) {
  if (!k_new || !v_new || !k_cache || !v_cache) return LG_ERR_NULL;
  if (T < 1 || pos < 0 || (long long)pos + T > 0x7fffffffLL) return LG_ERR_INVALID_ARG;
  int st = check_common(B, Hkv, Hkv, pos + T, D, sink, window, block, stride, dtype);
  if (st != LG_OK) return st;
  const size_t need = lg_kv_cache_slots(pos + T, sink, window, block, stride);
  if (need == 0 || cache_slots < 0 || (size_t)cache_slots < need) return LG_ERR_INVALID_ARG;
  if ((double)B * Hkv * (double)cache_slots * D > 1099511627776.0) return LG_ERR_INVALID_ARG;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache))
    return LG_ERR_INVALID_ARG;
  const LgMask m = lg_make_cache_mask(pos + T, sink, window, block, stride);
  const int row_bytes = D * (dtype == LG_F32 ? 4 : 2);
  hipError_t e = lg_launch_kv_append(k_new, v_new, k_cache, v_cache, B, Hkv, row_bytes, T, pos, cache_slots,
                                     m, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? LG_OK : LG_ERR_LAUNCH;
}

size_t lg_sparse_attn_decode_cache_workspace_bytes(int B, int Hq, int Hkv, int N, int D,
                                                   int sink, int window, int block, int stride, int dtype) {
  if (check_decode(B, Hq, Hkv, N, D, sink, window, block, stride, dtype) != LG_OK) return 0;
  const LgDecSegs g = lg_decode_segments(lg_make_cache_mask(N, sink, window, block, stride));
  return lg_decode_workspace_bytes(B, Hq, Hkv, D, g.pre[g.n]);
}

int lg_sparse_attn_decode_cache(const void* q, const void* k_cache, const void* v_cache, void* out,
                                float* lse, void* workspace, size_t workspace_bytes,
                                int B, int Hq, int Hkv, int N, int D,
                                int sink, int window, int block, int stride, int cache_slots,
                                int dtype, float scale, void* hip_stream) {
  if (!q || !k_cache || !v_cache || !out) return LG_ERR_NULL;
  int st = check_decode(B, Hq, Hkv, N, D, sink, window, block, stride, dtype);
  if (st != LG_OK) return st;
  const size_t slots_needed = lg_kv_cache_slots(N, sink, window, block, stride);
  if (slots_needed == 0 || cache_slots < 0 || (size_t)cache_slots < slots_needed) return LG_ERR_INVALID_ARG;
  if ((double)B * Hkv * (double)cache_slots * D > 1099511627776.0) return LG_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out) ||
      !aligned16(lse) || !aligned16(workspace))
    return LG_ERR_INVALID_ARG;
  const LgDecSegs g = lg_decode_segments(lg_make_cache_mask(N, sink, window, block, stride));
  const size_t need = lg_decode_workspace_bytes(B, Hq, Hkv, D, g.pre[g.n]);
  if (need > 0 && (!workspace || workspace_bytes < need)) return LG_ERR_WORKSPACE;
  const LgShape sh = make_shape(B, Hq, Hkv, N, D, scale);
  hipError_t e = lg_launch_decode(q, k_cache, v_cache, out, lse, workspace, B, Hq, Hkv, cache_slots, g, D,
                                  dtype, sh.scale, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? LG_OK : LG_ERR_LAUNCH;
}

int lg_sparse_attn_decode_cache_static(const void* q, const void* k_cache, const void* v_cache, void* out,
                                       float* lse, int B, int Hq, int Hkv, int N, int D,
                                       int sink, int window, int block, int stride, int cache_slots,
                                       int dtype, float scale, void* hip_stream) {
  if (!q || !k_cache || !v_cache || !out) return LG_ERR_NULL;
  int st = check_decode(B, Hq, Hkv, N, D, sink, window, block, stride, dtype);
  if (st != LG_OK) return st;
  const size_t need = lg_sparse_attn_decode_cache_workspace_bytes(B, Hq, Hkv, N, D, sink, window, block, stride, dtype);
  if (need > (size_t)LG_DECODE_STATIC_SCRATCH_BYTES) return LG_ERR_WORKSPACE;  // beyond the built-in scratch
  // run the remaining argument checks with a stand-in workspace before the first HIP call
  st = lg_sparse_attn_decode_cache(q, k_cache, v_cache, out, lse, nullptr, 0, B, Hq, Hkv, N, D, sink, window, block,
                                   stride, cache_slots, dtype, scale, hip_stream);
  if (need == 0 || st != LG_ERR_WORKSPACE) return st;  // no scratch needed (done), or a bad argument
  void* ws = static_scratch_ptr();
  if (!ws) return LG_ERR_LAUNCH;
  return lg_sparse_attn_decode_cache(q, k_cache, v_cache, out, lse, ws, LG_DECODE_STATIC_SCRATCH_BYTES, B, Hq, Hkv,
                                     N, D, sink, window, block, stride, cache_slots, dtype, scale, hip_stream);
}

size_t lg_sparse_attn_decode_workspace_bytes(int B, int Hq, int Hkv, int N, int D,
                                             int sink, int window, int dtype) {
  return lg_sparse_attn_decode_cache_workspace_bytes(B, Hq, Hkv, N, D, sink, window, 1, 0, dtype);
}

int lg_sparse_attn_decode(const void* q, const void* k_cache, const void* v_cache, void* out, float* lse,
                          void* workspace, size_t workspace_bytes,
                          int B, int Hq, int Hkv, int N, int D,
                          int sink, int window, int block, int stride,
                          int dtype, float scale, void* hip_stream) {
  if (!q || !k_cache || !v_cache || !out) return LG_ERR_NULL;
  int st = check_decode(B, Hq, Hkv, N, D, sink, window, block, stride, dtype);
  if (st != LG_OK) return st;
  if (stride > 0) return LG_ERR_UNSUPPORTED;  // needs the retained-block part of the cache
  return lg_sparse_attn_decode_cache(q, k_cache, v_cache, out, lse, workspace, workspace_bytes, B, Hq, Hkv, N,
                                     D, sink, window, block, stride, sink + window, dtype, scale, hip_stream);
}

static int check_paged(int n_max, int sink, int window, int block, int stride, int page_size,
                       int pages_per_seq, int num_pages, int* page_shift) {
  if (page_size < 16 || page_size > 4096 || (page_size & (page_size - 1)) != 0) return LG_ERR_INVALID_ARG;
  if (pages_per_seq < 1 || num_pages < 1) return LG_ERR_INVALID_ARG;
  const size_t need = lg_kv_cache_slots(n_max, sink, window, block, stride);
  if (need == 0 || (size_t)pages_per_seq * (size_t)page_size < need) return LG_ERR_INVALID_ARG;
  int sh = 0;
  while ((1 << sh) < page_size) ++sh;
  *page_shift = sh;
  return LG_OK;
}

size_t lg_sparse_attn_decode_paged_workspace_bytes(int B, int Hq, int Hkv, int n_max, int D,
                                                   int sink, int window, int block, int stride, int dtype) {
  return lg_sparse_attn_decode_cache_workspace_bytes(B, Hq, Hkv, n_max, D, sink, window, block, stride, dtype);
}

int lg_sparse_attn_decode_paged(const void* q, const void* k_pages, const void* v_pages,
                                const int32_t* page_table, const int32_t* seq_lens, void* out, float* lse,
                                void* workspace, size_t workspace_bytes,
                                int B, int Hq, int Hkv, int n_max, int D,
                                int sink, int window, int block, int stride,
                                int page_size, int pages_per_seq, int num_pages,
                                int dtype, float scale, void* hip_stream) {
  if (!q || !k_pages || !v_pages || !page_table || !seq_lens || !out) return LG_ERR_NULL;
  int st = check_decode(B, Hq, Hkv, n_max, D, sink, window, block, stride, dtype);
  if (st != LG_OK) return st;
  int page_shift = 0;
  st = check_paged(n_max, sink, window, block, stride, page_size, pages_per_seq, num_pages, &page_shift);
  if (st != LG_OK) return st;
  if ((double)num_pages * Hkv * (double)page_size * D > 1099511627776.0) return LG_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_pages) || !aligned16(v_pages) || !aligned16(out) || !aligned16(lse) ||
      !aligned16(workspace) || ((uintptr_t)page_table & 3) || ((uintptr_t)seq_lens & 3))
    return LG_ERR_INVALID_ARG;
  const LgMask cm = lg_make_cache_mask(n_max, sink, window, block, stride);
  const LgDecSegs g = lg_decode_segments(cm);  // the longest context: most keys
  const size_t need = lg_decode_workspace_bytes(B, Hq, Hkv, D, g.pre[g.n]);
  if (need > 0 && (!workspace || workspace_bytes < need)) return LG_ERR_WORKSPACE;
  const LgShape sh = make_shape(B, Hq, Hkv, n_max, D, scale);
  hipError_t e = lg_launch_decode(q, k_pages, v_pages, out, lse, workspace, B, Hq, Hkv, 0, g, D, dtype, sh.scale,
                                  static_cast<hipStream_t>(hip_stream), page_table, seq_lens, pages_per_seq,
                                  page_shift, n_max, &cm, num_pages);
  return e == hipSuccess ? LG_OK : LG_ERR_LAUNCH;
}

int lg_kv_paged_append(const void* k_new, const void* v_new, void* k_pages, void* v_pages,
                       const int32_t* page_table, const int32_t* positions,
                       int B, int Hkv, int D, int T, int n_max,
                       int sink, int window, int block, int stride,
                       int page_size, int pages_per_seq, int num_pages, int dtype, void* hip_stream) {
  if (!k_new || !v_new || !k_pages || !v_pages || !page_table || !positions) return LG_ERR_NULL;
  if (T < 1 || T > n_max) return LG_ERR_INVALID_ARG;
  int st = check_common(B, Hkv, Hkv, n_max, D, sink, window, block, stride, dtype);
  if (st != LG_OK) return st;
  if ((double)sink + (double)window > 1073741824.0) return LG_ERR_INVALID_ARG;
  int page_shift = 0;
  st = check_paged(n_max, sink, window, block, stride, page_size, pages_per_seq, num_pages, &page_shift);
  if (st != LG_OK) return st;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_pages) || !aligned16(v_pages) ||
      ((uintptr_t)page_table & 3) || ((uintptr_t)positions & 3))
    return LG_ERR_INVALID_ARG;
  const LgMask m = lg_make_cache_mask(n_max, sink, window, block, stride);
  const int row_bytes = D * (dtype == LG_F32 ? 4 : 2);
  hipError_t e = lg_launch_kv_paged_append(k_new, v_new, k_pages, v_pages, page_table, positions, B, Hkv,
                                           row_bytes, T, pages_per_seq, page_shift, num_pages, m,
                                           static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? LG_OK : LG_ERR_LAUNCH;
}

size_t lg_debug_decode_split_headdim_workspace_bytes(int B, int Hq, int sink, int window) {
  if (B < 1 || Hq < 1 || sink < 0 || window < 1 || (double)sink + (double)window > 1073741824.0) return 0;
  return lg_decode_split_headdim_workspace_bytes(B, Hq, sink + window);
}

int lg_debug_decode_split_headdim(const void* q, const void* k_cache, const void* v_cache, void* out, float* lse,
                                  void* workspace, size_t workspace_bytes,
                                  int B, int Hq, int Hkv, int N, int D, int sink, int window,
                                  int dtype, float scale, void* hip_stream) {
  if (!q || !k_cache || !v_cache || !out || !workspace) return LG_ERR_NULL;
  int st = check_decode(B, Hq, Hkv, N, D, sink, window, 1, 0, dtype);
  if (st != LG_OK) return st;
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out) || !aligned16(lse) ||
      !aligned16(workspace))
    return LG_ERR_INVALID_ARG;
  const int C = sink + window;
  if (workspace_bytes < lg_decode_split_headdim_workspace_bytes(B, Hq, C)) return LG_ERR_WORKSPACE;
  const LgShape sh = make_shape(B, Hq, Hkv, N, D, scale);
  hipError_t e = lg_launch_decode_split_headdim(q, k_cache, v_cache, out, lse, workspace, B, Hq, Hkv, C,
                                                N < C ? N : C, D, dtype, sh.scale,
                                                static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? LG_OK : LG_ERR_LAUNCH;
}

int lg_debug_decode_segments(int N, int sink, int window, int block, int stride,
                             int* nseg, int32_t* start, int32_t* len) {
  if (!nseg || !start || !len) return LG_ERR_NULL;
  int st = check_decode(1, 1, 1, N, 64, sink, window, block, stride, LG_F32);
  if (st != LG_OK) return st;
  const LgDecSegs g = lg_decode_segments(lg_make_cache_mask(N, sink, window, block, stride));
  *nseg = g.n;
  for (int x = 0; x < 4; ++x) {
    start[x] = x < g.n ? g.start[x] : 0;
    len[x] = x < g.n ? g.pre[x + 1] - g.pre[x] : 0;
  }
  return LG_OK;
}

int lg_debug_tile_map(int N, int sink, int window, int block, int stride, int dtype, int transposed,
                      int* tq, int* tk, int32_t* row_ptr, size_t row_cap,
                      int32_t* col_idx, uint8_t* kind, size_t cap,
                      size_t* rows, size_t* needed) {
  if (!tq || !tk || !rows || !needed) return LG_ERR_NULL;
  int st = check_common(1, 1, 1, N, 64, sink, window, block, stride, dtype);
  if (st != LG_OK) return st;
  const LgMask m = lg_make_mask(N, sink, window, block, stride);
  int Tq, Tk;
  if (dtype == LG_F32) {
    Tq = transposed ? LG_F32_BTQ : LG_F32_TQ;
    Tk = transposed ? LG_F32_BTK : LG_F32_TK;
  } else {
    Tq = transposed ? LG_BF16_BTQ : LG_BF16_TQ;
    Tk = transposed ? LG_BF16_BTK : LG_BF16_TK;
  }
  *tq = Tq;
  *tk = Tk;
  size_t n = 0, r = 0;
  auto emit = [&](int col, int kd) {
    if (n < cap) {
      if (col_idx) col_idx[n] = col;
      if (kind) kind[n] = (uint8_t)(kd == LG_TILE_FULL);
    }
    ++n;
  };
  auto mark_row = [&]() {
    if (row_ptr && r < row_cap) row_ptr[r] = (int32_t)n;
    ++r;
  };
  if (!transposed) {
    const int nq = (N + Tq - 1) / Tq;
    for (int u = 0; u < nq; ++u) {
      mark_row();
      const int q0 = u * Tq, q1 = (q0 + Tq - 1 < N - 1) ? q0 + Tq - 1 : N - 1;
      // the per-query-tile schedule the kernels' main loops run
      const LgQSched qs = lg_qsched_init(m, q0, q1);
      for (int t = lg_qsched_next(m, qs, -1); t >= 0; t = lg_qsched_next(m, qs, t))
        emit(t, lg_qsched_full(m, qs, t) ? LG_TILE_FULL : LG_TILE_PARTIAL);
    }
  } else {
    const int nk = (N + Tk - 1) / Tk;
    for (int t = 0; t < nk; ++t) {
      mark_row();
      const int k0 = t * Tk, k1 = (k0 + Tk - 1 < N - 1) ? k0 + Tk - 1 : N - 1;
      int lo, hi;
      lg_qtile_range(m, k0, k1, Tq, &lo, &hi);
      for (int u = lo; u <= hi; ++u) {
        const int q0 = u * Tq, q1 = (q0 + Tq - 1 < N - 1) ? q0 + Tq - 1 : N - 1;
        emit(u, lg_tile_kind(m, q0, q1, k0, t * Tk + Tk - 1));
      }
    }
  }
  if (row_ptr && r < row_cap) row_ptr[r] = (int32_t)n;
  *rows = r;
  *needed = n;
  return LG_OK;
}

int lg_debug_partial_tile_bits(int N, int sink, int window, int block, int stride, int transposed,
                               int fixed, int tile0, int half, uint32_t* bits) {
  if (!bits) return LG_ERR_NULL;
  int st = check_common(1, 1, 1, N, 64, sink, window, block, stride, LG_BF16);
  if (st != LG_OK) return st;
  if (fixed < 0 || fixed >= N || tile0 < 0 || tile0 > (1 << 30) || (half != 0 && half != 1))
    return LG_ERR_INVALID_ARG;
  const LgMask m = lg_make_mask(N, sink, window, block, stride);
  *bits = transposed ? lg_row_bits(m, fixed, tile0, half) : lg_key_bits(m, fixed, tile0, half);
  return LG_OK;
}

int lg_debug_pattern_fields(int n_made_for, int n, int sink, int window, int block, int stride, int32_t* fields) {
  if (!fields) return LG_ERR_NULL;
  int st = check_common(1, 1, 1, n_made_for, 64, sink, window, block, stride, LG_BF16);
  if (st != LG_OK) return st;
  if (n < 1 || n > n_made_for) return LG_ERR_INVALID_ARG;
  const LgMask t = lg_make_mask(n_made_for, sink, window, block, stride);
  const LgMask m = n == n_made_for ? t : lg_mask_for_length(t, n);
  const int f[9] = {m.N, m.sink, m.window, m.b, m.stride, m.sb, m.wb, m.bshift, m.smask};
  for (int x = 0; x < 9; ++x) fields[x] = f[x];
  return LG_OK;
}

int lg_debug_tile_walk(int N, int sink, int window, int block, int stride, int transposed, int row,
                       int32_t* order, size_t cap, size_t* count) {
  if (!count) return LG_ERR_NULL;
  int st = check_common(1, 1, 1, N, 64, sink, window, block, stride, LG_BF16);
  if (st != LG_OK) return st;
  const LgMask m = lg_make_mask(N, sink, window, block, stride);
  const int Tq = transposed ? LG_BF16_BTQ : LG_BF16_TQ, Tk = transposed ? LG_BF16_BTK : LG_BF16_TK;
  const int nrows = transposed ? (N + Tk - 1) / Tk : (N + Tq - 1) / Tq;
  if (row < 0 || row >= nrows) return LG_ERR_INVALID_ARG;
  size_t n = 0;
  auto emit = [&](int t) {
    if (order && n < cap) order[n] = t;
    ++n;
  };
  if (!transposed) {
    const int q0 = row * Tq, q1 = (q0 + Tq - 1 < N - 1) ? q0 + Tq - 1 : N - 1;
    const LgQSched qs = lg_qsched_init(m, q0, q1);
    if (m.stride == 0) {  // patterns without strided columns: the rotated walk
      const LgQWalk w = lg_qwalk_init(qs);
      for (int t = lg_qwalk_first(w); t >= 0; t = lg_qwalk_next(w, t)) emit(t);
    } else {
      for (int t = lg_qsched_next(m, qs, -1); t >= 0; t = lg_qsched_next(m, qs, t)) emit(t);
    }
  } else {
    const int k0 = row * Tk, k1 = (k0 + Tk - 1 < N - 1) ? k0 + Tk - 1 : N - 1;
    int lo, hi;
    lg_qtile_range(m, k0, k1, Tq, &lo, &hi);
    const int hw = lg_qtile_window_hi(m, k1, Tq);  // window part [lo, hw], walked rotated
    const int len = hw - lo + 1;
    int u = lo + (len - lo % len) % len;
    for (int x = 0; x < len; ++x) {
      emit(u);
      u = (u == hw) ? lo : u + 1;
    }
    for (int c = hw + 1; c <= hi; ++c) emit(c);  // column part (its own workgroups, or the same one)
  }
  *count = n;
  return LG_OK;
}

}  // extern "C"
