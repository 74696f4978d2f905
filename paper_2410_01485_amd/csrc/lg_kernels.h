// lg_kernels.h — internal interface between the C ABI (lg_api.hip) and the kernel
// translation units.  Tile sizes live here because the host-side tile map
// (lg_debug_tile_map) must enumerate exactly the tiles the kernels walk.
#ifndef LG_KERNELS_H_
#define LG_KERNELS_H_

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "lg_mask.h"

// Kernel tile sizes (query rows x keys per step).  Independent of the pattern's
// `block`: they never change results, only which tiles count as PARTIAL.
enum {
  LG_F32_TQ = 64, LG_F32_TK = 64,        // float32 kernels, forward / dq order
  LG_F32_BTQ = 64, LG_F32_BTK = 64,      // float32 dk/dv kernel (key-tile major)
  LG_BF16_TQ = 256, LG_BF16_TK = 64,     // bf16 MFMA forward and dq kernels
  LG_BF16_BTQ = 64, LG_BF16_BTK = 256    // bf16 MFMA dk/dv kernel (key-tile major)
};

struct LgShape {
  int B, Hq, Hkv, N, D;
  float scale;  // already resolved (> 0)
};

// Each launcher enqueues on `s` and returns hipGetLastError().
hipError_t lg_launch_fwd_f32(const float* q, const float* k, const float* v, float* out, float* lse,
                             const LgShape& sh, const LgMask& m, hipStream_t s);
hipError_t lg_launch_fwd_bf16(const void* q, const void* k, const void* v, void* out, float* lse,
                              const LgShape& sh, const LgMask& m, hipStream_t s);

// Several sequences of different lengths, packed along the token axis of every head, in ONE forward launch:
// sequence x owns rows row0[x] .. row0[x+1]-1 of each head and the launch's query tiles tile0[x] .. tile0[x+1]-1.
// Passed to the kernel by value (about 1 KB of kernel arguments).
enum { LG_PACK_MAX = 128 };
struct LgPack {
  int n;                        // sequences, 1 .. LG_PACK_MAX, none of them empty
  int row0[LG_PACK_MAX + 1];
  int tile0[LG_PACK_MAX + 1];
};
// Fills tile0 from row0 (bf16 forward tile size); returns the number of query tiles.
long long lg_fwd_bf16_pack_tiles(LgPack* pack);
// sh: B = 1, N unused; tmpl: the pattern made for a length no sequence exceeds, ld = rows per head.
hipError_t lg_launch_fwd_bf16_pack(const void* q, const void* k, const void* v, void* out, float* lse,
                                   const LgShape& sh, const LgMask& tmpl, const LgPack& pack, hipStream_t s);

// delta_i = dsign * <dout_i, out_i> for rows = B*Hq*N rows of D elements of either dtype;
// lse2 (may be NULL) = lse * lscale.  delta and lse2 are dense; in dout, out and lse a head's N rows are
// followed by the next head's after ld rows.
hipError_t lg_launch_delta(const void* dout, const void* out, float* delta, const float* lse, float* lse2,
                           float dsign, float lscale, long long rows, int N, int ld, int D, int dtype,
                           hipStream_t s);
size_t lg_bwd_workspace_bytes(const LgShape& sh, const LgMask& m, int dtype);
size_t lg_bwd_bf16_workspace_bytes(const LgShape& sh, const LgMask& m, size_t head_bytes);
// ev: NULL, or 4 events recorded before the Delta pre-pass, between the kernels and after the
// last one (measurement aid).
hipError_t lg_launch_bwd_f32(const float* q, const float* k, const float* v, const float* out,
                             const float* lse, const float* dout, float* dq, float* dk, float* dv,
                             void* ws, const LgShape& sh, const LgMask& m, hipStream_t s,
                             hipEvent_t* ev);
hipError_t lg_launch_bwd_bf16(const void* q, const void* k, const void* v, const void* out,
                              const float* lse, const void* dout, void* dq, void* dk, void* dv,
                              void* ws, const LgShape& sh, const LgMask& m, hipStream_t s,
                              hipEvent_t* ev);

// Decode: C = sink + window cache slots per (b, hkv), `valid` of them in use.
int lg_decode_splits(int B, int Hkv, int valid);
size_t lg_decode_workspace_bytes(int B, int Hq, int Hkv, int D, int valid);
hipError_t lg_launch_decode(const void* q, const void* kc, const void* vc, void* out, float* lse,
                            void* ws, int B, int Hq, int Hkv, int C, const LgDecSegs& segs, int D,
                            int dtype, float scale, hipStream_t s, const int* page_table = nullptr,
                            const int* seq_lens = nullptr, int pages_per_seq = 0, int page_shift = 0,
                            int n_max = 0, const LgMask* cache_mask = nullptr, int num_pages = 0);
size_t lg_decode_split_headdim_workspace_bytes(int B, int Hq, int C);
hipError_t lg_launch_decode_split_headdim(const void* q, const void* kc, const void* vc, void* out, float* lse,
                                          void* ws, int B, int Hq, int Hkv, int C, int valid, int D, int dtype,
                                          float scale, hipStream_t s);
hipError_t lg_launch_kv_paged_append(const void* k_new, const void* v_new, void* k_pages, void* v_pages,
                                     const int* page_table, const int* positions, int B, int Hkv,
                                     int row_bytes, int T, int pages_per_seq, int page_shift, int num_pages,
                                     const LgMask& m, hipStream_t s);
hipError_t lg_launch_kv_append(const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                               int B, int Hkv, int row_bytes, int T, int pos, int slots,
                               const LgMask& m, hipStream_t s);

#endif  // LG_KERNELS_H_
