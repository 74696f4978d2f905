// lg_stage.h — staging of 64-row bf16 tiles from global memory into LDS for the
// MFMA kernels, in the two layouts the matrix cores need.
//
// A tile is 64 rows (keys or queries) x D dims, D contiguous in global memory.
//   row-major layout  ("RM"): rows padded to D*2+16 bytes.  Feeds an A operand whose
//        contraction runs over the head dim (lane n reads 16 bytes of row n).
//   transposed layout ("T"):  D rows of 64 entries (128 bytes), 16-byte chunks XOR-
//        swizzled.  Feeds an A operand whose contraction runs over the 64 tile rows
//        (lane n reads 16 bytes = 8 tile rows of dim n).  The 8 tile rows of a chunk
//        are stored in "slot order": chunk x = 2c+g of 16-row group c holds tile rows
//        16c + 8q' + 4g + t at position 4q' + t.  That is exactly the order in which
//        lane-half g of a 32x32 accumulator holds its rows (registers 8h..8h+7 of
//        32-row block kb cover 16-row group c = 2kb+h), so an accumulator can be fed
//        back as the B operand of the next product without any lane exchange.
// A group of 256 threads moves one tile; each thread owns one unit of 4 rows x 8 dims
// (four 16-byte global loads).  All LDS offsets are computed once per thread.
#ifndef LG_STAGE_H_
#define LG_STAGE_H_

#include "lg_mfma.h"

template <int D>
struct LgTile {
  static constexpr int ROWS = 64;
  static constexpr int RM_STRIDE = D * 2 + 16;
  static constexpr int RM_BYTES = ROWS * RM_STRIDE;
  static constexpr int T_BYTES = D * ROWS * 2;
  static constexpr int UNITS = 16 * (D / 8);  // 256 threads cover D=128; half of them D=64
};

// byte offset of (dim d, chunk x) in a transposed tile
__device__ __forceinline__ int lg_t_off(int d, int x) {
  const int prow = d ^ ((d >> 3) & 1);
  const int sw = ((d >> 1) ^ (d >> 4)) & 7;
  return prow * 128 + ((x ^ sw) << 4);
}

template <int D>
struct LgStager {
  uint4 r[4];
  int goff;      // element offset of this thread's first row inside a tile: (4u)*D + 8du
  int rm_off;    // byte offset of that row in a row-major tile
  int t_off[8];  // byte offsets of the 8 dims of the unit in a transposed tile
  int u;
  bool active;
  // t256: index of the thread inside its 256-thread staging group
  __device__ __forceinline__ void init(int t256, bool want_t) {
    u = t256 / (D / 8);
    const int du = t256 % (D / 8);
    active = LgTile<D>::UNITS >= 256 || t256 < LgTile<D>::UNITS;
    goff = 4 * u * D + du * 8;
    rm_off = 4 * u * LgTile<D>::RM_STRIDE + du * 16;
    const int x = 2 * (u >> 2) + (u & 1);
    const int half = ((u >> 1) & 1) * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) t_off[e] = want_t ? lg_t_off(du * 8 + e, x) + half : 0;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) r[kk] = make_uint4(0, 0, 0, 0);
  }
  // tile = first row of the tile (wave-uniform pointer); rows_left = rows of the matrix
  // from there on (rows beyond it are replaced by the last valid row)
  __device__ __forceinline__ void load(const uint16_t* __restrict__ tile, int rows_left) {
    if (!active) return;
    if (rows_left >= LgTile<D>::ROWS) {
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) r[kk] = *reinterpret_cast<const uint4*>(tile + goff + kk * D);
    } else {
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int row = min(4 * u + kk, rows_left - 1);
        r[kk] = *reinterpret_cast<const uint4*>(tile + goff + (row - 4 * u) * D);
      }
    }
  }
  __device__ __forceinline__ void store_rm(unsigned char* s) const {
    if (!active) return;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
      *reinterpret_cast<uint4*>(s + rm_off + kk * LgTile<D>::RM_STRIDE) = r[kk];
  }
  __device__ __forceinline__ void store_t(unsigned char* s) const {
    if (!active) return;
    const uint32_t w[4][4] = {{r[0].x, r[0].y, r[0].z, r[0].w},
                              {r[1].x, r[1].y, r[1].z, r[1].w},
                              {r[2].x, r[2].y, r[2].z, r[2].w},
                              {r[3].x, r[3].y, r[3].z, r[3].w}};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
      uint2 val;
      val.x = __builtin_amdgcn_perm(w[1][e >> 1], w[0][e >> 1], sel);  // rows +0, +1
      val.y = __builtin_amdgcn_perm(w[3][e >> 1], w[2][e >> 1], sel);  // rows +2, +3
      *reinterpret_cast<uint2*>(s + t_off[e]) = val;
    }
  }
};

// Per-lane LDS read offsets of the MFMA A operands, computed once.
template <int D>
struct LgReader {
  int rm;     // row-major: lane (n, g) -> row n, 16-byte half g of a 32-byte dim chunk
  int t[4];   // transposed: lane (n, g) -> dim row n; t[e] selects chunk pair e = c ^ (db & 3)
  __device__ __forceinline__ void init(int n, int g) {
    rm = n * LgTile<D>::RM_STRIDE + g * 16;
    const int pn = n ^ ((n >> 3) & 1);
    const int s0 = ((n >> 1) ^ (n >> 4)) & 7;
#pragma unroll
    for (int e = 0; e < 4; ++e) t[e] = pn * 128 + (((2 * e + g) ^ s0) << 4);
  }
  // A operand from a row-major tile: 32-row block rb, 16-dim chunk dc.
  __device__ __forceinline__ bf16x8_t read_rm(const unsigned char* s, int rb, int dc) const {
    return lg_as_bf16x8(
        *reinterpret_cast<const uint4*>(s + rm + rb * 32 * LgTile<D>::RM_STRIDE + dc * 32));
  }
  // A operand from a transposed tile: 32-dim block db, 16-row group c (both compile-time
  // constants after unrolling, so the select below costs nothing).
  __device__ __forceinline__ bf16x8_t read_t(const unsigned char* s, int db, int c) const {
    return lg_as_bf16x8(*reinterpret_cast<const uint4*>(s + t[c ^ (db & 3)] + db * 4096));
  }
};

// Pack accumulator registers 8h..8h+7 (rounded to bf16) as a B operand.
__device__ __forceinline__ bf16x8_t lg_pack_acc(const float* p) {
  uint4 w;
  w.x = lg_pack_bf16(p[0], p[1]);
  w.y = lg_pack_bf16(p[2], p[3]);
  w.z = lg_pack_bf16(p[4], p[5]);
  w.w = lg_pack_bf16(p[6], p[7]);
  return lg_as_bf16x8(w);
}

// Live bits of one lane's 32 keys (or rows) of a 64-wide tile half: bit r = live(i, j0 + crow(r))
// for r in 0..15 of 32-block 0 and r-16 of 32-block 1.  Rolled loop: only PARTIAL tiles pay.
__device__ __forceinline__ uint32_t lg_live_bits_q(const LgMask& m, int i, int k0, int g) {
  uint32_t bits = 0;
#pragma unroll 1
  for (int r = 0; r < 32; ++r) {
    const int j = k0 + (r >> 4) * 32 + lg_crow(r & 15, g);
    bits |= (uint32_t)lg_live(m, i, j) << r;
  }
  return bits;
}

#endif  // LG_STAGE_H_
