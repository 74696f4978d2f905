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
// Each thread moves one unit of 4 rows x 8 dims (four 16-byte global loads).
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
  int u, du;
  bool active;
  __device__ __forceinline__ void init(int tid) {
    u = tid / (D / 8);
    du = tid % (D / 8);
    active = LgTile<D>::UNITS >= 256 || tid < LgTile<D>::UNITS;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) r[kk] = make_uint4(0, 0, 0, 0);
  }
  // rows row0 + 4u .. +3 of a [nrows, D] matrix at base; row index clamped to nrows-1
  __device__ __forceinline__ void load(const uint16_t* __restrict__ base, int row0, int nrows) {
    if (active) {
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int j = min(row0 + 4 * u + kk, nrows - 1);
        r[kk] = *reinterpret_cast<const uint4*>(base + (size_t)j * D + du * 8);
      }
    }
  }
  __device__ __forceinline__ void store_rm(unsigned char* s) const {
    if (active) {
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        *reinterpret_cast<uint4*>(s + (4 * u + kk) * LgTile<D>::RM_STRIDE + du * 16) = r[kk];
    }
  }
  __device__ __forceinline__ void store_t(unsigned char* s) const {
    if (active) {
      const int x = 2 * (u >> 2) + (u & 1);
      const int half = ((u >> 1) & 1) * 8;
      const uint32_t w[4][4] = {{r[0].x, r[0].y, r[0].z, r[0].w},
                                {r[1].x, r[1].y, r[1].z, r[1].w},
                                {r[2].x, r[2].y, r[2].z, r[2].w},
                                {r[3].x, r[3].y, r[3].z, r[3].w}};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int d = du * 8 + e;
        const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
        uint2 val;
        val.x = __builtin_amdgcn_perm(w[1][e >> 1], w[0][e >> 1], sel);  // rows +0, +1
        val.y = __builtin_amdgcn_perm(w[3][e >> 1], w[2][e >> 1], sel);  // rows +2, +3
        *reinterpret_cast<uint2*>(s + lg_t_off(d, x) + half) = val;
      }
    }
  }
};

// A operand from a row-major tile: 32-row block rb, lane (n, g), 16-dim chunk dc.
template <int D>
__device__ __forceinline__ bf16x8_t lg_read_rm(const unsigned char* s, int rb, int n, int g, int dc) {
  return lg_as_bf16x8(
      *reinterpret_cast<const uint4*>(s + (rb * 32 + n) * LgTile<D>::RM_STRIDE + dc * 32 + g * 16));
}

// A operand from a transposed tile: 32-dim block db, lane (n, g), 16-row group c.
__device__ __forceinline__ bf16x8_t lg_read_t(const unsigned char* s, int db, int n, int g, int c) {
  return lg_as_bf16x8(*reinterpret_cast<const uint4*>(s + lg_t_off(db * 32 + n, 2 * c + g)));
}

// Pack accumulator registers 8h..8h+7 (rounded to bf16) as a B operand.
__device__ __forceinline__ bf16x8_t lg_pack_acc(const float* p) {
  uint4 w;
  w.x = lg_pack_bf16(p[0], p[1]);
  w.y = lg_pack_bf16(p[2], p[3]);
  w.z = lg_pack_bf16(p[4], p[5]);
  w.w = lg_pack_bf16(p[6], p[7]);
  return lg_as_bf16x8(w);
}

#endif  // LG_STAGE_H_
