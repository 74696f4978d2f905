// lg_swz.h — 64-row bf16 tiles in LDS for the gfx950 MFMA kernels, filled by direct
// global->LDS loads and read in both orientations the matrix cores need.
//
// A tile is 64 rows (keys or queries) x D dims, kept ROW-MAJOR in LDS (row = D*2 bytes)
// with its 16-byte chunks XOR-swizzled:  chunk c of row r sits at chunk position c ^ pi(r),
//     pi(r) = ((r & 7) << 1) | ((r >> 3) & 1)   for D = 128 (16 chunks per row)
//     pi(r) = (r >> 1) & 7                       for D = 64  (8 chunks per row)
// Filling: global_load_lds_dwordx4 — every lane names a 16-byte global source, the wave's
//   64 x 16 bytes land contiguously in LDS at the address in M0, bypassing registers.  The
//   swizzle is applied on the global side (lane at LDS position p fetches the chunk that
//   belongs there).  Loads are issued through inline asm so that the tile pipeline, not the
//   compiler, decides how many of them stay in flight (s_waitcnt vmcnt(n) + barrier).
// Reading with the contraction over dims (A operand rows = tile rows): ds_read_b128, lane n
//   reads 16 bytes of row n; the swizzle makes the 16 rows of a pass hit 16 different chunk
//   positions (no bank conflicts).
// Reading with the contraction over tile rows (A operand rows = dims): ds_read_b64_tr_b16.
//   Within each group of 16 lanes the hardware transposes a 4-row x 16-dim block: source
//   lane s points at (row s/4, dims 4*(s%4)..+3) and result lane l receives the 4 rows of
//   dim l.  Two such reads give a lane the 8 contraction slots of one 16-row group, ordered
//   rows 16c + 8q' + 4g + t at slot 4q' + t — the order in which lane-half g of a 32x32
//   accumulator holds its rows, so an accumulator (rounded to bf16) can be fed back as the B
//   operand without any lane exchange.
#ifndef LG_SWZ_H_
#define LG_SWZ_H_

#include "lg_mfma.h"

typedef short lg_s16x4 __attribute__((ext_vector_type(4)));
#define LG_LDS_PTR(T, p) ((T __attribute__((address_space(3)))*)(p))

template <int D>
struct LgSwzTile {
  static constexpr int ROWS = 64;
  static constexpr int CPR = D / 8;          // 16-byte chunks per row
  static constexpr int ROW_BYTES = D * 2;
  static constexpr int BYTES = ROWS * ROW_BYTES;
  __device__ __forceinline__ static int pi(int r) {
    return D == 128 ? (((r & 7) << 1) | ((r >> 3) & 1)) : ((r >> 1) & 7);
  }
};

// s_waitcnt vmcnt(n) only (expcnt / lgkmcnt left unconstrained), n < 64: the count sits in
// bits [3:0] and [15:14] of the immediate
#define LG_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

// Direct global->LDS copy of one tile by NT threads.
template <int D, int NT>
struct LgDma {
  using T = LgSwzTile<D>;
  static constexpr int CH = T::ROWS * T::CPR / NT;  // 16-byte chunks per thread
  static_assert(CH >= 1, "tile smaller than the workgroup");
  uint32_t voff[CH];   // global byte offset of this lane's chunk inside the tile
  uint32_t wave_off;   // LDS byte offset of this wave's first chunk inside the tile
  __device__ __forceinline__ void init(int tid) {
#pragma unroll
    for (int x = 0; x < CH; ++x) {
      const int p = x * NT + tid;
      const int row = p / T::CPR;
      const int chunk = (p % T::CPR) ^ T::pi(row);
      voff[x] = row * T::ROW_BYTES + chunk * 16;
    }
    wave_off = (uint32_t)__builtin_amdgcn_readfirstlane(tid >> 6) * 1024u;  // wave-uniform: stays scalar
  }
  // src: first row of the tile in global memory (wave-uniform); rows_left: rows of the matrix
  // from there on (rows past the end are replaced by the last valid row); lds: LDS byte
  // address of the tile (wave-uniform).
  __device__ __forceinline__ void issue(const uint16_t* src, int rows_left, uint32_t lds) const {
    // two copies of the loop behind one wave-uniform branch: whole tiles (nearly all) spend no
    // vector instructions on addresses
    if (rows_left >= T::ROWS) {
#pragma unroll
      for (int x = 0; x < CH; ++x) load(src, voff[x], lds, x);
    } else {  // ragged tile: rows past the end repeat the last valid row
#pragma unroll
      for (int x = 0; x < CH; ++x) {
        const int row = (int)(voff[x] / T::ROW_BYTES);
        const int r = min(row, rows_left - 1);
        load(src, voff[x] - row * T::ROW_BYTES + r * T::ROW_BYTES, lds, x);
      }
    }
  }
  __device__ __forceinline__ void load(const uint16_t* src, uint32_t off, uint32_t lds, int x) const {
    const uint32_t m0 = lds + wave_off + x * NT * 16;  // all scalar
    // (an LDS-bound load reads M0 one issue slot after a scalar write at the earliest)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(__builtin_amdgcn_readfirstlane(m0)), "v"(off), "s"(src)
                 : "memory");
  }
};

// Direct global->LDS copy of 64 consecutive floats by one wave: lane l fetches src[l]
// (src is this lane's own address) and the wave's 256 bytes land contiguously at `lds`.
__device__ __forceinline__ void lg_dma_f32x64(const float* lane_src, uint32_t lds) {
  const uint32_t m0 = __builtin_amdgcn_readfirstlane(lds);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(m0), "v"(lane_src) : "memory");
}

// Per-lane read offsets into a swizzled tile (lane = 32g + n).  Only two lane-dependent
// bases are kept in registers; the per-chunk addresses differ from them by XORs with small
// constants (bits 4..7 of the byte address), applied after the tile's LDS offset is added.
// Tiles must therefore start at multiples of 256 bytes.
template <int D>
struct LgSwzReader {
  using T = LgSwzTile<D>;
  int kbase;  // row reads: 16 bytes of row n, dims 8g .. +7 (chunk g ^ pi(n))
  int vbase;  // transpose reads: see read_cols
  __device__ __forceinline__ void init(int n, int g) {
    kbase = n * T::ROW_BYTES + ((g ^ T::pi(n)) << 4);
    const int s = n & 15;
    const int a = (n >> 4) * 2 + ((s & 3) >> 1);  // 16-byte chunk inside the 64-byte dim block
    const int half = (s & 1) * 8;
    const int rho = 4 * g + (s >> 2);             // row inside the 8-row group
    const int lanepi = D == 128 ? 2 * rho : 2 * g + (s >> 3);
    vbase = rho * T::ROW_BYTES + half + ((a ^ lanepi) << 4);
  }
  // A operand, contraction over dims: rows 32*rb + n, dim chunk dc.  tile = byte offset of the
  // tile inside smem (wave-uniform).
  __device__ __forceinline__ bf16x8_t read_rows(const unsigned char* smem, int tile, int rb, int dc) const {
    const int a = ((kbase + tile) ^ (dc << 5)) + rb * 32 * T::ROW_BYTES;
    return lg_as_bf16x8(*reinterpret_cast<const uint4*>(smem + a));
  }
  // A operand, contraction over tile rows: dims 32*db + n, 16-row group c (slot order above).
  __device__ __forceinline__ bf16x8_t read_cols(const unsigned char* smem, int tile, int db, int c) const {
    // rows 16c + 8q' + rho; chunk (4db + a) ^ pi(row): the constant part of the XOR is
    // (4db | q') for D = 128 and 4(db ^ q') for D = 64
    const int x0 = D == 128 ? ((4 * db) << 4) : ((db ^ 0) << 6);
    const int x1 = D == 128 ? ((4 * db | 1) << 4) : ((db ^ 1) << 6);
    const int a0 = ((vbase + tile) ^ x0) + (16 * c) * T::ROW_BYTES;
    const int a1 = ((vbase + tile) ^ x1) + (16 * c + 8) * T::ROW_BYTES;
    const lg_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LG_LDS_PTR(lg_s16x4, smem + a0));
    const lg_s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LG_LDS_PTR(lg_s16x4, smem + a1));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const s16x8 w = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, w);
  }
};

// Pack accumulator registers 8h..8h+7 (rounded to bf16) as a B operand.
__device__ __forceinline__ bf16x8_t lg_pack8(const float* p) {
  uint4 w;
  w.x = lg_pack_bf16(p[0], p[1]);
  w.y = lg_pack_bf16(p[2], p[3]);
  w.z = lg_pack_bf16(p[4], p[5]);
  w.w = lg_pack_bf16(p[6], p[7]);
  return lg_as_bf16x8(w);
}

#endif  // LG_SWZ_H_
