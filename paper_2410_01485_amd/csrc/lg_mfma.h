// lg_mfma.h — small device helpers shared by the bf16 MFMA kernels (gfx950).
//
// Matrix-core layout used throughout (v_mfma_f32_32x32x16_bf16, one wavefront):
//   lane = 32*g + n,  g in {0,1},  n in 0..31
//   A operand (32 x 16): lane holds row n,    contraction slots 8g .. 8g+7  (8 bf16)
//   B operand (16 x 32): lane holds column n, contraction slots 8g .. 8g+7  (8 bf16)
//   C/D (32 x 32, 16 floats): register r of a lane is row 8*(r/4) + 4g + (r%4), column n
// Both operands always take their 8 slots from the same 8 positions of the
// contracted index, so the product does not depend on how the hardware orders
// the slots internally.
#ifndef LG_MFMA_H_
#define LG_MFMA_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ f32x16_t lg_mfma32(bf16x8_t a, bf16x8_t b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Row of register r (0..15) of a 32x32 accumulator for lane-half g.
__device__ __forceinline__ constexpr int lg_crow(int r, int g) { return 8 * (r >> 2) + 4 * g + (r & 3); }

// Value held by lane ^ 32.
__device__ __forceinline__ float lg_other_half(float x) {
  const unsigned u = __builtin_bit_cast(unsigned, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  // one of the two results is this lane's own value, the other the partner's
  const unsigned own_xor = r[0] ^ r[1];
  return __builtin_bit_cast(float, own_xor ^ u);
}

// Round two floats to bf16 (nearest even) and pack them, low element first.
__device__ __forceinline__ uint32_t lg_pack_bf16(float lo, float hi) {
  f32x2_t f = {lo, hi};
  bf16x2_t h = __builtin_convertvector(f, bf16x2_t);
  return __builtin_bit_cast(uint32_t, h);
}

__device__ __forceinline__ bf16x8_t lg_as_bf16x8(uint4 x) { return __builtin_bit_cast(bf16x8_t, x); }

#endif  // LG_MFMA_H_
