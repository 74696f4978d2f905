// lg_wide.h — building blocks of the kernels that keep 64 rows (keys) per wave, one wave per
// SIMD, and write their matrix instructions as inline statements with explicit register classes
// (see the kernels in lg_bwd_bf16.hip for the reasons and the rules they follow).
#ifndef LG_WIDE_H_
#define LG_WIDE_H_

#include <utility>

#include "lg_mfma.h"

namespace {

// Accumulator I (0..15) is the fixed register block a[16 I : 16 I + 15]; the compiler only learns
// that the statement overwrites those registers.  It must not use AGPRs for anything of its own
// in such a kernel (it has no reason to while nothing spills; tests/test_build_isa.py checks the
// generated code).  zero clears the block through the matrix pipe (0 * 0 + 0); get copies it to
// 16 floats once the last matrix instruction has certainly finished.
template <int I>
struct LgAcc;
#define LG_ACC_CLOBBER(R0, R1, R2, R3, R4, R5, R6, R7, R8, R9, R10, R11, R12, R13, R14, R15) \
  "a" #R0, "a" #R1, "a" #R2, "a" #R3, "a" #R4, "a" #R5, "a" #R6, "a" #R7, "a" #R8, "a" #R9, "a" #R10, "a" #R11, \
      "a" #R12, "a" #R13, "a" #R14, "a" #R15
#define LG_ACC(I, LO, HI, R0, R1, R2, R3, R4, R5, R6, R7, R8, R9, R10, R11, R12, R13, R14, R15) \
  template <> \
  struct LgAcc<I> { \
    static __device__ __forceinline__ void fma(bf16x8_t a, bf16x8_t b) { \
      asm volatile("v_mfma_f32_32x32x16_bf16 a[" #LO ":" #HI "], %0, %1, a[" #LO ":" #HI "]" ::"v"(a), "v"(b) \
                   : LG_ACC_CLOBBER(R0, R1, R2, R3, R4, R5, R6, R7, R8, R9, R10, R11, R12, R13, R14, R15)); \
    } \
    static __device__ __forceinline__ void zero(bf16x8_t z) { \
      asm volatile("v_mfma_f32_32x32x16_bf16 a[" #LO ":" #HI "], %0, %0, 0" ::"v"(z) \
                   : LG_ACC_CLOBBER(R0, R1, R2, R3, R4, R5, R6, R7, R8, R9, R10, R11, R12, R13, R14, R15)); \
    } \
    static __device__ __forceinline__ void get(float* x) { \
      asm volatile("v_accvgpr_read_b32 %0, a" #R0 "\n\t" "v_accvgpr_read_b32 %1, a" #R1 "\n\t" "v_accvgpr_read_b32 %2, a" #R2 "\n\t" "v_accvgpr_read_b32 %3, a" #R3 "\n\t" "v_accvgpr_read_b32 %4, a" #R4 "\n\t" "v_accvgpr_read_b32 %5, a" #R5 "\n\t" "v_accvgpr_read_b32 %6, a" #R6 "\n\t" "v_accvgpr_read_b32 %7, a" #R7 "\n\t" "v_accvgpr_read_b32 %8, a" #R8 "\n\t" "v_accvgpr_read_b32 %9, a" #R9 "\n\t" "v_accvgpr_read_b32 %10, a" #R10 "\n\t" "v_accvgpr_read_b32 %11, a" #R11 "\n\t" "v_accvgpr_read_b32 %12, a" #R12 "\n\t" "v_accvgpr_read_b32 %13, a" #R13 "\n\t" "v_accvgpr_read_b32 %14, a" #R14 "\n\t" "v_accvgpr_read_b32 %15, a" #R15 "\n\t" \
                   : "=v"(x[0]), "=v"(x[1]), "=v"(x[2]), "=v"(x[3]), "=v"(x[4]), "=v"(x[5]), "=v"(x[6]), "=v"(x[7]), "=v"(x[8]), "=v"(x[9]), "=v"(x[10]), "=v"(x[11]), "=v"(x[12]), "=v"(x[13]), "=v"(x[14]), "=v"(x[15])); \
    } \
  };
LG_ACC(0, 0, 15, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15)
LG_ACC(1, 16, 31, 16, 17, 18, 19, 20, 21, 22, 23, 24, 25, 26, 27, 28, 29, 30, 31)
LG_ACC(2, 32, 47, 32, 33, 34, 35, 36, 37, 38, 39, 40, 41, 42, 43, 44, 45, 46, 47)
LG_ACC(3, 48, 63, 48, 49, 50, 51, 52, 53, 54, 55, 56, 57, 58, 59, 60, 61, 62, 63)
LG_ACC(4, 64, 79, 64, 65, 66, 67, 68, 69, 70, 71, 72, 73, 74, 75, 76, 77, 78, 79)
LG_ACC(5, 80, 95, 80, 81, 82, 83, 84, 85, 86, 87, 88, 89, 90, 91, 92, 93, 94, 95)
LG_ACC(6, 96, 111, 96, 97, 98, 99, 100, 101, 102, 103, 104, 105, 106, 107, 108, 109, 110, 111)
LG_ACC(7, 112, 127, 112, 113, 114, 115, 116, 117, 118, 119, 120, 121, 122, 123, 124, 125, 126, 127)
LG_ACC(8, 128, 143, 128, 129, 130, 131, 132, 133, 134, 135, 136, 137, 138, 139, 140, 141, 142, 143)
LG_ACC(9, 144, 159, 144, 145, 146, 147, 148, 149, 150, 151, 152, 153, 154, 155, 156, 157, 158, 159)
LG_ACC(10, 160, 175, 160, 161, 162, 163, 164, 165, 166, 167, 168, 169, 170, 171, 172, 173, 174, 175)
LG_ACC(11, 176, 191, 176, 177, 178, 179, 180, 181, 182, 183, 184, 185, 186, 187, 188, 189, 190, 191)
LG_ACC(12, 192, 207, 192, 193, 194, 195, 196, 197, 198, 199, 200, 201, 202, 203, 204, 205, 206, 207)
LG_ACC(13, 208, 223, 208, 209, 210, 211, 212, 213, 214, 215, 216, 217, 218, 219, 220, 221, 222, 223)
LG_ACC(14, 224, 239, 224, 225, 226, 227, 228, 229, 230, 231, 232, 233, 234, 235, 236, 237, 238, 239)
LG_ACC(15, 240, 255, 240, 241, 242, 243, 244, 245, 246, 247, 248, 249, 250, 251, 252, 253, 254, 255)
#undef LG_ACC
#define LG_ACC_CASES(OP)                                                                                   \
  switch (i) {                                                                                             \
    case 0: OP(0); break; case 1: OP(1); break; case 2: OP(2); break; case 3: OP(3); break;                \
    case 4: OP(4); break; case 5: OP(5); break; case 6: OP(6); break; case 7: OP(7); break;                \
    case 8: OP(8); break; case 9: OP(9); break; case 10: OP(10); break; case 11: OP(11); break;            \
    case 12: OP(12); break; case 13: OP(13); break; case 14: OP(14); break; default: OP(15); break;        \
  }
// i is a compile-time constant at every call (fully unrolled loops): the switch folds away
__device__ __forceinline__ void lg_acc_fma(int i, bf16x8_t a, bf16x8_t b) {
#define LG_OP(I) LgAcc<I>::fma(a, b)
  LG_ACC_CASES(LG_OP)
#undef LG_OP
}
__device__ __forceinline__ void lg_acc_zero(int i, bf16x8_t z) {
#define LG_OP(I) LgAcc<I>::zero(z)
  LG_ACC_CASES(LG_OP)
#undef LG_OP
}
__device__ __forceinline__ void lg_acc_get(int i, float* x) {
#define LG_OP(I) LgAcc<I>::get(x)
  LG_ACC_CASES(LG_OP)
#undef LG_OP
}
__device__ __forceinline__ void lg_mfma_v(f32x16_t& c, bf16x8_t a, bf16x8_t b) {  // accumulate in VGPRs
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
}
__device__ __forceinline__ void lg_mfma_vi(f32x16_t& c, bf16x8_t a, bf16x8_t b, const f32x16_t& init) {  // c = a b + init
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(c) : "v"(a), "v"(b), "v"(init));
}
// Operands that vector instructions produce (P / dS rounded to bf16, the zero operand) must be
// complete a few issue slots before the matrix instruction that reads them: the pieces that produce
// P / dS end at least one matrix instruction earlier, the zero operand is followed by idle slots.
// Program-order anchor without an instruction: everything that reads x or y is placed after this
// point, everything that wrote them before it.  A vector instruction may read the result of an 8-pass
// matrix instruction only 11 issue slots after that instruction was issued, and neither the hardware nor the
// compiler (which does not look inside the statements) waits for it.  Four later matrix instructions
// guarantee those slots whatever the state of the pipe; the unrolled steps keep LG_MFMA_GAP = 6, as
// compile-time assertions on the instruction indices (lg_readable_after), and tests/test_build_isa.py checks
// the distance in the generated code.
__device__ __forceinline__ void lg_tie(f32x16_t& x, f32x16_t& y) { asm volatile("" : "+v"(x), "+v"(y)); }
constexpr int LG_MFMA_GAP = 6;
// Vector code placed after matrix instruction number `reader` of an unrolled step may read what
// instruction number `last_writer` (the last of an accumulation chain) wrote.
constexpr bool lg_readable_after(int reader, int last_writer) { return reader >= last_writer + LG_MFMA_GAP; }
// A matrix instruction number `consumer` may read an operand that the vector piece placed after
// instruction number `last_piece` completed: at least one whole matrix instruction lies in between.
constexpr bool lg_operand_ready(int consumer, int last_piece) { return consumer >= last_piece + 2; }

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order
template <int... I, typename F>
__device__ __forceinline__ void lg_static_for_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void lg_static_for(F&& f) {
  lg_static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

template <int I>
struct LgFrag;
#define LG_FRAG(I, LO, HI, R0, R1, R2, R3)                                                                     \
  template <>                                                                                                  \
  struct LgFrag<I> {                                                                                           \
    static __device__ __forceinline__ void set(uint4 v) {                                                      \
      asm volatile("v_accvgpr_write_b32 a" #R0 ", %0\n\tv_accvgpr_write_b32 a" #R1 ", %1\n\t"                   \
                   "v_accvgpr_write_b32 a" #R2 ", %2\n\tv_accvgpr_write_b32 a" #R3 ", %3" ::"v"(v.x),            \
                   "v"(v.y), "v"(v.z), "v"(v.w)                                                                \
                   : "a" #R0, "a" #R1, "a" #R2, "a" #R3);                                                      \
    }                                                                                                          \
    static __device__ __forceinline__ void fma(f32x16_t& c, bf16x8_t a) {                                      \
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, a[" #LO ":" #HI "], %0" : "+v"(c) : "v"(a));               \
    }                                                                                                          \
    static __device__ __forceinline__ void mul(f32x16_t& c, bf16x8_t a) {                                      \
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, a[" #LO ":" #HI "], 0" : "=&v"(c) : "v"(a));               \
    }                                                                                                          \
    static __device__ __forceinline__ void mad(f32x16_t& c, bf16x8_t a, const f32x16_t& init) {                \
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, a[" #LO ":" #HI "], %2" : "=&v"(c) : "v"(a), "v"(init));   \
    }                                                                                                          \
  };
LG_FRAG(0, 128, 131, 128, 129, 130, 131)
LG_FRAG(1, 132, 135, 132, 133, 134, 135)
LG_FRAG(2, 136, 139, 136, 137, 138, 139)
LG_FRAG(3, 140, 143, 140, 141, 142, 143)
LG_FRAG(4, 144, 147, 144, 145, 146, 147)
LG_FRAG(5, 148, 151, 148, 149, 150, 151)
LG_FRAG(6, 152, 155, 152, 153, 154, 155)
LG_FRAG(7, 156, 159, 156, 157, 158, 159)
LG_FRAG(8, 160, 163, 160, 161, 162, 163)
LG_FRAG(9, 164, 167, 164, 165, 166, 167)
LG_FRAG(10, 168, 171, 168, 169, 170, 171)
LG_FRAG(11, 172, 175, 172, 173, 174, 175)
LG_FRAG(12, 176, 179, 176, 177, 178, 179)
LG_FRAG(13, 180, 183, 180, 181, 182, 183)
LG_FRAG(14, 184, 187, 184, 185, 186, 187)
LG_FRAG(15, 188, 191, 188, 189, 190, 191)
LG_FRAG(16, 192, 195, 192, 193, 194, 195)
LG_FRAG(17, 196, 199, 196, 197, 198, 199)
LG_FRAG(18, 200, 203, 200, 201, 202, 203)
LG_FRAG(19, 204, 207, 204, 205, 206, 207)
LG_FRAG(20, 208, 211, 208, 209, 210, 211)
LG_FRAG(21, 212, 215, 212, 213, 214, 215)
LG_FRAG(22, 216, 219, 216, 217, 218, 219)
LG_FRAG(23, 220, 223, 220, 221, 222, 223)
LG_FRAG(24, 224, 227, 224, 225, 226, 227)
LG_FRAG(25, 228, 231, 228, 229, 230, 231)
LG_FRAG(26, 232, 235, 232, 233, 234, 235)
LG_FRAG(27, 236, 239, 236, 237, 238, 239)
LG_FRAG(28, 240, 243, 240, 241, 242, 243)
LG_FRAG(29, 244, 247, 244, 245, 246, 247)
LG_FRAG(30, 248, 251, 248, 249, 250, 251)
LG_FRAG(31, 252, 255, 252, 253, 254, 255)
#undef LG_FRAG
#define LG_FRAG_CASES(OP) \
  switch (i) { case 0: OP(0); break; case 1: OP(1); break; case 2: OP(2); break; case 3: OP(3); break; case 4: OP(4); break; case 5: OP(5); break; case 6: OP(6); break; case 7: OP(7); break; case 8: OP(8); break; case 9: OP(9); break; case 10: OP(10); break; case 11: OP(11); break; case 12: OP(12); break; case 13: OP(13); break; case 14: OP(14); break; case 15: OP(15); break; case 16: OP(16); break; case 17: OP(17); break; case 18: OP(18); break; case 19: OP(19); break; case 20: OP(20); break; case 21: OP(21); break; case 22: OP(22); break; case 23: OP(23); break; case 24: OP(24); break; case 25: OP(25); break; case 26: OP(26); break; case 27: OP(27); break; case 28: OP(28); break; case 29: OP(29); break; case 30: OP(30); break; default: OP(31); break; }
// i is a compile-time constant at every call: the switch folds away
__device__ __forceinline__ void lg_frag_set(int i, uint4 v) {
#define LG_OP(I) LgFrag<I>::set(v)
  LG_FRAG_CASES(LG_OP)
#undef LG_OP
}
// c = init + a * fragment i
__device__ __forceinline__ void lg_frag_mfma_init(int i, f32x16_t& c, bf16x8_t a, const f32x16_t& init) {
#define LG_OP(I) LgFrag<I>::mad(c, a, init)
  LG_FRAG_CASES(LG_OP)
#undef LG_OP
}
// c = (first ? 0 : c) + a * fragment i
__device__ __forceinline__ void lg_frag_mfma(int i, bool first, f32x16_t& c, bf16x8_t a) {
#define LG_OP(I)                    \
  do {                              \
    if (first) LgFrag<I>::mul(c, a); \
    else LgFrag<I>::fma(c, a);      \
  } while (0)
  LG_FRAG_CASES(LG_OP)
#undef LG_OP
}

}  // namespace

#endif  // LG_WIDE_H_
