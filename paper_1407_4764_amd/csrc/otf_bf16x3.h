// fp32-accurate products on the bf16 matrix instructions.
//
// Measured on this chip: v_mfma_f32_32x32x2_f32 and the vector ALU do not overlap (a SIMD that
// alternates them takes the sum of the two times), whereas v_mfma_f32_32x32x16_bf16 runs beside the
// ALU and does eight times the multiply-adds of the fp32 instruction in half the cycles.  An fp32
// value is the exact sum of three bf16 pieces (8 mantissa bits each, truncating splits), and the
// product of two pieces is exact in the fp32 accumulator, so <x, c> in fp32 accuracy is the sum of
// the six piece products of order <= 2: x0c0 + x0c1 + x1c0 + x0c2 + x1c1 + x2c0 (the three left
// out are below 2^-23 of |x_i c_i|).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace otf {

typedef float float16v __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float top16(float v) { return __uint_as_float(__float_as_uint(v) & 0xFFFF0000u); }

// The three bf16 pieces of v0 and of v1, as dwords {low half: v0's piece, high half: v1's}.
__device__ __forceinline__ void split3(float v0, float v1, uint32_t &p0, uint32_t &p1, uint32_t &p2) {
    const float r0 = v0 - top16(v0), r1 = v1 - top16(v1);   // exact: the low 16 mantissa bits
    const float s0 = r0 - top16(r0), s1 = r1 - top16(r1);   // exact: at most 8 bits are left
    p0 = __builtin_amdgcn_perm(__float_as_uint(v1), __float_as_uint(v0), 0x07060302u);
    p1 = __builtin_amdgcn_perm(__float_as_uint(r1), __float_as_uint(r0), 0x07060302u);
    p2 = __builtin_amdgcn_perm(__float_as_uint(s1), __float_as_uint(s0), 0x07060302u);
}

// Operands: lane (i, g) of the wave holds row i (A) or column i (B) of a 32 x 32 block and its K
// slots 8 g .. 8 g + 7, two per dword.
__device__ __forceinline__ float16v mfma_bf16(u32x4 a, u32x4 b, float16v c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

}  // namespace otf
