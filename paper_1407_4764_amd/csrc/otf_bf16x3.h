// fp32-accurate products on the bf16 matrix instructions.
//
// Measured on this chip: v_mfma_f32_32x32x2_f32 and the vector ALU do not overlap (a SIMD that
// alternates them takes the sum of the two times), whereas v_mfma_f32_32x32x16_bf16 runs beside the
// ALU and does eight times the multiply-adds of the fp32 instruction in half the cycles.  A finite
// fp32 value v is the exact sum of three bf16 pieces: p0 = bf16(v), p1 = bf16(v - p0),
// p2 = v - p0 - p1 (round to nearest each time: both differences are exact in fp32 and the last
// has at most 8 significant bits left), with |p1| <= 2^-8 |v| and |p2| <= 2^-16 |v| up to a factor
// (1 + 2^-7).  The product of two pieces is exact in the fp32 accumulator, so <x, c> in fp32
// accuracy is the sum of the six piece products of order <= 2: x0c0 + x0c1 + x1c0 + x0c2 + x1c1 +
// x2c0; the three left out are below 2^-22 of |x_i c_i| together.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace otf {

typedef float float16v __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// {low half: bf16(lo), high half: bf16(hi)}, round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){lo, hi}, bf16x2));
}
__device__ __forceinline__ float bf16_lo(uint32_t pk) { return __uint_as_float(pk << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t pk) { return __uint_as_float(pk & 0xFFFF0000u); }

// The three bf16 pieces of v0 and of v1, as dwords {low half: v0's piece, high half: v1's}.
__device__ __forceinline__ void split3(float v0, float v1, uint32_t &p0, uint32_t &p1, uint32_t &p2) {
    p0 = pack_bf16(v0, v1);
    const float r0 = v0 - bf16_lo(p0), r1 = v1 - bf16_hi(p0);   // exact
    p1 = pack_bf16(r0, r1);
    p2 = pack_bf16(r0 - bf16_lo(p1), r1 - bf16_hi(p1));         // exact differences that fit a bf16
}

// Operands: lane (i, g) of the wave holds row i (A) or column i (B) of a 32 x 32 block and its K
// slots 8 g .. 8 g + 7, two per dword.
__device__ __forceinline__ float16v mfma_bf16(u32x4 a, u32x4 b, float16v c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

}  // namespace otf
