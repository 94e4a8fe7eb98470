// Building blocks for the bf16 MFMA kernels (gfx950).
#pragma once

#include "flurka_internal.h"

namespace flurka {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;

// v_mfma_f32_32x32x16_bf16, one wavefront: D(32x32) += A(32x16) B(16x32).
// Operand layout, lane l (verified on hardware):
//   A: row l%32, reduction slots 8*(l/32) .. +7        (8 bf16, 16 bytes)
//   B: column l%32, reduction slots 8*(l/32) .. +7
//   D: column l%32, element g (0..15) is row 8*(g/4) + 4*(l/32) + g%4
__device__ __forceinline__ floatx16 mfma32(const uint4& a, const uint4& b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

__device__ __forceinline__ floatx16 zero16() {
    floatx16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
    return z;
}

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float floatx2;

// two floats -> packed bf16 pair (low half = a), round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    const floatx2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// 2^x on the transcendental unit, no denormal fix-up (inputs here are <= 0 and results that
// underflow are meant to be 0)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint4 ld16(const void* p) { return *(const uint4*)p; }

}  // namespace flurka
