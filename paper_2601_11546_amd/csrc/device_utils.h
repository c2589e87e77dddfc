// Small device helpers for the gfx950 kernels: bf16 packing, wave reductions, MFMA types.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace relserve {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef int i32x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// fp32 -> bf16, round to nearest even (NaN stays NaN): gfx950's conversion instructions
// (v_cvt_pk_bf16_f32 rounds two values at once).
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) { return pack_bf16x2(f, 0.f) & 0xffffu; }

// Four fp32 values -> four 8-bit floating point codes (1-4-3 bits, bias 7), round to nearest even, in memory order.
// Magnitudes are limited to 448, the format's largest, before the conversion, so that its own overflow rule never
// matters.
__device__ __forceinline__ uint32_t pack_fp8x4(float a, float b, float c, float d) {
    a = __builtin_amdgcn_fmed3f(a, -448.0f, 448.0f);
    b = __builtin_amdgcn_fmed3f(b, -448.0f, 448.0f);
    c = __builtin_amdgcn_fmed3f(c, -448.0f, 448.0f);
    d = __builtin_amdgcn_fmed3f(d, -448.0f, 448.0f);
    int r = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
    r = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, r, true);
    return (uint32_t)r;
}

// Eight such codes (8 bytes) -> eight bf16 values (every code is a bf16 number: four significant bits).
__device__ __forceinline__ uint4 fp8x8_to_bf16x8(uint2 raw) {
    const f32x2_t a = __builtin_amdgcn_cvt_pk_f32_fp8((int)raw.x, false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)raw.x, true);
    const f32x2_t c = __builtin_amdgcn_cvt_pk_f32_fp8((int)raw.y, false), d = __builtin_amdgcn_cvt_pk_f32_fp8((int)raw.y, true);
    return make_uint4(pack_bf16x2(a[0], a[1]), pack_bf16x2(b[0], b[1]), pack_bf16x2(c[0], c[1]), pack_bf16x2(d[0], d[1]));
}

// silu(gate) * up = gate * up / (1 + e^-gate) with the hardware exponential and reciprocal (about one unit in the
// last place each, far below the bf16 rounding of the result); a full-precision division would cost ten instructions.
__device__ __forceinline__ float silu_mul(float gate, float up) {
    return gate * up * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(gate * -1.4426950408889634f));
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ bf16x8_t as_bf16x8(uint4 u) { return __builtin_bit_cast(bf16x8_t, u); }

// D[i][j] += sum_k A[i][k] B[k][j], 32x32 output, k = 16.  Lane l holds A[l % 32][8 (l / 32) ..+7],
// B[8 (l / 32) ..+7][l % 32]; accumulator register r holds D[8 (r / 4) + 4 (l / 32) + r % 4][l % 32].
__device__ __forceinline__ f32x16_t mfma_32x32x16(bf16x8_t a, bf16x8_t b, f32x16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// 32x32x64 product of 8-bit floating point codes (1-4-3 bits, both operands), fp32 accumulate: lane (l32, g) supplies
// row l32 and 32 of the 64 k values (half g) of each operand.  The scale operands are zero: the unscaled instruction.
__device__ __forceinline__ f32x16_t mfma_32x32x64_f8(i32x8_t a, i32x8_t b, f32x16_t c) {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0);
}

}  // namespace relserve
