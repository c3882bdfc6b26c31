// gfx950 matrix-core helpers: 16-bit MFMA wrappers and their register layouts.
//
// Numerics of the library: weights are bf16 (as given); every activation that feeds a matrix
// product (normed rows, queries, cached keys/values, softmax weights, FFN activations, final hidden
// state) is IEEE fp16, because bf16's 8-bit mantissa on activations exceeds the logit tolerance
// after a few layers while fp16's 11 bits keep a 32-layer model inside it. bf16 weights are widened
// to fp16 in registers right after the load (exact for |w| >= 2^-14; smaller weights keep an
// absolute error below 2^-24) and all products run on v_mfma_f32_*_f16 with fp32 accumulation.
//
// v_mfma_f32_16x16x32_f16 (D = A[16x32] * B[32x16] + C), wave64, lane l, g = l / 16:
//   A: lane holds A[row = l % 16][k = 8 g .. 8 g + 7]      (8 halves, one 16-byte register quad)
//   B: lane holds B[k = 8 g .. 8 g + 7][col = l % 16]
//   D: lane holds D[row = 4 g + i][col = l % 16], i = 0..3
// v_mfma_f32_16x16x16_f16: same with k = 4 g .. 4 g + 3 (4 halves per lane).
// Only products of equal k meet, so A and B may use ANY common permutation of k: kernels exploit
// that to let each lane read long contiguous runs of the streamed operand.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace laser {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));   // native 16-byte vector (arrays of it stay in registers)

union Frag8 {            // 8 x 16-bit = 16 bytes (fp16 for MFMA operands; raw bf16 right after a weight load)
    uint4 u;
    u32x4 v4;
    uint32_t w[4];
    half8_t v;
    half2_t v2[4];
    uint16_t h[8];
};
union Frag4 {            // 4 x fp16 = 8 bytes
    uint2 u;
    u32x2 v2;
    half4_t v;
    uint16_t h[4];
};

__device__ inline float4_t mfma_16x16x32(const Frag8& a, const Frag8& b, float4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a.v, b.v, c, 0, 0, 0);
}
__device__ inline float4_t mfma_16x16x16(const Frag4& a, const Frag4& b, float4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x16f16(a.v, b.v, c, 0, 0, 0);
}

__device__ inline float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// 8 bf16 (as loaded) -> 8 fp16, in place. Truncation never triggers for normal-range results
// because bf16 has fewer mantissa bits than fp16.
__device__ inline void bf16x8_to_f16x8(Frag8& f) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t u = f.w[i];
        f.w[i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(__uint_as_float(u << 16), __uint_as_float(u & 0xFFFF0000u)));
    }
}

__device__ inline uint16_t f32_to_f16(float f) {            // round to nearest even
    _Float16 h = (_Float16)f;
    return __builtin_bit_cast(uint16_t, h);
}
__device__ inline float f16_to_f32(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }

}  // namespace laser
