// gfx950 matrix-core helpers: 16-bit MFMA wrappers and their register layouts.
//
// Numerics of the library: weights are bf16 (as given); every activation that feeds a matrix
// product (normed rows, queries, cached keys/values, softmax weights, FFN activations, final hidden
// state) is IEEE fp16, because bf16's 8-bit mantissa on activations exceeds the logit tolerance
// after a few layers while fp16's 11 bits keep a 32-layer model inside it. bf16 weights are widened
// to fp16 in registers right after the load (exact for |w| >= 2^-14; smaller weights keep an
// absolute error below 2^-24) and all products run on v_mfma_f32_*_f16 with fp32 accumulation.
//
// Split operands. At the 7B shape (32 layers, width 4096, weights of standard deviation 0.02) a single
// fp16 rounding of the normed rows, queries, keys or attention outputs already moves the logits by
// 0.2-0.45 % of their spread each, and together they exceed the logit tolerance. Those tensors are
// therefore carried as TWO fp16 planes, hi = fp16(x) and lo = fp16(4096 (x - hi)), and every product
// with them is evaluated as W.hi + 2^-12 W.lo (two matrix instructions sharing the weight operand, two
// accumulators). The factor 4096 keeps lo in the normal fp16 range whenever hi is. Values, softmax
// weights and FFN activations stay single fp16.
// Where LDS space is the limit (the persistent few-row kernel stages its activation rows there) the low
// plane is narrowed to 8 bits, the upper byte of its fp16 pattern rounded to nearest (sign, 5 exponent
// bits, 2 fraction bits): the operand then carries 11 + 3 significant bits. It is widened back to fp16 by
// a byte permute on its way into the matrix instruction.
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

#include <type_traits>

namespace laser {

// f(integral_constant<int, J>) for J = J0 .. N-1, unrolled at compile time: ring slots and fragment sets indexed
// by J stay in named registers.
template <int J, int N, class F>
__device__ inline void static_for(F&& f) {
    if constexpr (J < N) { f(std::integral_constant<int, J>{}); static_for<J + 1, N>(f); }
}

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

constexpr float kLoScale = 4096.f, kLoInv = 1.f / 4096.f;
// x -> (hi, lo) with x ~= hi + lo / 4096
__device__ inline void split_f16(float x, uint16_t& hi, uint16_t& lo) {
    const _Float16 h = (_Float16)x;
    hi = __builtin_bit_cast(uint16_t, h);
    lo = __builtin_bit_cast(uint16_t, (_Float16)((x - (float)h) * kLoScale));
}
// fp16 pattern -> its upper byte, rounded to nearest even
__device__ inline uint32_t f16_to_b8(uint16_t h) { return ((uint32_t)h + 0x7Fu + ((h >> 8) & 1u)) >> 8; }
// two values -> packed fp16 high parts and packed 8-bit low parts
__device__ inline void split_pack_h2_b8(float a, float b, uint32_t& hi, uint16_t& lo8) {
    uint16_t ah, al, bh, bl;
    split_f16(a, ah, al);
    split_f16(b, bh, bl);
    hi = (uint32_t)ah | ((uint32_t)bh << 16);
    lo8 = (uint16_t)(f16_to_b8(al) | (f16_to_b8(bl) << 8));
}
// 8 low-plane bytes (two dwords) -> 8 fp16
__device__ inline void b8x8_to_f16x8(uint32_t d0, uint32_t d1, Frag8& f) {
    f.w[0] = __builtin_amdgcn_perm(0u, d0, 0x010C000Cu);
    f.w[1] = __builtin_amdgcn_perm(0u, d0, 0x030C020Cu);
    f.w[2] = __builtin_amdgcn_perm(0u, d1, 0x010C000Cu);
    f.w[3] = __builtin_amdgcn_perm(0u, d1, 0x030C020Cu);
}
__device__ inline void split_pack_h2(float a, float b, uint32_t& hi, uint32_t& lo) {
    uint16_t ah, al, bh, bl;
    split_f16(a, ah, al);
    split_f16(b, bh, bl);
    hi = (uint32_t)ah | ((uint32_t)bh << 16);
    lo = (uint32_t)al | ((uint32_t)bl << 16);
}

}  // namespace laser
