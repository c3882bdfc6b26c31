// Weight-streaming GEMM for few activation rows (M = B*(K+1) from 1 to a few hundred):
//   Y[M][N] = X[M][Kd] * W[N][Kd]^T,  W bf16 (widened to fp16 in registers), X fp16, fp32 accumulation
//   on the matrix cores.
//
// The weight matrix is read exactly once from HBM and never staged: each wavefront owns 16 output
// features (MFMA "A" operand) and walks the reduction dimension; a lane loads 64 contiguous bytes of
// its weight row per step (lane l -> row l%16, bytes [64*(l/16), +64) of a 256-byte row segment), so
// one wave-step covers 16 rows x 256 contiguous bytes. The activation rows are the "B" operand,
// re-read from L2 (they are tiny). MFMA reduction indices are permuted identically on both operands,
// which the instruction permits, to get those long per-lane runs.
#pragma once

#include "mfma.h"

namespace laser {

constexpr int kGemmKStep = 128;   // reduction elements per wave step

// acc[mb][i] <-> feature (n0 + 4*(lane/16) + i), row (row0 + 16*mb + lane%16)
// SPLIT: the activations come as two fp16 planes (X, Xlo with x = X + Xlo / 4096); the weight fragment
// meets both and the low products are accumulated apart, then folded in.
template <int MB, bool SPLIT>
__device__ inline void wave_gemm_tile(const uint16_t* __restrict__ Wrow0, size_t ldw,
                                      const uint16_t* __restrict__ X, const uint16_t* __restrict__ Xlo, int ldx, int M, int row0,
                                      int kbeg, int kend, float4_t (&acc)[MB]) {
    const int lane = threadIdx.x & 63;
    const int r = lane & 15, g = lane >> 4;
    const uint16_t* wp = Wrow0 + (size_t)r * ldw + g * 32;
    const uint16_t* xp[MB];
    const uint16_t* xlp[MB];
    float4_t acl[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        int row = row0 + mb * 16 + r;
        row = row < M ? row : M - 1;
        xp[mb] = X + (size_t)row * ldx + g * 32;
        xlp[mb] = SPLIT ? Xlo + (size_t)row * ldx + g * 32 : nullptr;
        acl[mb] = float4_t{0.f, 0.f, 0.f, 0.f};
    }
    Frag8 a_cur[4], a_nxt[4];
    if (kbeg < kend) {
#pragma unroll
        for (int c = 0; c < 4; ++c) a_cur[c].u = *reinterpret_cast<const uint4*>(wp + kbeg + c * 8);
    }
    for (int k0 = kbeg; k0 < kend; k0 += kGemmKStep) {
        const int kn = k0 + kGemmKStep;
        if (kn < kend) {
#pragma unroll
            for (int c = 0; c < 4; ++c) a_nxt[c].u = *reinterpret_cast<const uint4*>(wp + kn + c * 8);
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) bf16x8_to_f16x8(a_cur[c]);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            Frag8 b[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) b[c].u = *reinterpret_cast<const uint4*>(xp[mb] + k0 + c * 8);
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[mb] = mfma_16x16x32(a_cur[c], b[c], acc[mb]);
            if constexpr (SPLIT) {
                Frag8 bl[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) bl[c].u = *reinterpret_cast<const uint4*>(xlp[mb] + k0 + c * 8);
#pragma unroll
                for (int c = 0; c < 4; ++c) acl[mb] = mfma_16x16x32(a_cur[c], bl[c], acl[mb]);
            }
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) a_cur[c] = a_nxt[c];
    }
    if constexpr (SPLIT) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[mb][i] += acl[mb][i] * kLoInv;
    }
}

}  // namespace laser
