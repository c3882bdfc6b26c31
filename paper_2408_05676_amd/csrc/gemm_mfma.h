// LDS-tiled matrix-core GEMM for many activation rows (M = B*(K+1) in the hundreds):
//   Y[M][N] = X[M][Kd] * W[N][Kd]^T,  X fp16, W bf16 (widened to fp16 on its way into LDS), fp32 accumulate.
//
// Workgroup tile 128 x 128, 256 threads = 2 x 2 waves of 64 x 64, each wave 2 x 2
// v_mfma_f32_32x32x16_f16 tiles (64 accumulator registers). Reduction step 64; three stages in flight: the
// global loads of step kt + 2 (registers), the conversion and LDS write of step kt + 1 (interleaved with the
// matrix instructions), the multiplication of step kt out of one of two LDS buffers (36 KiB each pair, rows
// padded 128 -> 144 bytes against bank conflicts); one workgroup barrier per step; two workgroups per CU. Measured at M = 704, N = 12288, K = 4096:
// 108-114 us = 25 % of the fp16 matrix peak (reduction step 32: 115-120 us, 16: 170 us, 128: 151 us).
// Counters show 89 % L2 hits and the weights fetched from HBM once per launch, i.e. the XCD-aware tile
// order works; what is left is the quantisation of 576 tiles over 256 CUs (75 %) and the L2 -> LDS ->
// register path.
//
// v_mfma_f32_32x32x16_f16, wave64, lane l, g = l / 32:
//   A: lane holds A[row = l % 32][k = 8 g .. 8 g + 7];  B: lane holds B[k = 8 g .. 8 g + 7][col = l % 32]
//   D: lane holds D[row = 8 (i / 4) + 4 g + i % 4][col = l % 32], i = 0..15
//
// Workgroup ids are remapped so that the workgroups sharing a weight tile (same n-tile, all m-tiles)
// have consecutive "virtual" ids on ONE XCD (hardware deals consecutive ids round-robin over the 8
// XCDs, each with its own L2): the weight tile is then fetched from HBM once and hit in that L2.
#pragma once

#include <type_traits>

#include "head_part.h"
#include "mfma.h"

namespace laser {

typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int GM_BM = 128, GM_BN = 128;
constexpr int GM_BK_PLAIN = 64, GM_WGS = 2;   // unsplit kernels: reduction step, workgroups per CU
constexpr int GM_DEPTH = 2;         // register slots per thread: GM_DEPTH - 1 k-steps of global loads in flight (even)

struct GemmTileArgs {
    const uint16_t* W;      // [N][Kd] bf16, or the same values already widened to fp16 (WF16 kernels)
                            // (SwiGLU: [2F][Kd], gate rows then up rows; N = F)
    const uint16_t* X;      // [M][Kd] fp16
    const uint16_t* Xlo;    // [M][Kd] low plane of split activations (x = X + Xlo / 4096), SPLIT kernels only
    int M, N, Kd;
    int tiles_m, tiles_n;   // tiles_n counts BN-column tiles (SwiGLU: 64-feature tiles), times ksplit
    int ksplit;             // > 1: the reduction is cut into ksplit equal parts, each a unit of its own that STORES its
                            // partial result at outf + part * M * N (store epilogue only; the consumer adds the parts
                            // in a fixed order). It evens out tile counts that do not fill the chip's slots.
    float* outf;            // EPI_F32: [M][N] store; EPI_RESID: [M][N] accumulate
    uint16_t* outh;         // EPI_SWIGLU: [M][N] fp16
    HeadPart hp{};          // GEPI_HEAD: where the per-(row, n-tile) statistics go (chunk = n-tile)
};

// GEPI_HEAD: the output head. The tile's logits are not stored: each row's 128 columns are reduced to one record of
// partial statistics (head_part.h).
enum { GEPI_F32 = 0, GEPI_RESID = 1, GEPI_SWIGLU = 2, GEPI_HEAD = 3 };

// workgroups of a launch: 8 x the largest per-XCD tile count (n-tiles are dealt round-robin to the XCDs)
inline unsigned gemm_mfma_grid(int tiles_m, int tiles_n) { return 8u * (unsigned)(((tiles_n + 7) / 8) * tiles_m); }

__device__ inline float16_t mfma_32x32x16(const Frag8& a, const Frag8& b, float16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a.v, b.v, c, 0, 0, 0);
}

// weight row behind tile column j (0..BN-1) of n-tile tn
template <int EPI, int BN>
__device__ inline int w_row(const GemmTileArgs& a, int tn, int j) {
    if (EPI == GEPI_SWIGLU) {
        // columns of a wave: [32 gate | 32 up] of the same 32 features, so that one lane holds both
        const int wn = j >> 6, ct = (j >> 5) & 1, c = j & 31;
        return (ct ? a.N : 0) + tn * 64 + wn * 32 + c;
    }
    return tn * BN + j;
}


// BN = 128: 2 x 2 waves of 64 x 64. BN = 64 (narrow outputs, where 128-column tiles would leave CUs
// without work): 2 x 2 waves of 64 x 32. The SwiGLU epilogue needs BN = 128.
// SPLIT: the activations come as two fp16 planes; every weight fragment meets both (second accumulator
// set, folded in with the factor 2^-12 at the end). The reduction step drops to 32 so that the third
// LDS tile still leaves room for two workgroups per CU.
// WF16: the weights were widened to fp16 beforehand (the model handle keeps such a copy for the many-row
// path): the loop then has no conversion arithmetic, which otherwise competes with the matrix instructions
// for issue slots (about 50 of the ~100 vector instructions per k-step).
template <int EPI, int BN, bool SPLIT, bool WF16 = false>
__global__ __launch_bounds__(256, SPLIT ? 2 : GM_WGS) void gemm_mfma_kernel(GemmTileArgs a) {
    static_assert(BN == 128 || (BN == 64 && EPI != GEPI_SWIGLU), "tile width");
    constexpr int GM_BK = SPLIT ? 32 : GM_BK_PLAIN;   // reduction step
    // LDS rows. Single-plane kernel: 64 + 8 halves, the padding spreads 16-byte reads of consecutive rows over the banks.
    // Split kernel (step 32): padded 80-byte rows left a third of the LDS-active cycles in bank conflicts (hardware
    // counter), so its rows are unpadded 64 bytes and the four 16-byte chunks of row r sit at chunk ^ ((r >> 2) & 3):
    // 16 consecutive rows at one logical chunk, and 4 rows x 4 chunks of a staging write, each touch 16 distinct
    // 16-byte bank groups.
    constexpr bool SWZ = SPLIT;
    constexpr int GM_LD = SWZ ? GM_BK : GM_BK + 8;
    constexpr int CH = GM_BK / 8;            // 16-byte chunks per tile row and k-step
    constexpr int RPT = 256 / CH;            // rows staged per pass of the 256 threads
    constexpr int ST = GM_BM / RPT;          // passes over the activation rows
    constexpr int STB = BN / RPT;            // passes over the weight rows
    constexpr int WN = BN / 2;               // columns per wave
    constexpr int NJ = WN / 32;              // 32-column MFMA tiles per wave
    constexpr int D = (SPLIT && BN == 128) ? 2 : (SPLIT ? 4 : GM_DEPTH);   // the split 128-column kernel has no registers for a deeper ring
    __shared__ __attribute__((aligned(16))) uint16_t sA[2][GM_BM][GM_LD];
    __shared__ __attribute__((aligned(16))) uint16_t sB[2][BN][GM_LD];
    __shared__ __attribute__((aligned(16))) uint16_t sAl[SPLIT ? 2 : 1][SPLIT ? GM_BM : 1][SPLIT ? GM_LD : 8];
    // ---- XCD-aware tile order, longest tiles first ----
    // n-tile tn belongs to XCD tn % 8 (consecutive workgroup ids go round-robin over the XCDs). Inside an XCD the
    // workgroups come in dispatch order: first every FULL m-tile of every owned n-tile (m fastest, so the m-tiles
    // that share a weight tile run together and hit it in L2), then the ragged last m-tiles, whose dead waves make
    // them finish in about half the time: issued last they fill the tail of the launch instead of holding slots
    // that full tiles are waiting for (704 rows: QKV 199 -> 189 us, gate/up 169 -> 167 us).
    const int xcd = blockIdx.x % 8, li = blockIdx.x / 8;
    const int nt_x = (a.tiles_n - xcd + 7) / 8;                 // n-tiles owned by this XCD
    const bool ragged = a.M % GM_BM != 0 && a.tiles_m > 1;
    const int full_m = ragged ? a.tiles_m - 1 : a.tiles_m;
    if (li >= nt_x * a.tiles_m) return;
    int tn, tm;
    if (li < nt_x * full_m) { tn = xcd + 8 * (li / full_m); tm = li % full_m; }
    else { tn = xcd + 8 * (li - nt_x * full_m); tm = a.tiles_m - 1; }
    const int kpart = tn % a.ksplit;          // (n-tile, reduction part) pairs were dealt out as one index
    tn /= a.ksplit;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = lane & 31, lg = lane >> 5;

    // global -> LDS staging: thread t moves chunk t % CH of rows t / CH + RPT i of both operands
    const int srow = tid / CH, sk = (tid % CH) * 8;
    const int skw = SWZ ? ((tid % CH) ^ ((srow >> 2) & 3)) * 8 : sk;       // LDS column of this thread's chunk (RPT is a multiple of 16)
    const uint16_t* xa[ST];
    const uint16_t* xl[ST];
    const uint16_t* wb[STB];
#pragma unroll
    for (int i = 0; i < ST; ++i) {
        int row = tm * GM_BM + srow + RPT * i;
        row = row < a.M ? row : a.M - 1;
        xa[i] = a.X + (size_t)row * a.Kd + sk;
        xl[i] = SPLIT ? a.Xlo + (size_t)row * a.Kd + sk : nullptr;
    }
#pragma unroll
    for (int i = 0; i < STB; ++i) {
        int wr = w_row<EPI, BN>(a, tn, srow + RPT * i);
        const int wmax = (EPI == GEPI_SWIGLU ? 2 * a.N : a.N) - 1;
        wr = wr < wmax ? wr : wmax;
        wb[i] = a.W + (size_t)wr * a.Kd + sk;
    }
    // head epilogue: thread t will own half of row t / 2; its candidate list is fetched now, under the main loop
    int hc_b = 0, hc_n = 0, hc_x0 = -1;
    if constexpr (EPI == GEPI_HEAD) {
        const int grow = tm * GM_BM + (tid >> 1);
        if (grow < a.M) { hc_b = a.hp.cand_beg[grow]; hc_n = a.hp.cand_cnt[grow]; }
        hc_x0 = hc_n > 0 ? a.hp.cand_x[hc_b] : -1;
    }
    float16_t acc[2][NJ];
    float16_t acl[SPLIT ? 2 : 1][SPLIT ? NJ : 1];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                acc[i][j][e] = 0.f;
                if constexpr (SPLIT) acl[i][j][e] = 0.f;
            }

    // a wave whose 64 rows all lie past M (ragged last m-tile) stages and synchronises but multiplies nothing
    const bool dead = __builtin_amdgcn_readfirstlane(tm * GM_BM + wm * 64) >= a.M;

    // Register ring of D k-steps. The element type must be a native vector: an array of HIP's uint4
    // (a struct) that is only copied as a whole is not promoted to registers and lands in scratch.
    u32x4 ra[D][ST], rb[D][STB], rl[D][SPLIT ? ST : 1];
    const int nk = a.Kd / GM_BK / a.ksplit;  // the host guarantees Kd % (GM_BK * ksplit) == 0
    {
        const int k0 = kpart * nk * GM_BK;
#pragma unroll
        for (int i = 0; i < ST; ++i) { xa[i] += k0; if constexpr (SPLIT) xl[i] += k0; }
#pragma unroll
        for (int i = 0; i < STB; ++i) wb[i] += k0;
    }
    float* const outf = a.outf ? a.outf + (size_t)kpart * a.M * a.N : nullptr;
    auto gload = [&](auto slot_c, int kt) {
        constexpr int slot = decltype(slot_c)::value;
        kt = kt < nk ? kt : nk - 1;          // unconditional, clamped: a load under a branch would be waited for at once
#pragma unroll
        for (int i = 0; i < ST; ++i) ra[slot][i] = *reinterpret_cast<const u32x4*>(xa[i] + kt * GM_BK);
        if constexpr (SPLIT) {
#pragma unroll
            for (int i = 0; i < ST; ++i) rl[slot][i] = *reinterpret_cast<const u32x4*>(xl[i] + kt * GM_BK);
        }
#pragma unroll
        for (int i = 0; i < STB; ++i) rb[slot][i] = *reinterpret_cast<const u32x4*>(wb[i] + kt * GM_BK);
    };
    // Software pipeline over k-steps: while step kt is multiplied out of LDS buffer kt % 2, the registers that
    // hold step kt + 1 are converted and written to the other buffer in pieces BETWEEN the matrix instructions
    // of the same basic block (so the vector ALU and LDS-write work hides behind the matrix pipe instead of
    // preceding it), and the global loads of step kt + 2 are in flight. One workgroup barrier per step: it
    // publishes buffer (kt + 1) % 2 and guarantees that every wave has finished reading buffer kt % 2 before
    // the next step overwrites it.
    constexpr int NKK = GM_BK / 16;
    auto stage_piece = [&](auto slot_c, int buf, int kk, unsigned keep) {       // piece kk (of NKK) of one k-step
        constexpr int slot = decltype(slot_c)::value;
#pragma unroll
        for (int i = 0; i < ST; ++i)
            if (i * NKK / ST == kk) {
                *reinterpret_cast<u32x4*>(&sA[buf][srow + RPT * i][skw]) = ra[slot][i] & keep;
                if constexpr (SPLIT) *reinterpret_cast<u32x4*>(&sAl[buf][srow + RPT * i][skw]) = rl[slot][i] & keep;
            }
#pragma unroll
        for (int i = 0; i < STB; ++i)
            if (i * NKK / STB == kk) {
                Frag8 fw;
                fw.v4 = rb[slot][i];
                if constexpr (!WF16) bf16x8_to_f16x8(fw);
                *reinterpret_cast<u32x4*>(&sB[buf][srow + RPT * i][skw]) = fw.v4;
            }
    };
    auto multiply_piece = [&](int buf, int kk) {
        Frag8 fa[2], fb[NJ];
        // LDS column of this lane's fragment (every row offset above lr is a multiple of 32)
        const int fc = SWZ ? ((kk * 2 + lg) ^ ((lr >> 2) & 3)) * 8 : kk * 16 + lg * 8;
#pragma unroll
        for (int i = 0; i < 2; ++i)
            fa[i].v4 = *reinterpret_cast<const u32x4*>(&sA[buf][wm * 64 + i * 32 + lr][fc]);
#pragma unroll
        for (int i = 0; i < NJ; ++i)
            fb[i].v4 = *reinterpret_cast<const u32x4*>(&sB[buf][wn * WN + i * 32 + lr][fc]);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int jj = 0; jj < NJ; ++jj) acc[i][jj] = mfma_32x32x16(fa[i], fb[jj], acc[i][jj]);
        if constexpr (SPLIT) {
            Frag8 fl[2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
                fl[i].v4 = *reinterpret_cast<const u32x4*>(&sAl[buf][wm * 64 + i * 32 + lr][fc]);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int jj = 0; jj < NJ; ++jj) acl[i][jj] = mfma_32x32x16(fl[i], fb[jj], acl[i][jj]);
        }
    };
    static_assert(D % 2 == 0, "slot j of the unrolled loop must map to LDS buffer j & 1");
    static_for<0, D>([&](auto sc) { gload(sc, decltype(sc)::value); });
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) stage_piece(std::integral_constant<int, 0>{}, 0, kk, 0xFFFFFFFFu);
    __syncthreads();
    // The whole loop exists twice (live and dead waves) so that neither body contains a branch: with a branch
    // inside, the conversions common to both arms are hoisted in front of it and run before, not between, the
    // matrix instructions.
    // Steps are taken in groups of D (D register slots, two LDS buffers). If the step count is not a multiple
    // of D the last group multiplies steps that do not exist: they are staged as zeros, which only that
    // group's code pays for (the mask costs a vector instruction per staged register).
    auto run = [&](auto dead_c) {
        constexpr bool kDead = decltype(dead_c)::value;
        auto pairs = [&](int kt_begin, int kt_end, auto mask_c) {
            constexpr bool kMask = decltype(mask_c)::value;
            for (int kt0 = kt_begin; kt0 < kt_end; kt0 += D) {
                static_for<0, D>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;      // step kt lives in LDS buffer j & 1; registers slot j are free
                    constexpr int jn = (j + 1) % D;             // slot that holds step kt + 1
                    const int kt = kt0 + j;
                    gload(jc, kt + D);
                    __builtin_amdgcn_sched_barrier(0);
                    const unsigned keep = (!kMask || kt + 1 < nk) ? 0xFFFFFFFFu : 0u;
#pragma unroll
                    for (int kk = 0; kk < NKK; ++kk) {
                        if constexpr (!kDead) multiply_piece(j & 1, kk);
                        stage_piece(std::integral_constant<int, jn>{}, jn & 1, kk, keep);
                    }
                    __syncthreads();
                });
            }
        };
        const int full_end = nk - nk % D;                // whole groups of D steps need no mask
        pairs(0, full_end, std::false_type{});
        if (nk % D) pairs(full_end, nk, std::true_type{});
    };
    if (dead) run(std::true_type{});
    else run(std::false_type{});
    if constexpr (SPLIT) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] += acl[i][j][e] * kLoInv;
    }
    if constexpr (EPI == GEPI_HEAD) {
        // ---- output-head epilogue: the tile goes through LDS in two halves of 64 columns (the staging buffer of the
        // activations is free after the loop's last barrier and holds 128 rows x 65 floats), where thread t owns half a
        // row (row t / 2, 32 of the 64 columns) and folds it into its running statistics; ids ascend per thread.
        static_assert(BN == 128 && !SPLIT, "the head epilogue is written for 128-column single-plane tiles");
        static_assert(sizeof(sA) >= GM_BM * 65 * sizeof(float), "the activation staging buffer must hold half a tile of floats");
        float* sC = reinterpret_cast<float*>(&sA[0][0][0]);
        const int trow = tid >> 1, part = tid & 1;
        const int grow = tm * GM_BM + trow;
        RowStat st;
        st.init();
        const int kt = a.hp.topk;                       // 1..KT
        float thr_v = -INFINITY;                        // the list's kt-th entry: what a value has to beat to enter
        int thr_i = 0x7FFFFFFF;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            if (wn == h) {
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
#pragma unroll
                        for (int e = 0; e < 16; ++e)
                            sC[(wm * 64 + i * 32 + 8 * (e >> 2) + 4 * lg + (e & 3)) * 65 + j * 32 + lr] = acc[i][j][e];
            }
            __syncthreads();
            const int n0 = tn * BN + h * 64 + part * 32;
            const float* src = sC + trow * 65 + part * 32;
            if (grow < a.M) {
                // 32 columns at once, without data-dependent branches on the common path: their maximum and its first
                // position, the sum of exponentials against the new running maximum, and the few values that beat the
                // list's kt-th entry (kt = the call's k: deeper list entries are never needed for "rank < k")
                float vals[32];
#pragma unroll
                for (int c = 0; c < 32; ++c) vals[c] = (n0 + c < a.N) ? src[c] : -INFINITY;
                float mloc = vals[0];
#pragma unroll
                for (int c = 1; c < 32; ++c) mloc = fmaxf(mloc, vals[c]);
                int cloc = 31;
#pragma unroll
                for (int c = 30; c >= 0; --c) cloc = vals[c] == mloc ? c : cloc;
                const float m_new = fmaxf(st.mx, mloc);
                float ssum = 0.f;
                if (m_new != -INFINITY) {
#pragma unroll
                    for (int c = 0; c < 32; ++c) ssum += __expf(vals[c] - m_new);          // exp(-inf) = 0 for columns past N
                    st.sum = st.sum * __expf(st.mx - m_new) + ssum;
                }
                if (mloc > st.mx) st.arg = n0 + cloc;                                      // ids ascend per thread: earlier ties stay
                st.mx = m_new;
                if (hc_x0 >= n0 && hc_x0 < n0 + 32) a.hp.cand_lx[hc_b] = src[hc_x0 - n0];
                for (int c = 1; c < hc_n; ++c) {                                         // further children of a tree node
                    const int x = a.hp.cand_x[hc_b + c];
                    if (x >= n0 && x < n0 + 32) a.hp.cand_lx[hc_b + c] = src[x - n0];
                }
#pragma unroll
                for (int c = 0; c < 32; ++c) {
                    if (n0 + c < a.N && before(vals[c], n0 + c, thr_v, thr_i)) {
                        st.push_top(vals[c], n0 + c);
#pragma unroll
                        for (int j = 0; j < KT; ++j) if (j == kt - 1) { thr_v = st.tv[j]; thr_i = st.ti[j]; }
                    }
                }
                if (a.hp.logits_dbg) {
#pragma unroll
                    for (int c = 0; c < 32; ++c) if (n0 + c < a.N) a.hp.logits_dbg[(size_t)grow * a.N + n0 + c] = vals[c];
                }
            }
            __syncthreads();
        }
        st.merge_from_lane(1);
        if (part == 0 && grow < a.M) st.store(a.hp, grow, tn);
        return;
    }
    // ---- epilogue: lane holds column lr of each 32-wide tile, rows 8 (e / 4) + 4 lg + e % 4 ----
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int row = tm * GM_BM + wm * 64 + i * 32 + 8 * (e >> 2) + 4 * lg + (e & 3);
            if (row >= a.M) continue;
            if (EPI == GEPI_SWIGLU) {
                const int feat = tn * 64 + wn * 32 + lr;
                if (feat < a.N) {
                    const float gt = acc[i][0][e], up = acc[i][NJ - 1][e];
                    a.outh[(size_t)row * a.N + feat] = f32_to_f16(gt / (1.f + __expf(-gt)) * up);
                }
            } else {
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    const int col = tn * BN + wn * WN + j * 32 + lr;
                    if (col < a.N) {
                        float* p = outf + (size_t)row * a.N + col;
                        if (EPI == GEPI_RESID) *p += acc[i][j][e];
                        else *p = acc[i][j][e];
                    }
                }
            }
        }
    }
}

}  // namespace laser
