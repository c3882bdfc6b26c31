// Verify forward of the target model (Sec. 2.1 Eq. 3, Sec. 3.4 Eq. 6): R = K+1 rows per sequence
// against the paged KV cache. Generic kernel set: works for any row count; the shapes it is tuned
// for are the few-row, weight-streaming ones.
#include <cmath>
#include <string>
#include <vector>

#include "gemm_mfma.h"
#include "gemm_skinny.h"
#include "gemm_mid.h"
#include "state.h"

namespace laser {

bool fused_supported(const Model* m, int B, int K, int max_len_ub);
void fused_free(Model* m);
int run_fused(Model* m, KV* kv, const int32_t* ids_dev, const int32_t* pending, const int32_t* drafts, const int32_t* parent,
              const int32_t* draft_len, int B, int K, int topk, float p, int mode, int32_t* accept_len,
              int32_t* out_tokens, int32_t* accept_path, float* logits_dbg, int max_len_ub, hipStream_t stream);
int fused_status(Model* m, hipStream_t stream, int* aborted);
int fused_read_trace(Model* m, hipStream_t stream, long long* out, int max_elems, int* nwg, int* cap);

int run_head(Model* m, const uint16_t* h, const int32_t* tokens, const int32_t* parent, const int32_t* n_nodes, int B, int K,
             int topk, float p, int mode, int32_t* accept_len, int32_t* out_tokens, int32_t* accept_path, float* logits_dbg,
             hipStream_t stream);
int head_chunks_cap(const Model* m);
int run_head_static(Model* m, const uint16_t* h, const int32_t* drafts, const int32_t* draft_len, int B, int K,
                    int topk, float p, int mode, int32_t* accept_len, int32_t* out_tokens, hipStream_t stream);

// ------------------------------------------------------------------------------------------------
__device__ inline float block_sum_256(float v, float* sm /*[4]*/) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm[w] = v;
    __syncthreads();
    return sm[0] + sm[1] + sm[2] + sm[3];
}

// One thread per row: where the row sits. Row r of sequence b holds the pending token (r = 0) or node r - 1 of the
// drafts' pseudo-sequence (Sec. 3.3). Its key/value go to cache slot len + r; its position is len + its depth in the
// token tree (chain: depth = r); it attends to the committed cache and to the rows on its own branch (bit mask).
__global__ void rows_kernel(const int32_t* __restrict__ parent, const int32_t* __restrict__ n_nodes, const int32_t* __restrict__ seq_ids,
                            const int32_t* __restrict__ lens, int B, int R, int32_t* __restrict__ row_pos,
                            int32_t* __restrict__ row_slot, unsigned long long* __restrict__ row_anc) {
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    if (m >= B * R) return;
    const int b = m / R, r = m % R, K = R - 1;
    const int len = lens[seq_ids[b]];
    int nn = n_nodes[b];
    nn = nn < 0 ? 0 : (nn > K ? K : nn);
    unsigned long long anc = 1ull;                 // the pending token's row
    int depth = 0;
    for (int i = r - 1; i >= 0; i = tree_parent_of(parent, b, K, i, nn)) { anc |= 1ull << (i + 1); ++depth; }
    row_pos[m] = len + depth;
    row_slot[m] = len + r;
    row_anc[m] = anc;
}

// One block per row: token lookup, embedding gather, first RMSNorm.
__global__ __launch_bounds__(256) void embed_rmsnorm_kernel(
    const uint16_t* __restrict__ emb, const float* __restrict__ gain, const int32_t* __restrict__ pending,
    const int32_t* __restrict__ drafts, const int32_t* __restrict__ draft_len, int R, int d, int vocab, float eps,
    float* __restrict__ x, uint16_t* __restrict__ xn, uint16_t* __restrict__ xn_lo) {
    __shared__ float sm[4];
    const int m = blockIdx.x, b = m / R, r = m % R, K = R - 1;
    int tok = r == 0 ? pending[b] : ((r - 1) < draft_len[b] ? drafts[(size_t)b * K + r - 1] : 0);
    if (tok < 0 || tok >= vocab) tok = 0;
    const uint16_t* e = emb + (size_t)tok * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += 256) { float v = bf16_to_f32(e[i]); ss += v * v; }
    ss = block_sum_256(ss, sm);
    const float rs = rsqrtf(ss / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += 256) {
        float v = bf16_to_f32(e[i]);
        x[(size_t)m * d + i] = v;
        split_f16(v * rs * gain[i], xn[(size_t)m * d + i], xn_lo[(size_t)m * d + i]);
    }
}

// xn_lo may be NULL (the final norm feeds the output head, which takes single fp16 rows).
// n_part > 0: the projection before this norm left its result as n_part partial sums (part + p * part_stride, same
// [row][d] layout): they are added to the residual row in order p = 0, 1, .. and the row is written back, in the
// same pass that takes the row into registers and sums its squares (every thread touches only its own columns).
// NPART is a template argument (0, 2, 4 or 8) so that the parts' loads are all issued before the first is added: with
// a run-time trip count they were waited for one after the other, a memory round trip each.
template <int NPART>
__global__ __launch_bounds__(256) void rmsnorm_kernel(float* __restrict__ x, const float* __restrict__ gain,
                                                      int d, float eps, uint16_t* __restrict__ xn, uint16_t* __restrict__ xn_lo,
                                                      const float* __restrict__ part, size_t part_stride) {
    __shared__ float sm[4];
    const size_t m = blockIdx.x;
    // the row stays in registers between the two passes (up to 8192 columns; d is a multiple of 128)
    constexpr int NV = 8;
    const int n4 = d / 4;
    float4* xw = reinterpret_cast<float4*>(x + m * d);
    const float4* xr = xw;
    auto take = [&](int i) {                     // column group i of the row, partial sums added and stored back
        float4 t = xr[i];
        if constexpr (NPART > 0) {
            float4 q[NPART];
#pragma unroll
            for (int p = 0; p < NPART; ++p) q[p] = reinterpret_cast<const float4*>(part + p * part_stride + m * d)[i];
#pragma unroll
            for (int p = 0; p < NPART; ++p) { t.x += q[p].x; t.y += q[p].y; t.z += q[p].z; t.w += q[p].w; }
            xw[i] = t;
        }
        return t;
    };
    float4 v[NV];
    float ss = 0.f;
#pragma unroll
    for (int c = 0; c < NV; ++c) {
        const int i = c * 256 + threadIdx.x;
        if (i < n4) {
            v[c] = take(i);
            ss += v[c].x * v[c].x + v[c].y * v[c].y + v[c].z * v[c].z + v[c].w * v[c].w;
        }
    }
    for (int i = NV * 256 + threadIdx.x; i < n4; i += 256) {      // wider rows: re-read below by the same thread
        const float4 t = take(i);
        ss += t.x * t.x + t.y * t.y + t.z * t.z + t.w * t.w;
    }
    ss = block_sum_256(ss, sm);
    const float rs = rsqrtf(ss / (float)d + eps);
    const float4* g4 = reinterpret_cast<const float4*>(gain);
    uint2* out = reinterpret_cast<uint2*>(xn + m * d);
    uint2* out_lo = xn_lo ? reinterpret_cast<uint2*>(xn_lo + m * d) : nullptr;
    auto emit = [&](int i, const float4& t) {
        const float4 g = g4[i];
        Frag4 o, ol;
        split_f16(t.x * rs * g.x, o.h[0], ol.h[0]); split_f16(t.y * rs * g.y, o.h[1], ol.h[1]);
        split_f16(t.z * rs * g.z, o.h[2], ol.h[2]); split_f16(t.w * rs * g.w, o.h[3], ol.h[3]);
        out[i] = o.u;
        if (out_lo) out_lo[i] = ol.u;
    };
#pragma unroll
    for (int c = 0; c < NV; ++c) {
        const int i = c * 256 + threadIdx.x;
        if (i < n4) emit(i, v[c]);
    }
    for (int i = NV * 256 + threadIdx.x; i < n4; i += 256) emit(i, xr[i]);
}

static void launch_rmsnorm(int M, hipStream_t stream, float* x, const float* gain, int d, float eps, uint16_t* xn, uint16_t* xn_lo,
                           const float* part, int n_part, size_t part_stride) {
    switch (n_part) {
        case 0: hipLaunchKernelGGL(rmsnorm_kernel<0>, dim3(M), dim3(256), 0, stream, x, gain, d, eps, xn, xn_lo, part, part_stride); break;
        case 2: hipLaunchKernelGGL(rmsnorm_kernel<2>, dim3(M), dim3(256), 0, stream, x, gain, d, eps, xn, xn_lo, part, part_stride); break;
        case 4: hipLaunchKernelGGL(rmsnorm_kernel<4>, dim3(M), dim3(256), 0, stream, x, gain, d, eps, xn, xn_lo, part, part_stride); break;
        default: hipLaunchKernelGGL(rmsnorm_kernel<8>, dim3(M), dim3(256), 0, stream, x, gain, d, eps, xn, xn_lo, part, part_stride); break;
    }
}

// ------------------------------------------------------------------------------------------------

struct GemmArgs {
    const uint16_t* W;      // [N][Kd]  (EPI_SWIGLU: [2N][Kd], gate rows then up rows)
    const uint16_t* W16;    // the same matrix widened to fp16 (many-row path only), or NULL
    const uint16_t* X;      // [M][Kd]
    const uint16_t* Xlo;    // [M][Kd] low plane of split activations, or NULL
    int M, N, Kd, S;
    float* outf;            // EPI_F32: [M][N] store;  EPI_RESID: [M][N] accumulate
    uint16_t* outh;         // EPI_SWIGLU: [M][N] fp16
    float* part = nullptr;  // many-row path: workspace for reduction-split partial results (store / accumulate epilogues)
    size_t part_floats = 0;
    int want_split = 0;     // 0: choose; 1, 2, 4: force this many reduction parts
    int n_part = 0;         // out: parts left in `part` for the consumer to add up (0: the result is complete)
    int mid_waves = 0;      // 17..80 rows: 0 = choose the waves per workgroup, 4 or 8 = force
};

template <int MB, int EPI, bool SPLIT>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(GemmArgs a) {
    constexpr int NA = EPI == EPI_SWIGLU ? 2 : 1;
    __shared__ float red[4][NA][MB][4][64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int unit = blockIdx.x * 4 + wave;
    const int tile = unit / a.S, ks = unit % a.S;
    const int ntiles = a.N / 16;
    const int row0 = blockIdx.y * MB * 16;
    const bool active = tile < ntiles;
    const int ksteps = a.Kd / kGemmKStep;
    const int per = (ksteps + a.S - 1) / a.S;
    const int kbeg = ks * per * kGemmKStep;
    const int kend = min(a.Kd, kbeg + per * kGemmKStep);

    float4_t acc[NA][MB];
#pragma unroll
    for (int s = 0; s < NA; ++s)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[s][mb] = float4_t{0.f, 0.f, 0.f, 0.f};
    if (active) {
        wave_gemm_tile<MB, SPLIT>(a.W + (size_t)tile * 16 * a.Kd, (size_t)a.Kd, a.X, a.Xlo, a.Kd, a.M, row0, kbeg, kend, acc[0]);
        if (NA == 2)
            wave_gemm_tile<MB, SPLIT>(a.W + ((size_t)a.N + (size_t)tile * 16) * a.Kd, (size_t)a.Kd, a.X, a.Xlo, a.Kd, a.M, row0,
                                      kbeg, kend, acc[NA - 1]);
    }
    if (a.S > 1) {
#pragma unroll
        for (int s = 0; s < NA; ++s)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int i = 0; i < 4; ++i) red[wave][s][mb][i][lane] = acc[s][mb][i];
        __syncthreads();
        if (ks == 0) {
            for (int o = 1; o < a.S; ++o)
#pragma unroll
                for (int s = 0; s < NA; ++s)
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                        for (int i = 0; i < 4; ++i) acc[s][mb][i] += red[wave + o][s][mb][i][lane];
        }
    }
    if (!active || ks != 0) return;
    const int r = lane & 15, g = lane >> 4;
    const int n = tile * 16 + 4 * g;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int row = row0 + mb * 16 + r;
        if (row >= a.M) continue;
        if (EPI == EPI_F32) {
            *reinterpret_cast<float4*>(a.outf + (size_t)row * a.N + n) =
                make_float4(acc[0][mb][0], acc[0][mb][1], acc[0][mb][2], acc[0][mb][3]);
        } else if (EPI == EPI_RESID) {
            float4* p = reinterpret_cast<float4*>(a.outf + (size_t)row * a.N + n);
            float4 v = *p;
            v.x += acc[0][mb][0]; v.y += acc[0][mb][1]; v.z += acc[0][mb][2]; v.w += acc[0][mb][3];
            *p = v;
        } else {
            Frag4 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float gt = acc[0][mb][i], up = acc[NA - 1][mb][i];
                o.h[i] = f32_to_f16(gt / (1.f + __expf(-gt)) * up);
            }
            *reinterpret_cast<uint2*>(a.outh + (size_t)row * a.N + n) = o.u;
        }
    }
}

constexpr int kSkinnyMaxRows = 80;   // beyond this the weights would be streamed more than once

// bf16 -> fp16 copy of a weight matrix, 8 elements per thread and iteration; counts the values whose magnitude fp16
// cannot hold (they would become infinities)
__global__ __launch_bounds__(256) void widen_weights_kernel(const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, size_t n8,
                                                            int* __restrict__ overflow) {
    int bad = 0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
        Frag8 f;
        f.u = reinterpret_cast<const uint4*>(src)[i];
#pragma unroll
        for (int j = 0; j < 8; ++j) bad += (f.h[j] & 0x7FFFu) > 0x477Fu ? 1 : 0;     // |w| > 65280 (bf16 pattern), inf and NaN included
        bf16x8_to_f16x8(f);
        reinterpret_cast<uint4*>(dst)[i] = f.u;
    }
    if (bad) atomicAdd(overflow, bad);
}

// fp16 copies of `n` bf16 matrices for the tiled many-row kernels (made once, at the first call that needs them; that
// call synchronises the stream). All or nothing: on failure nothing is kept. LASER_E_LIMIT if a weight does not fit fp16.
int widen_copies(const uint16_t* const* src, const size_t* elems, int n, uint16_t** dst, hipStream_t stream) {
    uint16_t* cp[4] = {nullptr, nullptr, nullptr, nullptr};
    int* flag = nullptr;
    auto drop = [&] { for (int i = 0; i < n; ++i) if (cp[i]) (void)hipFree(cp[i]); if (flag) (void)hipFree(flag); };
    hipError_t e = hipMalloc((void**)&flag, sizeof(int));
    for (int i = 0; i < n && e == hipSuccess; ++i) e = hipMalloc((void**)&cp[i], elems[i] * 2);
    if (e == hipSuccess) e = hipMemsetAsync(flag, 0, sizeof(int), stream);
    if (e != hipSuccess) {
        drop();
        set_error("allocating the fp16 weight copies failed: %s", hipGetErrorString(e));
        return LASER_E_HIP;
    }
    for (int i = 0; i < n; ++i)
        hipLaunchKernelGGL(widen_weights_kernel, dim3(2048), dim3(256), 0, stream, src[i], cp[i], elems[i] / 8, flag);
    int bad = 0;
    e = hipMemcpyAsync(&bad, flag, sizeof(int), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess || bad) {
        drop();
        if (e != hipSuccess) { set_error("widening the weights to fp16 failed: %s", hipGetErrorString(e)); return LASER_E_HIP; }
        set_error("%d weights exceed the fp16 range (|w| > 65280): set option f16_copies = 0 to stream them as bf16", bad);
        return LASER_E_LIMIT;
    }
    (void)hipFree(flag);
    for (int i = 0; i < n; ++i) dst[i] = cp[i];
    return LASER_OK;
}

// Reduction parts for a tiled launch of `tiles` 128 x 128 tiles. Two workgroups share a CU ("slots" = 2 x CUs) and a
// launch takes ceil(units / slots) rounds; a lone workgroup on a CU runs at about 0.6 of the shared time. Cutting the
// reduction into S parts makes S times as many units of 1/S the length, which evens out tile counts like 576 (2 rounds
// for 1.1 rounds of work) or 192 (most slots empty); each part costs one more pass of the output through memory.
static int choose_ksplit(long tiles, int ksteps, long out_elems, int slots) {
    int best = 1;
    double best_cost = 1e30;
    for (int S = 1; S <= 4; S *= 2) {
        if (ksteps % S || ksteps / S < 8) continue;
        if (S > 2 && out_elems > (4L << 20)) continue;          // large outputs: the extra passes cost more than they save
        const long units = tiles * S;
        const double rounds = units <= slots / 2 ? 0.6 : (double)((units + slots - 1) / slots);
        const double cost = rounds / S + 0.04 * (S - 1);
        if (cost < best_cost - 1e-9) { best_cost = cost; best = S; }
    }
    return best;
}

template <int EPI>
static int launch_gemm(GemmArgs& a_in, hipStream_t stream) {
    GemmArgs& a = a_in;
    a.n_part = 0;
    if (a.M > kSkinnyMaxRows) {
        constexpr int GE = EPI == EPI_F32 ? GEPI_F32 : (EPI == EPI_RESID ? GEPI_RESID : GEPI_SWIGLU);
        const int tiles_m = (a.M + GM_BM - 1) / GM_BM;
        int ncu = 0;
        LASER_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, 0));
        using std::integral_constant;
        if constexpr (EPI != EPI_SWIGLU) {
            // store / accumulate epilogues may split the reduction: partial results go to the workspace and the
            // next kernel (rotary + cache write, or the norm) adds them up in a fixed order
            const int bk = a.Xlo ? 32 : 64;
            const long tiles = (long)tiles_m * ((a.N + 127) / 128);
            int S = a.want_split ? a.want_split : choose_ksplit(tiles, a.Kd / bk, (long)a.M * a.N, 2 * ncu);
            if ((a.Kd / bk) % S || !a.part || (size_t)S * a.M * a.N > a.part_floats) S = 1;
            if (S > 1) {
                GemmTileArgs t{a.W16 ? a.W16 : a.W, a.X, a.Xlo, a.M, a.N, a.Kd, tiles_m, ((a.N + 127) / 128) * S, S, a.part, nullptr};
                dim3 grid(gemm_mfma_grid(t.tiles_m, t.tiles_n));
                auto gos = [&](auto splitc) {
                    if (a.W16)
                        hipLaunchKernelGGL((gemm_mfma_kernel<GEPI_F32, 128, decltype(splitc)::value, true>), grid, dim3(256), 0, stream, t);
                    else
                        hipLaunchKernelGGL((gemm_mfma_kernel<GEPI_F32, 128, decltype(splitc)::value, false>), grid, dim3(256), 0, stream, t);
                };
                if (a.Xlo) gos(integral_constant<bool, true>{});
                else gos(integral_constant<bool, false>{});
                LASER_HIP_CHECK(hipGetLastError());
                a.n_part = S;
                return LASER_OK;
            }
        }
        // narrow outputs: 128-column tiles would leave compute units without work; 64-column tiles double the count
        const bool narrow = EPI != EPI_SWIGLU && (long)tiles_m * ((a.N + 127) / 128) * 4 < (long)ncu * 5;
        const int bn = narrow ? 64 : 128;
        GemmTileArgs t{a.W16 ? a.W16 : a.W, a.X, a.Xlo, a.M, a.N, a.Kd, tiles_m, EPI == EPI_SWIGLU ? (a.N + 63) / 64 : (a.N + bn - 1) / bn, 1, a.outf, a.outh};
        dim3 grid(gemm_mfma_grid(t.tiles_m, t.tiles_n));
        auto go = [&](auto bnc, auto splitc) {
            if (a.W16)
                hipLaunchKernelGGL((gemm_mfma_kernel<GE, decltype(bnc)::value, decltype(splitc)::value, true>), grid, dim3(256), 0, stream, t);
            else
                hipLaunchKernelGGL((gemm_mfma_kernel<GE, decltype(bnc)::value, decltype(splitc)::value, false>), grid, dim3(256), 0, stream, t);
        };
        if constexpr (EPI != EPI_SWIGLU) {
            if (narrow) {
                if (a.Xlo) go(integral_constant<int, 64>{}, integral_constant<bool, true>{});
                else go(integral_constant<int, 64>{}, integral_constant<bool, false>{});
                LASER_HIP_CHECK(hipGetLastError());
                return LASER_OK;
            }
        }
        if (a.Xlo) go(integral_constant<int, 128>{}, integral_constant<bool, true>{});
        else go(integral_constant<int, 128>{}, integral_constant<bool, false>{});
        LASER_HIP_CHECK(hipGetLastError());
        return LASER_OK;
    }
    const int ntiles = a.N / 16;
    const int mblocks = (a.M + 15) / 16;
    if (mblocks >= 2 && (a.Xlo || EPI == EPI_RESID) && a.Kd % kGemmKStep == 0) {
        // 17..80 rows: activations staged in LDS and shared by the workgroup's four weight tiles
        GemmMidArgs t{a.W, a.X, a.Xlo, a.M, a.N, a.Kd, a.outf, a.outh, a.part};
        const GemmMidPlan pl = gemm_mid_plan(a.M, a.N, a.Kd, a.Xlo ? 2 : 1, EPI == EPI_SWIGLU, a.part ? a.part_floats : 0, a.mid_waves);
        if (a.Xlo) launch_gemm_mid<EPI, true>(t, pl, stream);
        else if constexpr (EPI == EPI_RESID) launch_gemm_mid<EPI, false>(t, pl, stream);
        LASER_HIP_CHECK(hipGetLastError());
        a.n_part = pl.S > 1 ? pl.S : 0;
        return LASER_OK;
    }
    const int MB = mblocks >= 5 ? 5 : mblocks;
    const int passes = (mblocks + MB - 1) / MB;
    int S = 1;
    while (S < 4 && (long)ntiles * passes * S < 2048 && (a.Kd / kGemmKStep) >= 2 * S * 2) S *= 2;
    a.S = S;
    dim3 grid((unsigned)((ntiles * S + 3) / 4), (unsigned)passes);
    // the down projection (EPI_RESID without a low plane) is the only unsplit product
    constexpr bool kMaySplit = true, kMayPlain = EPI == EPI_RESID;      // few rows: gate/up and QKV are always split
    auto go = [&](auto mbc) {
        constexpr int mb = decltype(mbc)::value;
        if (a.Xlo) {
            if constexpr (kMaySplit) hipLaunchKernelGGL((gemm_skinny_kernel<mb, EPI, true>), grid, dim3(256), 0, stream, a);
        } else {
            if constexpr (kMayPlain) hipLaunchKernelGGL((gemm_skinny_kernel<mb, EPI, false>), grid, dim3(256), 0, stream, a);
        }
    };
    LASER_REQUIRE(a.Xlo || kMayPlain, LASER_E_INVALID_ARG, "this product needs split activations");
    switch (MB) {
        case 1: go(std::integral_constant<int, 1>{}); break;
        case 2: go(std::integral_constant<int, 2>{}); break;
        case 3: go(std::integral_constant<int, 3>{}); break;
        case 4: go(std::integral_constant<int, 4>{}); break;
        default: go(std::integral_constant<int, 5>{}); break;
    }
    LASER_HIP_CHECK(hipGetLastError());
    return LASER_OK;
}

// ------------------------------------------------------------------------------------------------
// One block per row: rotate q and k, store q (fp16) and the row's k, v into its cache slot.
struct RopeArgs {
    const float* qkv; const int32_t* row_pos; const int32_t* row_slot; const int32_t* seq_ids; const int32_t* block_table;
    const float2* rope; uint16_t* q; uint16_t* q_lo; uint16_t* kpages; uint8_t* klpages; uint16_t* vpages;
    int R, d, H, dh, mpps, layer, n_pages;
    int M, ny, B;          // rows, blocks per row; blocks past M * ny write the values (see below)
    int n_part;            // > 1: qkv holds that many partial results, n_part_stride floats apart, to be added in order
    size_t part_stride;
};

// NPART (1, 2, 4 or 8) is a template argument so that all parts are requested before the first is added.
template <int NPART>
__device__ inline float4 ld4_sum(const float* p, size_t stride) {
    float4 q[NPART];
#pragma unroll
    for (int s = 0; s < NPART; ++s) q[s] = *reinterpret_cast<const float4*>(p + s * stride);
    float4 t = q[0];
#pragma unroll
    for (int s = 1; s < NPART; ++s) { t.x += q[s].x; t.y += q[s].y; t.z += q[s].z; t.w += q[s].w; }
    return t;
}

// Values. The cache keeps them channel-major ([dh][16 tokens] per page and head), so one row's values are 2-byte
// pieces 32 bytes apart: written row by row they cost a partial-sector write each (2.9 M of them at 704 rows).
// Instead a thread owns one (sequence, head, channel): it reads that channel's 32-byte page row, replaces the
// slots of the sequence's R new tokens and writes the row back, so all loads and stores are whole 16-byte pieces
// and a wave covers 2 KiB of contiguous page memory.
template <int NPART>
__device__ inline void write_values(const RopeArgs& a, int blk) {
    const int per_blk = 256 / a.dh;                         // (sequence, head) items per block
    const int item = blk * per_blk + (int)threadIdx.x / a.dh, c = (int)threadIdx.x % a.dh;
    if (item >= a.B * a.H) return;
    const int b = item / a.H, h = item % a.H;
    const int pos0 = a.row_slot[b * a.R];                   // slot of the sequence's first row
    const int32_t* bt = a.block_table + (size_t)a.seq_ids[b] * a.mpps;
    const float* v = a.qkv + (size_t)b * a.R * 3 * a.d + 2 * a.d + (size_t)h * a.dh + c;
    for (int pg = pos0 / kPageSize; pg <= (pos0 + a.R - 1) / kPageSize; ++pg) {
        uint16_t* rowp = a.vpages + ((((size_t)a.layer * a.n_pages + bt[pg]) * a.H + h) * a.dh + c) * kPageSize;
        Frag8 lo, hi;                                       // tokens 0..7 and 8..15 of the page
        lo.u = reinterpret_cast<const uint4*>(rowp)[0];
        hi.u = reinterpret_cast<const uint4*>(rowp)[1];
#pragma unroll
        for (int tp = 0; tp < kPageSize; ++tp) {
            const int r = pg * kPageSize + tp - pos0;
            if (r >= 0 && r < a.R) {
                float vp[NPART];
#pragma unroll
                for (int s = 0; s < NPART; ++s) vp[s] = v[(size_t)r * 3 * a.d + s * a.part_stride];
                float vs = vp[0];
#pragma unroll
                for (int s = 1; s < NPART; ++s) vs += vp[s];
                const uint16_t val = f32_to_f16(vs);
                if (tp < 8) lo.h[tp & 7] = val; else hi.h[tp & 7] = val;
            }
        }
        reinterpret_cast<uint4*>(rowp)[0] = lo.u;
        reinterpret_cast<uint4*>(rowp)[1] = hi.u;
    }
}

template <int NPART>
__global__ __launch_bounds__(256) void rope_kv_kernel(RopeArgs a) {
    if ((int)blockIdx.x >= a.M * a.ny) { write_values<NPART>(a, (int)blockIdx.x - a.M * a.ny); return; }
    const int m = blockIdx.x / a.ny, by = blockIdx.x % a.ny, b = m / a.R;
    const int pos = a.row_pos[m], slot = a.row_slot[m];       // rotary position (depth in the token tree) / cache slot (row order)
    const int pg = a.block_table[(size_t)a.seq_ids[b] * a.mpps + slot / kPageSize], tp = slot % kPageSize;
    const int half = a.dh / 2;                            // a multiple of 4 (dh is 64 or 128)
    const float* row = a.qkv + (size_t)m * 3 * a.d;
    // a thread takes 4 consecutive rotary pairs (i .. i+3, partners at + half) of one head: 16-byte loads, 8-byte stores
    // ny blocks share a row (each takes every ny-th group of 1024 rotary pairs)
    for (int idx = (by * 256 + threadIdx.x) * 4; idx < a.d / 2; idx += a.ny * 256 * 4) {
        const int h = idx / half, i = idx % half;
        const int c0 = h * a.dh + i, c1 = c0 + half;
        const float4 csa = *reinterpret_cast<const float4*>(a.rope + (size_t)pos * half + i);       // (cos, sin) x 2
        const float4 csb = *reinterpret_cast<const float4*>(a.rope + (size_t)pos * half + i + 2);
        const float4 qa = ld4_sum<NPART>(row + c0, a.part_stride), qb = ld4_sum<NPART>(row + c1, a.part_stride);
        const float4 ka = ld4_sum<NPART>(row + a.d + c0, a.part_stride), kb = ld4_sum<NPART>(row + a.d + c1, a.part_stride);
        const float co[4] = {csa.x, csa.z, csb.x, csb.z}, si[4] = {csa.y, csa.w, csb.y, csb.w};
        const float q0[4] = {qa.x, qa.y, qa.z, qa.w}, q1[4] = {qb.x, qb.y, qb.z, qb.w};
        const float k0[4] = {ka.x, ka.y, ka.z, ka.w}, k1[4] = {kb.x, kb.y, kb.z, kb.w};
        Frag4 oq0, oq1, ok0, ok1, lq0, lq1, lk0, lk1;     // queries and keys are split (hi, lo planes)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            split_f16(q0[j] * co[j] - q1[j] * si[j], oq0.h[j], lq0.h[j]);
            split_f16(q0[j] * si[j] + q1[j] * co[j], oq1.h[j], lq1.h[j]);
            split_f16(k0[j] * co[j] - k1[j] * si[j], ok0.h[j], lk0.h[j]);
            split_f16(k0[j] * si[j] + k1[j] * co[j], ok1.h[j], lk1.h[j]);
        }
        *reinterpret_cast<uint2*>(a.q + (size_t)m * a.d + c0) = oq0.u;
        *reinterpret_cast<uint2*>(a.q + (size_t)m * a.d + c1) = oq1.u;
        *reinterpret_cast<uint2*>(a.q_lo + (size_t)m * a.d + c0) = lq0.u;
        *reinterpret_cast<uint2*>(a.q_lo + (size_t)m * a.d + c1) = lq1.u;
        const size_t base = (((size_t)a.layer * a.n_pages + pg) * a.H + h) * kPageSize * a.dh;
        *reinterpret_cast<uint2*>(a.kpages + base + (size_t)tp * a.dh + i) = ok0.u;
        *reinterpret_cast<uint2*>(a.kpages + base + (size_t)tp * a.dh + i + half) = ok1.u;
        // the keys' low plane is kept in 8 bits
        *reinterpret_cast<uint32_t*>(a.klpages + base + (size_t)tp * a.dh + i) =
            f16_to_b8(lk0.h[0]) | (f16_to_b8(lk0.h[1]) << 8) | (f16_to_b8(lk0.h[2]) << 16) | (f16_to_b8(lk0.h[3]) << 24);
        *reinterpret_cast<uint32_t*>(a.klpages + base + (size_t)tp * a.dh + i + half) =
            f16_to_b8(lk1.h[0]) | (f16_to_b8(lk1.h[1]) << 8) | (f16_to_b8(lk1.h[2]) << 16) | (f16_to_b8(lk1.h[3]) << 24);
    }
}

// ------------------------------------------------------------------------------------------------
// Attention of the R new rows of one (sequence, head) over cache + new slots, one 16-token page per
// wave step, online softmax, optional split over the context (partials merged by attn_combine).
struct AttnArgs {
    const uint16_t* q; const uint16_t* q_lo; const uint16_t* kpages; const uint8_t* klpages; const uint16_t* vpages;
    const int32_t* seq_ids; const int32_t* lens; const int32_t* block_table;
    const unsigned long long* row_anc;     // per row: the rows of its sequence it attends to (itself and its ancestors)
    uint16_t* out; uint16_t* out_lo; float* part;
    int R, d, H, mpps, layer, n_pages, nsplit, nqt;
    int split_pages;       // pages per context split (kSplitPages, or "all" when the launch is not split)
    float scale;
};

constexpr int kSplitPages = 16;   // pages (of 16 tokens) per context split

// NWV = waves per workgroup that share a context's pages (4, or 8 for unsplit launches of few workgroups: half
// the pages per wave; waves 4..7 hand their partial results to waves 0..3 before the four-way merge).
template <int DH, int NWV>
__global__ __launch_bounds__(NWV * 64, NWV == 4 ? 4 : 2) void attn_kernel(AttnArgs a) {
    constexpr int NC32 = DH / 32, NC16 = DH / 16;
    __shared__ float sm_m[4][16], sm_l[4][16];
    __shared__ float sm_o[4][16][DH];
    const int h = blockIdx.x, b = blockIdx.y;
    const int split = blockIdx.z % a.nsplit, qt = blockIdx.z / a.nsplit;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 15, g = lane >> 4;
    const int slot = a.seq_ids[b];
    const int len = a.lens[slot];
    const int qrow = qt * 16 + r;                       // this lane's query row in the S^T layout
    const int rows_here = min(a.R - qt * 16, 16);
    const int last_tok = len + qt * 16 + rows_here - 1;  // last slot any row of this tile may see
    const int npages = last_tok / kPageSize + 1;
    // A split is always kSplitPages pages at fixed positions and its pages go round-robin over the waves, so within
    // one launch shape (same split policy and waves per workgroup) the order in which a row's scores are reduced
    // depends on the row's position only, not on the draft count or the host's length bound: verifying a token as
    // a draft reproduces its one-at-a-time logits bit for bit. Launch shapes that take the context unsplit, or
    // with eight waves, reduce in a different order and may differ from the split form in the last bits.
    const int p0 = split * a.split_pages, p1 = min(npages, p0 + a.split_pages);

    const unsigned long long anc = a.row_anc[(size_t)b * a.R + min(qrow, a.R - 1)];
    Frag8 bq[NC32], bql[NC32];
    {
        const int rowc = min(qrow, a.R - 1);
        const size_t qo = ((size_t)b * a.R + rowc) * a.d + (size_t)h * DH + g * 8;
#pragma unroll
        for (int c = 0; c < NC32; ++c) bq[c].u = *reinterpret_cast<const uint4*>(a.q + qo + c * 32);
#pragma unroll
        for (int c = 0; c < NC32; ++c) bql[c].u = *reinterpret_cast<const uint4*>(a.q_lo + qo + c * 32);
    }
    float m_run = -INFINITY, l_run = 0.f;
    float4_t acc[NC16];
#pragma unroll
    for (int c = 0; c < NC16; ++c) acc[c] = float4_t{0.f, 0.f, 0.f, 0.f};
    const int32_t* bt = a.block_table + (size_t)slot * a.mpps;

    // Pages p0 + wave, + NWV, ..: the K and V fragments of the next page are requested before the current
    // one is multiplied (unconditionally: past the wave's last page the current page is requested again,
    // a cache hit), so a wave always has one page in flight.
    auto load_page = [&](int p, Frag8 (&ak)[NC32], u32x2 (&akl)[NC32], Frag4 (&bv)[NC16]) {
        const int pg = bt[p];
        const size_t base = (((size_t)a.layer * a.n_pages + pg) * a.H + h) * kPageSize * DH;
        const uint16_t* kp = a.kpages + base + (size_t)r * DH + g * 8;
        const uint8_t* klp = a.klpages + base + (size_t)r * DH + g * 8;
#pragma unroll
        for (int c = 0; c < NC32; ++c) ak[c].v4 = *reinterpret_cast<const u32x4*>(kp + c * 32);
#pragma unroll
        for (int c = 0; c < NC32; ++c) akl[c] = *reinterpret_cast<const u32x2*>(klp + c * 32);
        const uint16_t* vp = a.vpages + base + (size_t)r * kPageSize + 4 * g;
#pragma unroll
        for (int c = 0; c < NC16; ++c) bv[c].v2 = *reinterpret_cast<const u32x2*>(vp + (size_t)c * 16 * kPageSize);
    };
    Frag8 ak[NC32], akn[NC32];
    u32x2 akl[NC32], akln[NC32];        // 8-bit low plane of the keys, widened right before use
    Frag4 bv[NC16], bvn[NC16];
    int p = p0 + wave;
    if (p < p1) load_page(p, ak, akl, bv);
    for (; p < p1; p += NWV) {
        load_page(p + NWV < p1 ? p + NWV : p, akn, akln, bvn);
        // s[i] = K[tok 4g+i] . Q[row r] with both operands split: hi.hi + 2^-12 (hi.lo + lo.hi)
        float4_t s = float4_t{0.f, 0.f, 0.f, 0.f}, sl = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < NC32; ++c) s = mfma_16x16x32(ak[c], bq[c], s);
#pragma unroll
        for (int c = 0; c < NC32; ++c) sl = mfma_16x16x32(ak[c], bql[c], sl);
#pragma unroll
        for (int c = 0; c < NC32; ++c) {
            Frag8 kl;
            b8x8_to_f16x8(akl[c][0], akl[c][1], kl);
            sl = mfma_16x16x32(kl, bq[c], sl);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) s[i] += sl[i] * kLoInv;
        float sv[4], mx = -INFINITY;
        // Committed slots are visible to every row; a new slot (row t - len of this step) only along the row's branch.
        // Branch-free (a branch here would make the wait for the prefetched page conservative): the lane's four slots
        // start rel = t0 - len behind the committed length; rel <= -4: all committed; rel >= 0: four bits of the mask.
        {
            const int rel = p * kPageSize + 4 * g - len;
            const unsigned lo = (unsigned)(anc >> min(max(rel, 0), 63));
            const int sn = min(max(-rel, 0), 4);
            const unsigned hi = ((unsigned)anc << sn) | ((1u << sn) - 1u);
            const unsigned vis4 = (qrow < a.R) ? (rel >= 0 ? lo : hi) : 0u;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                sv[i] = ((vis4 >> i) & 1u) ? s[i] * a.scale : -INFINITY;
                mx = fmaxf(mx, sv[i]);
            }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = (m_new == -INFINITY) ? 1.f : __expf(m_run - m_new);   // m_run = -inf -> 0
        Frag4 pa;
        float rs = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float pv = (sv[i] == -INFINITY) ? 0.f : __expf(sv[i] - m_new);
            rs += pv;
            pa.h[i] = f32_to_f16(pv);
        }
        rs += __shfl_xor(rs, 16);
        rs += __shfl_xor(rs, 32);
        l_run = l_run * alpha + rs;
        m_run = m_new;
        float al[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) al[i] = __shfl(alpha, 4 * g + i);     // accumulator rows are q = 4g+i
#pragma unroll
        for (int c = 0; c < NC16; ++c) {
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[c][i] *= al[i];
            acc[c] = mfma_16x16x16(pa, bv[c], acc[c]);  // acc[c][i] = O[q 4g+i][channel 16c + r]
        }
#pragma unroll
        for (int c = 0; c < NC32; ++c) { ak[c] = akn[c]; akl[c] = akln[c]; }
#pragma unroll
        for (int c = 0; c < NC16; ++c) bv[c] = bvn[c];
    }
    if constexpr (NWV == 8) {
        // ---- waves 4..7 hand over to waves 0..3 (same lane layout on both sides) ----
        if (wave >= 4) {
            if (g == 0) { sm_m[wave - 4][r] = m_run; sm_l[wave - 4][r] = l_run; }
#pragma unroll
            for (int c = 0; c < NC16; ++c)
#pragma unroll
                for (int i = 0; i < 4; ++i) sm_o[wave - 4][4 * g + i][c * 16 + r] = acc[c][i];
        }
        __syncthreads();
        if (wave < 4) {
            const float pm = sm_m[wave][r], pl = sm_l[wave][r];
            const float m_new = fmaxf(m_run, pm);
            const float f = (m_run == -INFINITY) ? 0.f : __expf(m_run - m_new);
            const float fp = (pm == -INFINITY) ? 0.f : __expf(pm - m_new);
            l_run = l_run * f + pl * fp;
            m_run = m_new;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float fi = __shfl(f, 4 * g + i), fpi = __shfl(fp, 4 * g + i);     // accumulator rows are q = 4g+i
#pragma unroll
                for (int c = 0; c < NC16; ++c) acc[c][i] = acc[c][i] * fi + sm_o[wave][4 * g + i][c * 16 + r] * fpi;
            }
        }
        __syncthreads();               // waves 0..3 have read what they now overwrite
    }
    // ---- merge the four waves (all threads of the workgroup share the final pass) ----
    if (NWV == 4 || wave < 4) {
        if (g == 0) { sm_m[wave][r] = m_run; sm_l[wave][r] = l_run; }
#pragma unroll
        for (int c = 0; c < NC16; ++c)
#pragma unroll
            for (int i = 0; i < 4; ++i) sm_o[wave][4 * g + i][c * 16 + r] = acc[c][i];
    }
    __syncthreads();
    float* part = a.part + ((((size_t)b * a.H + h) * a.nqt + qt) * a.nsplit + split) * (32 + 16 * DH);
    for (int idx = threadIdx.x; idx < 16 * DH; idx += NWV * 64) {
        const int q = idx / DH, c = idx % DH;
        float M = fmaxf(fmaxf(sm_m[0][q], sm_m[1][q]), fmaxf(sm_m[2][q], sm_m[3][q]));
        float L = 0.f, O = 0.f;
        if (M != -INFINITY) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float f = __expf(sm_m[w][q] - M);
                L += sm_l[w][q] * f;
                O += sm_o[w][q][c] * f;
            }
        }
        if (a.nsplit == 1) {
            const int row = qt * 16 + q;
            if (row < a.R) {
                const size_t o = ((size_t)b * a.R + row) * a.d + (size_t)h * DH + c;
                split_f16(L > 0.f ? O / L : 0.f, a.out[o], a.out_lo[o]);
            }
        } else {
            if (c == 0) { part[q] = M; part[16 + q] = L; }
            part[32 + idx] = O;
        }
    }
}

template <int DH>
__global__ __launch_bounds__(256) void attn_combine_kernel(AttnArgs a) {
    const int h = blockIdx.x, b = blockIdx.y / a.nqt, qt = blockIdx.y % a.nqt;
    const float* part = a.part + (((size_t)b * a.H + h) * a.nqt + qt) * a.nsplit * (32 + 16 * DH);
    for (int idx = threadIdx.x; idx < 16 * DH; idx += 256) {
        const int q = idx / DH, c = idx % DH;
        const int row = qt * 16 + q;
        if (row >= a.R) continue;
        float M = -INFINITY;
        for (int s = 0; s < a.nsplit; ++s) M = fmaxf(M, part[(size_t)s * (32 + 16 * DH) + q]);
        float L = 0.f, O = 0.f;
        if (M != -INFINITY)
            for (int s = 0; s < a.nsplit; ++s) {
                const float* ps = part + (size_t)s * (32 + 16 * DH);
                const float f = __expf(ps[q] - M);
                L += ps[16 + q] * f;
                O += ps[32 + idx] * f;
            }
        const size_t o = ((size_t)b * a.R + row) * a.d + (size_t)h * DH + c;
        split_f16(L > 0.f ? O / L : 0.f, a.out[o], a.out_lo[o]);
    }
}

__global__ void rope_table_kernel(float2* tab, int max_pos, int half, int dh, double base) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)max_pos * half) return;
    const int pos = (int)(i / half), j = (int)(i % half);
    const double ang = (double)pos * pow(base, -2.0 * (double)j / (double)dh);
    tab[i] = make_float2((float)cos(ang), (float)sin(ang));
}

// ------------------------------------------------------------------------------------------------
// parent: NULL for a chain of drafts, else the token tree's parent array (see tree_parent_of)
static int forward(Model* m, KV* kv, const int32_t* ids_dev, const int32_t* pending, const int32_t* drafts,
                   const int32_t* parent, const int32_t* draft_len, int B, int K, int max_len_ub, hipStream_t stream) {
    const laser_model_desc& d = m->d;
    const int R = K + 1, M = B * R, dm = d.d_model, F = d.ffn;
    hipLaunchKernelGGL(rows_kernel, dim3((M + 255) / 256), dim3(256), 0, stream, parent, draft_len, ids_dev, kv->len, B, R,
                       m->row_pos, m->row_slot, m->row_anc);
    hipLaunchKernelGGL(embed_rmsnorm_kernel, dim3(M), dim3(256), 0, stream, d.emb, d.g1, pending, drafts, draft_len,
                       R, dm, d.vocab, d.eps, m->x, m->xn, m->xn_lo);
    if (M > kSkinnyMaxRows && m->f16_copies && !m->w16[0]) {
        // first many-row step: widen the four projection matrices to fp16 once (same rounding as the kernels' own)
        const size_t n[4] = {(size_t)d.n_layers * 3 * dm * dm, (size_t)d.n_layers * dm * dm, (size_t)d.n_layers * 2 * F * dm,
                             (size_t)d.n_layers * dm * F};
        const uint16_t* src[4] = {d.wqkv, d.wo, d.wgu, d.wdown};
        const int rc = widen_copies(src, n, 4, m->w16, stream);
        if (rc) return rc;
    }
    if (M > 16 && !m->kpart) {
        // workspace for reduction-split partial results: up to 8 parts of [max_rows][d] or 2 of [max_rows][3 d]
        m->kpart_floats = (size_t)d.max_rows * dm * 8;
        LASER_HIP_CHECK(hipMalloc((void**)&m->kpart, m->kpart_floats * 4));
    }
    int pend = 0;              // partial results of the last down projection still to be added to the residual
    const int nqt = (R + 15) / 16;
    const int npages_ub = (max_len_ub + R + kPageSize - 1) / kPageSize;
    // With a (sequence, head, query tile) triple for every second compute unit the context is not split: no
    // partials, no combine kernel; the four waves of a workgroup still share a context's pages. Measured: 128 triples
    // (1B shape, 8 sequences, context 512) 2.02 -> 1.99 ms per step unsplit, 256 triples (7B, 8 sequences, context
    // 1024) 8.17 -> 7.71 ms, 32 triples (7B, one sequence) slower unsplit. Option "attn_whole_min" moves the threshold. (The split policy is a function of the launch shape only, so steps
    // of one shape stay bit-identical to each other; different batch sizes may differ in the last bits.)
    int ncu = 0;
    LASER_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, 0));
    const bool whole = (long)B * d.n_heads * nqt >= (long)(m->attn_whole_min > 0 ? m->attn_whole_min : ncu / 2);
    const int split_pages = whole ? (1 << 20) : kSplitPages;
    const int nsplit = whole ? 1 : std::max(1, (npages_ub + kSplitPages - 1) / kSplitPages);
    const size_t part_need = (size_t)B * d.n_heads * nqt * nsplit * (32 + 16 * m->dh);
    if (nsplit > 1 && part_need > m->att_part_floats) {
        if (m->att_part) LASER_HIP_CHECK(hipFree(m->att_part));
        m->att_part = nullptr;
        LASER_HIP_CHECK(hipMalloc((void**)&m->att_part, part_need * 4));
        m->att_part_floats = part_need;
    }
    for (int l = 0; l < d.n_layers; ++l) {
        int rc;
        if (l > 0)
            launch_rmsnorm(M, stream, m->x, d.g1 + (size_t)l * dm, dm, d.eps, m->xn, m->xn_lo, (const float*)m->kpart, pend, (size_t)M * dm);
        pend = 0;
        const bool many = M > kSkinnyMaxRows && m->w16[0];      // tiled path: weights from the fp16 copy (if kept)
        GemmArgs g{d.wqkv + (size_t)l * 3 * dm * dm, many ? m->w16[0] + (size_t)l * 3 * dm * dm : nullptr, m->xn, m->xn_lo, M, 3 * dm, dm, 1, m->qkv, nullptr};
        g.part = m->kpart; g.part_floats = m->kpart_floats; g.want_split = m->ksplit_opt[0]; g.mid_waves = m->mid_waves;
        if ((rc = launch_gemm<EPI_F32>(g, stream))) return rc;
        RopeArgs ra{g.n_part ? m->kpart : m->qkv, m->row_pos, m->row_slot, ids_dev, kv->block_table, m->rope, m->q, m->q_lo, kv->kpages, kv->klpages, kv->vpages,
                    R, dm, d.n_heads, m->dh, kv->d.max_pages_per_seq, l, kv->d.n_pages,
                    M, std::max(1, std::min(4, dm / 2048)), B, std::max(1, g.n_part), (size_t)M * 3 * dm};
        const int v_blocks = (B * d.n_heads + 256 / m->dh - 1) / (256 / m->dh);
        const dim3 rg((unsigned)(M * ra.ny + v_blocks));
        switch (ra.n_part) {
            case 1: hipLaunchKernelGGL(rope_kv_kernel<1>, rg, dim3(256), 0, stream, ra); break;
            case 2: hipLaunchKernelGGL(rope_kv_kernel<2>, rg, dim3(256), 0, stream, ra); break;
            case 4: hipLaunchKernelGGL(rope_kv_kernel<4>, rg, dim3(256), 0, stream, ra); break;
            default: hipLaunchKernelGGL(rope_kv_kernel<8>, rg, dim3(256), 0, stream, ra); break;
        }
        AttnArgs aa{m->q, m->q_lo, kv->kpages, kv->klpages, kv->vpages, ids_dev, kv->len, kv->block_table, m->row_anc, m->attn, m->attn_lo, m->att_part,
                    R, dm, d.n_heads, kv->d.max_pages_per_seq, l, kv->d.n_pages, nsplit, nqt, split_pages, 1.0f / sqrtf((float)m->dh)};
        dim3 ag(d.n_heads, B, nsplit * nqt);
        // unsplit contexts: eight waves share the pages of a (sequence, head) up to 16 workgroups per compute unit (compared
        // inside one run: 128 and 256 workgroups 3-6 % of the step faster than with four waves, 2048 workgroups 0.3-0.6 %,
        // which is at the edge of that workload's repeatability)
        const bool wide = whole && (m->attn_waves ? m->attn_waves == 8 : (long)B * d.n_heads * nqt < 16L * ncu);
        if (m->dh == 128) {
            if (wide) hipLaunchKernelGGL((attn_kernel<128, 8>), ag, dim3(512), 0, stream, aa);
            else hipLaunchKernelGGL((attn_kernel<128, 4>), ag, dim3(256), 0, stream, aa);
        } else {
            if (wide) hipLaunchKernelGGL((attn_kernel<64, 8>), ag, dim3(512), 0, stream, aa);
            else hipLaunchKernelGGL((attn_kernel<64, 4>), ag, dim3(256), 0, stream, aa);
        }
        if (nsplit > 1) {
            dim3 cg(d.n_heads, B * nqt);
            if (m->dh == 128) hipLaunchKernelGGL(attn_combine_kernel<128>, cg, dim3(256), 0, stream, aa);
            else hipLaunchKernelGGL(attn_combine_kernel<64>, cg, dim3(256), 0, stream, aa);
        }
        GemmArgs go{d.wo + (size_t)l * dm * dm, many ? m->w16[1] + (size_t)l * dm * dm : nullptr, m->attn, m->attn_lo, M, dm, dm, 1, m->x, nullptr};
        go.part = m->kpart; go.part_floats = m->kpart_floats; go.want_split = m->ksplit_opt[1]; go.mid_waves = m->mid_waves;
        if ((rc = launch_gemm<EPI_RESID>(go, stream))) return rc;
        launch_rmsnorm(M, stream, m->x, d.g2 + (size_t)l * dm, dm, d.eps, m->xn, m->xn_lo, (const float*)m->kpart, go.n_part, (size_t)M * dm);
        // On the tiled many-row path a split operand doubles the matrix work; gate/up (45 % of the layer's
        // flops) takes the single fp16 rows there unless option "split_ffn" asks for the split (see set_option).
        const bool split_gu = M <= kSkinnyMaxRows || m->split_ffn;
        GemmArgs gg{d.wgu + (size_t)l * 2 * F * dm, many ? m->w16[2] + (size_t)l * 2 * F * dm : nullptr, m->xn, split_gu ? m->xn_lo : nullptr, M, F, dm, 1, nullptr, m->act};
        gg.mid_waves = m->mid_waves;
        const bool prof = m->prof_on && m->prof_n < m->prof_cap;
        if (prof) LASER_HIP_CHECK(hipEventRecord(m->prof_ev[2 * m->prof_n], stream));
        if ((rc = launch_gemm<EPI_SWIGLU>(gg, stream))) return rc;
        if (prof) { LASER_HIP_CHECK(hipEventRecord(m->prof_ev[2 * m->prof_n + 1], stream)); ++m->prof_n; }
        GemmArgs gd{d.wdown + (size_t)l * dm * F, many ? m->w16[3] + (size_t)l * dm * F : nullptr, m->act, nullptr, M, dm, F, 1, m->x, nullptr};
        gd.part = m->kpart; gd.part_floats = m->kpart_floats; gd.want_split = m->ksplit_opt[2]; gd.mid_waves = m->mid_waves;
        if ((rc = launch_gemm<EPI_RESID>(gd, stream))) return rc;
        pend = gd.n_part;        // added to the residual by the next norm (next layer's, or the final one)
    }
    launch_rmsnorm(M, stream, m->x, d.gf, dm, d.eps, m->xn, nullptr, (const float*)m->kpart, pend, (size_t)M * dm);
    LASER_HIP_CHECK(hipGetLastError());
    return LASER_OK;
}

}  // namespace laser

using namespace laser;

extern "C" int laser_model_destroy(laser_model* h) {
    if (!h) return LASER_OK;
    Model* m = reinterpret_cast<Model*>(h);
    void* ptrs[] = {m->kpart, m->wlm16, m->w16[0], m->w16[1], m->w16[2], m->w16[3], m->x, m->xn, m->xn_lo, m->q_lo, m->attn_lo, m->qkv, m->q, m->attn, m->act, m->row_pos, m->att_part, m->rope, m->hp_max,
                    m->hp_sum, m->hp_arg, m->hp_topv, m->hp_topi, m->cand_beg, m->cand_cnt, m->cand_x, m->node_cand, m->cand_lx, m->row_slot, m->row_anc,
                    m->row_mx, m->row_sum, m->row_arg, m->cand_rank};
    for (void* p : ptrs) if (p) (void)hipFree(p);
    for (hipEvent_t e : m->prof_ev) (void)hipEventDestroy(e);
    fused_free(m);
    delete m;
    return LASER_OK;
}

extern "C" int laser_model_create(const laser_model_desc* desc, void* stream_, laser_model** out) {
    LASER_REQUIRE(desc && out, LASER_E_INVALID_ARG, "NULL argument");
    const laser_model_desc& d = *desc;
    hipStream_t stream = (hipStream_t)stream_;
    LASER_REQUIRE(d.n_layers >= 0 && d.d_model > 0 && d.n_heads > 0 && d.vocab > 0 && d.max_rows > 0 && d.max_batch > 0,
                  LASER_E_INVALID_ARG, "non-positive size in laser_model_desc");
    LASER_REQUIRE(d.d_model % d.n_heads == 0, LASER_E_SHAPE, "d_model not divisible by n_heads");
    const int dh = d.d_model / d.n_heads;
    LASER_REQUIRE(dh == 64 || dh == 128, LASER_E_SHAPE, "head_dim %d unsupported (64 or 128)", dh);
    LASER_REQUIRE(d.d_model % 128 == 0 && d.vocab % 16 == 0, LASER_E_SHAPE, "d_model must be a multiple of 128, vocab of 16");
    LASER_REQUIRE(d.wlm != nullptr, LASER_E_INVALID_ARG, "wlm is NULL");
    if (d.n_layers > 0) {
        LASER_REQUIRE(d.ffn > 0 && d.ffn % 128 == 0, LASER_E_SHAPE, "ffn must be a positive multiple of 128");
        LASER_REQUIRE(d.max_pos > 0, LASER_E_INVALID_ARG, "max_pos must be positive");
        LASER_REQUIRE(d.wqkv && d.wo && d.wgu && d.wdown && d.g1 && d.g2 && d.emb && d.gf, LASER_E_INVALID_ARG, "NULL weight pointer");
    }
    Model* m = new Model();
    m->d = d;
    m->dh = dh;
    auto fail = [&](int rc) { laser_model_destroy(reinterpret_cast<laser_model*>(m)); return rc; };
#define M_TRY(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) { set_error("%s: %s", #expr, hipGetErrorString(e_)); return fail(LASER_E_HIP); } } while (0)
    const size_t R = (size_t)d.max_rows, dm = (size_t)d.d_model;
    M_TRY(hipMalloc((void**)&m->xn, R * dm * 2));
    M_TRY(hipMalloc((void**)&m->cand_beg, R * 4));
    M_TRY(hipMalloc((void**)&m->cand_cnt, R * 4));
    M_TRY(hipMalloc((void**)&m->cand_x, R * 4));
    M_TRY(hipMalloc((void**)&m->node_cand, R * 4));
    M_TRY(hipMalloc((void**)&m->cand_lx, R * 4));
    M_TRY(hipMalloc((void**)&m->row_mx, R * 4));
    M_TRY(hipMalloc((void**)&m->row_sum, R * 4));
    M_TRY(hipMalloc((void**)&m->row_arg, R * 4));
    M_TRY(hipMalloc((void**)&m->cand_rank, R * 4));
    if (d.n_layers > 0) {
        M_TRY(hipMalloc((void**)&m->x, R * dm * 4));
        M_TRY(hipMalloc((void**)&m->qkv, R * dm * 3 * 4));
        M_TRY(hipMalloc((void**)&m->q, R * dm * 2));
        M_TRY(hipMalloc((void**)&m->attn, R * dm * 2));
        M_TRY(hipMalloc((void**)&m->xn_lo, R * dm * 2));
        M_TRY(hipMalloc((void**)&m->q_lo, R * dm * 2));
        M_TRY(hipMalloc((void**)&m->attn_lo, R * dm * 2));
        M_TRY(hipMalloc((void**)&m->act, R * (size_t)d.ffn * 2));
        M_TRY(hipMalloc((void**)&m->row_pos, R * 4));
        M_TRY(hipMalloc((void**)&m->row_slot, R * 4));
        M_TRY(hipMalloc((void**)&m->row_anc, R * 8));
        const size_t nt = (size_t)d.max_pos * (dh / 2);
        M_TRY(hipMalloc((void**)&m->rope, nt * sizeof(float2)));
        hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((nt + 255) / 256)), dim3(256), 0, stream, m->rope,
                           d.max_pos, dh / 2, dh, (double)d.rope_base);
    }
    // output-head partials: one per (row, vocabulary chunk)
    {
        const int ntiles = d.vocab / 16;
        const int tpw = (ntiles + 1023) / 1024;
        m->head_chunks = (ntiles + tpw - 1) / tpw;
        const size_t n = R * (size_t)head_chunks_cap(m);      // the most records per row any row count produces
        M_TRY(hipMalloc((void**)&m->hp_max, n * 4));
        M_TRY(hipMalloc((void**)&m->hp_sum, n * 4));
        M_TRY(hipMalloc((void**)&m->hp_arg, n * 4));
        M_TRY(hipMalloc((void**)&m->hp_topv, n * LASER_MAX_TOPK * 4));
        M_TRY(hipMalloc((void**)&m->hp_topi, n * LASER_MAX_TOPK * 4));
    }
    M_TRY(hipStreamSynchronize(stream));
#undef M_TRY
    *out = reinterpret_cast<laser_model*>(m);
    return LASER_OK;
}

static int check_step_args(const Model* m, int B, int K, int topk, int mode, const void* draft_len,
                           const void* drafts, const void* accept_len, const void* out_tokens) {
    LASER_REQUIRE(m != nullptr, LASER_E_INVALID_ARG, "model is NULL");
    LASER_REQUIRE(B >= 0 && B <= m->d.max_batch, LASER_E_INVALID_ARG, "B %d outside 0..max_batch %d", B, m->d.max_batch);
    LASER_REQUIRE(K >= 0 && K <= LASER_MAX_DRAFT, LASER_E_INVALID_ARG, "K %d outside 0..%d", K, LASER_MAX_DRAFT);
    LASER_REQUIRE((long)B * (K + 1) <= m->d.max_rows, LASER_E_LIMIT, "B*(K+1) = %ld exceeds max_rows %d", (long)B * (K + 1), m->d.max_rows);
    LASER_REQUIRE(topk >= 1 && topk <= LASER_MAX_TOPK, LASER_E_INVALID_ARG, "topk %d outside 1..%d", topk, LASER_MAX_TOPK);
    LASER_REQUIRE(mode >= 0 && mode <= 3, LASER_E_INVALID_ARG, "unknown mode %d", mode);
    LASER_REQUIRE(B == 0 || (draft_len && accept_len && out_tokens && (drafts || K == 0)), LASER_E_INVALID_ARG, "NULL device buffer");
    return LASER_OK;
}

// laser_verify_step (parent == NULL: a chain) and laser_verify_tree; both take the persistent kernel where it applies
static int verify_impl(laser_model* mh, laser_kv* kh, const int32_t* seq_ids, const int32_t* pending, const int32_t* drafts,
                       const int32_t* parent, const int32_t* draft_len, int B, int K, int topk, float p, int mode,
                       int32_t* accept_len, int32_t* out_tokens, int32_t* accept_path, float* logits_dbg, void* stream_) {
    Model* m = reinterpret_cast<Model*>(mh);
    KV* kv = reinterpret_cast<KV*>(kh);
    hipStream_t stream = (hipStream_t)stream_;
    int rc = check_step_args(m, B, K, topk, mode, draft_len, drafts, accept_len, out_tokens);
    if (rc) return rc;
    LASER_REQUIRE(kv != nullptr, LASER_E_INVALID_ARG, "kv is NULL");
    LASER_REQUIRE(m->d.n_layers > 0, LASER_E_SHAPE, "model has no layers (head-only handle)");
    LASER_REQUIRE(kv->d.n_layers == m->d.n_layers && kv->d.n_heads == m->d.n_heads && kv->d.head_dim == m->dh,
                  LASER_E_SHAPE, "KV cache shape does not match the model");
    if (B == 0) return LASER_OK;
    LASER_REQUIRE(seq_ids && pending, LASER_E_INVALID_ARG, "NULL argument");
    LASER_REQUIRE(B <= kv->d.max_seqs, LASER_E_INVALID_ARG, "B exceeds max_seqs");
    const int R = K + 1;
    int max_ub = 0;
    {
        std::vector<char> seen(kv->d.max_seqs, 0);
        for (int b = 0; b < B; ++b) {
            const int s = seq_ids[b];
            LASER_REQUIRE(s >= 0 && s < kv->d.max_seqs, LASER_E_INVALID_ARG, "sequence slot %d out of range", s);
            LASER_REQUIRE(!seen[s], LASER_E_INVALID_ARG, "sequence slot %d appears twice", s);
            seen[s] = 1;
            LASER_REQUIRE(kv->h_len_ub[s] + R <= kv->h_npages[s] * kPageSize, LASER_E_OOM_PAGES,
                          "slot %d: length bound %d + %d rows exceeds the %d tokens reserved", s, kv->h_len_ub[s], R,
                          kv->h_npages[s] * kPageSize);
            LASER_REQUIRE(kv->h_len_ub[s] + R <= m->d.max_pos, LASER_E_LIMIT, "slot %d: position would exceed max_pos %d", s, m->d.max_pos);
            max_ub = std::max(max_ub, kv->h_len_ub[s]);
        }
    }
    const int32_t* ids_dev = nullptr;
    if ((rc = kv->stage_ids(seq_ids, B, stream, &ids_dev))) return rc;
    if (m->use_fused && fused_supported(m, B, K, max_ub)) {
        if (parent)          // token tree: positions (depth) and ancestor masks of the rows
            hipLaunchKernelGGL(rows_kernel, dim3((B * R + 255) / 256), dim3(256), 0, stream, parent, draft_len, ids_dev, kv->len, B, R,
                               m->row_pos, m->row_slot, m->row_anc);
        rc = run_fused(m, kv, ids_dev, pending, drafts, parent, draft_len, B, K, topk, p, mode, accept_len, out_tokens,
                       accept_path, logits_dbg, max_ub, stream);
    } else {
        if ((rc = forward(m, kv, ids_dev, pending, drafts, parent, draft_len, B, K, max_ub, stream))) return rc;
        rc = run_head(m, m->xn, drafts, parent, draft_len, B, K, topk, p, mode, accept_len, out_tokens, accept_path, logits_dbg, stream);
    }
    // only a step that has been enqueued may be committed
    if (rc == LASER_OK)
        for (int b = 0; b < B; ++b) kv->h_last_rows[seq_ids[b]] = R;
    return rc;
}

extern "C" int laser_verify_step(laser_model* mh, laser_kv* kh, const int32_t* seq_ids, const int32_t* pending,
                                 const int32_t* drafts, const int32_t* draft_len, int B, int K, int topk, float p,
                                 int mode, int32_t* accept_len, int32_t* out_tokens, float* logits_dbg, void* stream) {
    return verify_impl(mh, kh, seq_ids, pending, drafts, nullptr, draft_len, B, K, topk, p, mode, accept_len, out_tokens, nullptr,
                       logits_dbg, stream);
}

extern "C" int laser_verify_tree(laser_model* mh, laser_kv* kh, const int32_t* seq_ids, const int32_t* pending,
                                 const int32_t* tree_tokens, const int32_t* tree_parent, const int32_t* tree_len, int B, int K,
                                 int topk, float p, int mode, int32_t* accept_len, int32_t* out_tokens, int32_t* accept_path,
                                 float* logits_dbg, void* stream) {
    LASER_REQUIRE(B <= 0 || K == 0 || (tree_parent && accept_path), LASER_E_INVALID_ARG, "NULL tree_parent or accept_path");
    return verify_impl(mh, kh, seq_ids, pending, tree_tokens, K > 0 ? tree_parent : nullptr, tree_len, B, K, topk, p, mode, accept_len,
                       out_tokens, accept_path, logits_dbg, stream);
}

extern "C" int laser_verify_head(laser_model* mh, const uint16_t* h, const int32_t* drafts, const int32_t* draft_len,
                                 int B, int K, int topk, float p, int mode, int32_t* accept_len, int32_t* out_tokens,
                                 float* logits_dbg, void* stream) {
    Model* m = reinterpret_cast<Model*>(mh);
    int rc = check_step_args(m, B, K, topk, mode, draft_len, drafts, accept_len, out_tokens);
    if (rc) return rc;
    if (B == 0) return LASER_OK;
    LASER_REQUIRE(h != nullptr, LASER_E_INVALID_ARG, "h is NULL");
    return run_head(m, h, drafts, nullptr, draft_len, B, K, topk, p, mode, accept_len, out_tokens, nullptr, logits_dbg, (hipStream_t)stream);
}

extern "C" int laser_verify_head_static(laser_model* mh, const uint16_t* h, const int32_t* drafts, const int32_t* draft_len,
                                        int B, int K, int topk, float p, int mode, int32_t* accept_len, int32_t* out_tokens,
                                        void* stream) {
    Model* m = reinterpret_cast<Model*>(mh);
    int rc = check_step_args(m, B, K, topk, mode, draft_len, drafts, accept_len, out_tokens);
    if (rc) return rc;
    if (B == 0) return LASER_OK;
    LASER_REQUIRE(h != nullptr, LASER_E_INVALID_ARG, "h is NULL");
    return run_head_static(m, h, drafts, draft_len, B, K, topk, p, mode, accept_len, out_tokens, (hipStream_t)stream);
}

extern "C" int laser_profile_begin(laser_model* mh, int max_records) {
    Model* m = reinterpret_cast<Model*>(mh);
    LASER_REQUIRE(m != nullptr && max_records > 0 && max_records <= (1 << 20), LASER_E_INVALID_ARG, "bad argument");
    while ((int)m->prof_ev.size() < 2 * max_records) {
        hipEvent_t e;
        LASER_HIP_CHECK(hipEventCreate(&e));
        m->prof_ev.push_back(e);
    }
    m->prof_cap = max_records;
    m->prof_n = 0;
    m->prof_on = true;
    return LASER_OK;
}

extern "C" int laser_profile_end(laser_model* mh, void* stream, float* total_ms, int* n_launches) {
    Model* m = reinterpret_cast<Model*>(mh);
    LASER_REQUIRE(m != nullptr && total_ms && n_launches, LASER_E_INVALID_ARG, "NULL argument");
    m->prof_on = false;
    LASER_HIP_CHECK(hipStreamSynchronize((hipStream_t)stream));
    double tot = 0.0;
    for (int i = 0; i < m->prof_n; ++i) {
        float ms = 0.f;
        LASER_HIP_CHECK(hipEventElapsedTime(&ms, m->prof_ev[2 * i], m->prof_ev[2 * i + 1]));
        tot += ms;
    }
    *total_ms = (float)tot;
    *n_launches = m->prof_n;
    return LASER_OK;
}

extern "C" int laser_model_set_option(laser_model* mh, const char* name, int value) {
    Model* m = reinterpret_cast<Model*>(mh);
    LASER_REQUIRE(m != nullptr && name != nullptr, LASER_E_INVALID_ARG, "NULL argument");
    if (std::string(name) == "fused") { m->use_fused = value; return LASER_OK; }
    if (std::string(name) == "fused_trace") { m->fused_trace = value; return LASER_OK; }
    if (std::string(name) == "split_ffn") { m->split_ffn = value; return LASER_OK; }
    if (std::string(name) == "f16_copies") {
        LASER_REQUIRE(value == 0 || value == 1, LASER_E_INVALID_ARG, "f16_copies must be 0 or 1");
        m->f16_copies = value;
        return LASER_OK;
    }
    if (std::string(name) == "mid_waves") {
        LASER_REQUIRE(value == 0 || value == 4 || value == 8, LASER_E_INVALID_ARG, "mid_waves must be 0 (choose), 4 or 8");
        m->mid_waves = value;
        return LASER_OK;
    }
    if (std::string(name) == "attn_whole_min") {
        LASER_REQUIRE(value >= 0, LASER_E_INVALID_ARG, "attn_whole_min must be >= 0");
        m->attn_whole_min = value;
        return LASER_OK;
    }
    if (std::string(name) == "attn_waves") {
        LASER_REQUIRE(value == 0 || value == 4 || value == 8, LASER_E_INVALID_ARG, "attn_waves must be 0 (choose), 4 or 8");
        m->attn_waves = value;
        return LASER_OK;
    }
    for (int i = 0; i < 3; ++i)
        if (std::string(name) == (i == 0 ? "ksplit_qkv" : i == 1 ? "ksplit_o" : "ksplit_down")) {
            LASER_REQUIRE(value == 0 || value == 1 || value == 2 || value == 4, LASER_E_INVALID_ARG, "%s must be 0 (choose), 1, 2 or 4", name);
            m->ksplit_opt[i] = value;
            return LASER_OK;
        }
    set_error("unknown option %s", name);
    return LASER_E_INVALID_ARG;
}

extern "C" int laser_model_status(laser_model* mh, void* stream, int* aborted) {
    Model* m = reinterpret_cast<Model*>(mh);
    LASER_REQUIRE(m != nullptr && aborted != nullptr, LASER_E_INVALID_ARG, "NULL argument");
    return fused_status(m, (hipStream_t)stream, aborted);
}

extern "C" int laser_model_read_trace(laser_model* mh, void* stream, long long* out, int max_elems, int* nwg, int* cap) {
    Model* m = reinterpret_cast<Model*>(mh);
    LASER_REQUIRE(m != nullptr && out && nwg && cap, LASER_E_INVALID_ARG, "NULL argument");
    return fused_read_trace(m, (hipStream_t)stream, out, max_elems, nwg, cap);
}
