// Weight-streaming GEMM for 17..80 activation rows (MB = 2..5 row tiles of 16):
//   Y[M][N] = X[M][Kd] * W[N][Kd]^T,  W bf16 (widened to fp16 in registers), X fp16 in one or two planes,
//   fp32 accumulation on the matrix cores.
//
// The few-row kernel (gemm_skinny.h) re-reads the activation rows from L2 at every step: with MB row tiles in two
// planes that is 2 MB x 64 bytes per lane and step against 64 bytes of weights, and at 72 rows it is bound by L2,
// not by HBM. Here the waves of a workgroup own DIFFERENT 16-row weight tiles and walk the SAME reduction range,
// so the activation chunk of a step (rows x 128 elements, both planes) is staged once in LDS by the whole
// workgroup and read from there by every wave, while the next chunk(s) and weight fragments are in flight in
// named register sets (the loops are unrolled by the ring sizes: a register copy of a fragment still in flight
// would make the wave wait for it). 4-wave form: two chunk buffers, chunk s + 1 written in the middle of step s,
// one barrier per step. 8-wave form: one buffer, two barriers, chunk two steps and fragments three steps ahead,
// requests spread over the step. Register pressure is kept below the point of scratch spills inside the loops on
// purpose: a reload from scratch waits, in order, behind every global load issued before it, which puts a full
// HBM latency into each step.
//
// blockIdx.y = part of the reduction: with more than one part each workgroup stores its partial result at
// part + blockIdx.y * M * N and the consumer adds the parts in order (store / accumulate epilogues only).
// SwiGLU: a gate tile and its up tile go to neighbouring waves (twice the waves, half the registers each); the up
// wave hands its sums over through LDS at the end.
#pragma once

#include <type_traits>

#include "gemm_skinny.h"
#include "head_part.h"

namespace laser {

// EPI_HEAD: the output head; a workgroup keeps one record of partial statistics per row (head_part.h) instead of
// its logits (chunk = workgroup: NW x 16 vocabulary entries).
enum { EPI_F32 = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_HEAD = 3 };

struct GemmMidArgs {
    const uint16_t* W;      // [N][Kd] bf16  (EPI_SWIGLU: [2N][Kd], gate rows then up rows)
    const uint16_t* X;      // [M][Kd] fp16
    const uint16_t* Xlo;    // [M][Kd] low plane of split activations (SPLIT only)
    int M, N, Kd;           // 16 < M <= 80, N % 16 == 0, Kd % 128 == 0
    float* outf;            // EPI_F32: [M][N] store;  EPI_RESID: [M][N] accumulate (one part only)
    uint16_t* outh;         // EPI_SWIGLU: [M][N] fp16
    float* part;            // gridDim.y > 1: [gridDim.y][M][N] partial results
    HeadPart hp{};          // EPI_HEAD: where the per-(row, workgroup) statistics go
};

// NW = waves (weight tiles) per workgroup, 4 or 8: what enters a compute unit per step is NW x 4 KB of weights
// plus ONE activation chunk, so more waves per workgroup mean fewer chunk bytes per weight byte but fewer
// workgroups to spread over the chip; gemm_mid_plan picks per launch shape.
template <int MB, int EPI, bool SPLIT, int NW>
__global__ __launch_bounds__(NW * 64, NW == 4 ? 2 : 1) void gemm_mid_kernel(GemmMidArgs a) {
    constexpr bool DEEP = NW == 8;
    constexpr int ROWS = MB * 16, NP = SPLIT ? 2 : 1;
    constexpr int NT = NW * 64;                              // threads
    constexpr int NPIECE = (ROWS * 16 + NT - 1) / NT;        // 16-byte pieces of a plane's chunk per thread
    constexpr int LDH = kGemmKStep + 8;   // halves per LDS row: 272 bytes, the 16 rows of a 16-byte read hit distinct banks
    constexpr int BUFH = NP * ROWS * LDH; // halves per chunk buffer
    // dynamic LDS: one chunk buffer for the 8-wave form, two for the 4-wave form (gemm_mid_lds_bytes)
    extern __shared__ __attribute__((aligned(16))) uint16_t sx[];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int r = lane & 15, g = lane >> 4;
    const int ntiles = a.N / 16;
    const int vt = blockIdx.x * NW + wave;
    const int tile_raw = EPI == EPI_SWIGLU ? vt >> 1 : vt;
    const int sel = EPI == EPI_SWIGLU ? vt & 1 : 0;          // SwiGLU: 0 = gate rows, 1 = up rows
    const bool active = tile_raw < ntiles;
    const int tile = active ? tile_raw : ntiles - 1;        // idle waves stream a valid tile and drop the result
    const int S = gridDim.y, ks = blockIdx.y;
    const int ksteps = a.Kd / kGemmKStep, per = (ksteps + S - 1) / S;
    const int sbeg = ks * per, send = min(ksteps, sbeg + per);

    const uint16_t* const wp = a.W + ((size_t)sel * a.N + (size_t)tile * 16 + r) * a.Kd + g * 32;
    // staging: piece p = tid + NT i covers row p / 16, 16-byte column p % 16 of the chunk; where the pieces do not
    // divide evenly the last ones are staged twice (same bytes to the same place)
    // (32-bit element offsets from the uniform plane bases: M * Kd is far below 2^31 here)
    unsigned xoff[NPIECE];
    int xdst[NPIECE];
#pragma unroll
    for (int i = 0; i < NPIECE; ++i) {
        const int p = min(tid + NT * i, ROWS * 16 - 1), row = p >> 4, c = p & 15;
        xoff[i] = (unsigned)min(row, a.M - 1) * (unsigned)a.Kd + c * 8;
        xdst[i] = row * LDH + c * 8;
    }
    float4_t acc[MB], acl[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) { acc[mb] = float4_t{0.f, 0.f, 0.f, 0.f}; acl[mb] = float4_t{0.f, 0.f, 0.f, 0.f}; }

    // Register rings. DEEP = false: the activation pieces and the weight fragments of step s + 1 are requested during
    // step s, all at once (pieces right after the first barrier, fragments at the top). DEEP = true (the 8-wave form,
    // whose staging pieces per thread are few): pieces two steps ahead, fragments three, and the requests are spread
    // over the step's row tiles between the matrix instructions -- issued in one burst, the 80 vector loads of a
    // workgroup-step occupy the compute unit's one address unit for about as long as the matrix work takes, and every
    // wave sits behind its own burst before it reaches its LDS reads. Ring slots are indexed by the step's number
    // within the unrolled body, so they stay named registers (a register copy of a fragment in flight would wait for
    // it); the main loop has no branch between steps (at a join the compiler's wait counters fall back to
    // "everything", which would undo the prefetch), the last few steps run one by one.
    constexpr int XD = DEEP ? 2 : 1, WD = DEEP ? 3 : 1;
    constexpr int XR = XD, WR = WD + 1, UNROLL = DEEP ? 4 : 2;   // a common multiple of XR and WR
    constexpr int NLOAD = 4 + NP * NPIECE;                        // vector loads per thread and step
    Frag8 w[WR][4];
    u32x4 xr[XR][NP][NPIECE];
    // load l of a step: 0..3 = weight fragment l, then the activation pieces plane by plane. GUARD: requests for
    // steps past the part's end are skipped (a uniform branch; the main loop never asks for such a step and is
    // instantiated without it).
    auto load_one = [&](auto guard_c, int st_w, int st_x, auto l_c, auto ws_c, auto xs_c) {
        constexpr bool GUARD = decltype(guard_c)::value;
        constexpr int l = decltype(l_c)::value, WS = decltype(ws_c)::value, XS = decltype(xs_c)::value;
        if constexpr (l < 4) {
            if (!GUARD || st_w < send) w[WS][l].v4 = *reinterpret_cast<const u32x4*>(wp + st_w * kGemmKStep + l * 8);
        } else {
            constexpr int pl = (l - 4) / NPIECE, i = (l - 4) % NPIECE;
            if (!GUARD || st_x < send) xr[XS][pl][i] = *reinterpret_cast<const u32x4*>((pl == 0 ? a.X : a.Xlo) + st_x * kGemmKStep + xoff[i]);
        }
    };
    // one step, J = its number within the unrolled body: ring slots J % XR (chunk) and J % WR (fragments)
    auto step = [&](auto guard_c, int st, auto j_c) {
        constexpr int J = decltype(j_c)::value, XS = J % XR, WS = J % WR, WF = (J + WD) % WR;
        using WFc = std::integral_constant<int, WF>;
        using XSc = std::integral_constant<int, XS>;
        if constexpr (!DEEP) static_for<0, 4>([&](auto l) { load_one(guard_c, st + WD, send, l, WFc{}, XSc{}); });
#pragma unroll
        for (int i = 0; i < NPIECE; ++i) {
            *reinterpret_cast<u32x4*>(sx + xdst[i]) = xr[XS][0][i];
            if constexpr (SPLIT) *reinterpret_cast<u32x4*>(sx + ROWS * LDH + xdst[i]) = xr[XS][NP - 1][i];
        }
        __syncthreads();
        if constexpr (!DEEP) static_for<4, NLOAD>([&](auto l) { load_one(guard_c, send, st + XD, l, WFc{}, XSc{}); });
        Frag8 (&cur)[4] = w[WS];
#pragma unroll
        for (int c = 0; c < 4; ++c) bf16x8_to_f16x8(cur[c]);
        // The row tiles' fragments are read from LDS one tile ahead of the matrix instructions that use them (two
        // fragment sets; the scheduling fences keep the compiler from sinking the reads back to their uses: with
        // one or two waves per SIMD nothing else would cover the LDS latency of 8 reads per tile).
        Frag8 b[2][NP * 4];
        auto read_b = [&](int mb, Frag8 (&f)[NP * 4]) {
            const uint16_t* row = sx + (mb * 16 + r) * LDH + g * 32;
#pragma unroll
            for (int c = 0; c < 4; ++c) f[c].v4 = *reinterpret_cast<const u32x4*>(row + c * 8);
            if constexpr (SPLIT) {
#pragma unroll
                for (int c = 0; c < 4; ++c) f[4 + c].v4 = *reinterpret_cast<const u32x4*>(row + ROWS * LDH + c * 8);
            }
        };
        read_b(0, b[0]);
        static_for<0, MB>([&](auto mb_c) {
            constexpr int mb = decltype(mb_c)::value;
            if constexpr (mb + 1 < MB) read_b(mb + 1, b[(mb + 1) & 1]);
            if constexpr (DEEP)          // this row tile's share of the step's requests: loads [mb, mb + 1) * NLOAD / MB
                static_for<mb * NLOAD / MB, (mb + 1) * NLOAD / MB>([&](auto l) { load_one(guard_c, st + WD, st + XD, l, WFc{}, XSc{}); });
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[mb] = mfma_16x16x32(cur[c], b[mb & 1][c], acc[mb]);
            if constexpr (SPLIT) {
#pragma unroll
                for (int c = 0; c < 4; ++c) acl[mb] = mfma_16x16x32(cur[c], b[mb & 1][NP * 4 - 4 + c], acl[mb]);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        __syncthreads();                                     // the chunk is free for the next step's pieces
    };
    if constexpr (DEEP) {
        // prologue: the first XD chunks and WD fragment sets
        // (in the order of first use, pinned by scheduling fences: loads complete in issue order, and the loop header's
        // wait for the first chunk must not find a later request ahead of it)
        auto prologue = [&](auto guard_c) {
            static_for<0, XD>([&](auto d) {
                static_for<4, NLOAD>([&](auto l) { load_one(guard_c, send, sbeg + decltype(d)::value, l, std::integral_constant<int, 0>{}, d); });
                __builtin_amdgcn_sched_barrier(0);
            });
            static_for<0, WD>([&](auto d) {
                static_for<0, 4>([&](auto l) { load_one(guard_c, sbeg + decltype(d)::value, send, l, d, std::integral_constant<int, 0>{}); });
                __builtin_amdgcn_sched_barrier(0);
            });
        };
        // main loop: groups of UNROLL steps all of whose requests lie inside the part, entered through a prologue without
        // guards (so that the loop header sees known wait-counter states on both of its edges); then up to
        // UNROLL + WD - 1 steps one by one (the ring positions carry on: every group starts at position 0)
        int st = sbeg;                                           // sbeg, send are the same for every wave of the workgroup
        if (st + UNROLL + WD <= send) {
            prologue(std::false_type{});
            for (; st + UNROLL + WD <= send; st += UNROLL)
                static_for<0, UNROLL>([&](auto j) { step(std::false_type{}, st + decltype(j)::value, j); });
        } else {
            prologue(std::true_type{});
        }
        static_for<0, UNROLL + WD - 1>([&](auto j) {
            if (st + decltype(j)::value < send) step(std::true_type{}, st + decltype(j)::value, j);
        });
    } else {
        // 4-wave form: two chunk buffers. The pieces of chunk s + 1 (requested half a step or more earlier) are
        // written into the other buffer in the MIDDLE of step s, between the matrix instructions of two row tiles,
        // and the request for chunk s + 2 follows them: the write, its wait and the requests' issue time hide behind
        // the matrix work, and a step needs ONE workgroup barrier instead of two.
        auto write_chunk = [&](int buf) {
#pragma unroll
            for (int i = 0; i < NPIECE; ++i) {
                *reinterpret_cast<u32x4*>(sx + buf * BUFH + xdst[i]) = xr[0][0][i];
                if constexpr (SPLIT) *reinterpret_cast<u32x4*>(sx + buf * BUFH + ROWS * LDH + xdst[i]) = xr[0][NP - 1][i];
            }
        };
        using X0 = std::integral_constant<int, 0>;
        auto step2 = [&](auto guard_c, int st, auto j_c) {
            constexpr bool GUARD = decltype(guard_c)::value;
            constexpr int J = decltype(j_c)::value, CB = J % 2, NB = (J + 1) % 2, WS = J % WR, WF = (J + WD) % WR;
            using WFc = std::integral_constant<int, WF>;
            static_for<0, 4>([&](auto l) { load_one(guard_c, st + WD, send, l, WFc{}, X0{}); });
            Frag8 (&cur)[4] = w[WS];
#pragma unroll
            for (int c = 0; c < 4; ++c) bf16x8_to_f16x8(cur[c]);
            Frag8 b[2][NP * 4];
            auto read_b = [&](int mb, Frag8 (&f)[NP * 4]) {
                const uint16_t* row = sx + CB * BUFH + (mb * 16 + r) * LDH + g * 32;
#pragma unroll
                for (int c = 0; c < 4; ++c) f[c].v4 = *reinterpret_cast<const u32x4*>(row + c * 8);
                if constexpr (SPLIT) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) f[4 + c].v4 = *reinterpret_cast<const u32x4*>(row + ROWS * LDH + c * 8);
                }
            };
            read_b(0, b[0]);
            static_for<0, MB>([&](auto mb_c) {
                constexpr int mb = decltype(mb_c)::value;
                if constexpr (mb + 1 < MB) read_b(mb + 1, b[(mb + 1) & 1]);
                if constexpr (mb == MB / 2) {
                    if (!GUARD || st + 1 < send) write_chunk(NB);
                    static_for<4, NLOAD>([&](auto l) { load_one(guard_c, send, st + 2, l, WFc{}, X0{}); });
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[mb] = mfma_16x16x32(cur[c], b[mb & 1][c], acc[mb]);
                if constexpr (SPLIT) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) acl[mb] = mfma_16x16x32(cur[c], b[mb & 1][NP * 4 - 4 + c], acl[mb]);
                }
                __builtin_amdgcn_sched_barrier(0);
            });
            __syncthreads();         // chunk s + 1 is complete for everyone, chunk s is free
        };
        // prologue: chunk sbeg into buffer 0, chunk sbeg + 1 requested, the first fragment set
        auto prologue2 = [&](auto guard_c) {
            static_for<4, NLOAD>([&](auto l) { load_one(std::false_type{}, send, sbeg, l, X0{}, X0{}); });   // sbeg < send always
            __builtin_amdgcn_sched_barrier(0);
            static_for<0, 4>([&](auto l) { load_one(std::false_type{}, sbeg, send, l, X0{}, X0{}); });
            __builtin_amdgcn_sched_barrier(0);
            write_chunk(0);
            static_for<4, NLOAD>([&](auto l) { load_one(guard_c, send, sbeg + 1, l, X0{}, X0{}); });
            __syncthreads();
        };
        int st = sbeg;                                       // sbeg, send are the same for every wave of the workgroup
        if (st + UNROLL + 2 <= send) {
            prologue2(std::false_type{});
            for (; st + UNROLL + 2 <= send; st += UNROLL)
                static_for<0, UNROLL>([&](auto j) { step2(std::false_type{}, st + decltype(j)::value, j); });
        } else {
            prologue2(std::true_type{});
        }
        static_for<0, UNROLL + 1>([&](auto j) {
            if (st + decltype(j)::value < send) step2(std::true_type{}, st + decltype(j)::value, j);
        });
    }
    float v[MB][4];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int i = 0; i < 4; ++i) v[mb][i] = SPLIT ? acc[mb][i] + acl[mb][i] * kLoInv : acc[mb][i];
    const int n = tile * 16 + 4 * g;
    if constexpr (EPI == EPI_HEAD) {
        // per wave 16 vocabulary entries of every row: lane statistics, merged over the four lane groups, then over
        // the workgroup's waves in wave order through LDS (the loop's last barrier freed sx). A call with k <= 2 (the
        // paper's default, Sec. 4.1.4) keeps two-entry lists, which is all its rank test needs.
        float* ex = reinterpret_cast<float*>(sx);             // [NW][ROWS][kWords]
        auto head_epilogue = [&](auto depth) {
            using Stat = RowStatT<decltype(depth)::value>;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const int row = mb * 16 + r;
                Stat st;
                st.init();
                if (active) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) st.add(v[mb][i], n + i);
                    if (row < a.M)
                        store_candidates(a.hp, row, n, 4, [&](int c) { return c == 0 ? v[mb][0] : c == 1 ? v[mb][1] : c == 2 ? v[mb][2] : v[mb][3]; });
                    if (a.hp.logits_dbg && row < a.M)
                        *reinterpret_cast<float4*>(a.hp.logits_dbg + (size_t)row * a.N + n) = make_float4(v[mb][0], v[mb][1], v[mb][2], v[mb][3]);
                }
                st.merge_from_lane(16);
                st.merge_from_lane(32);
                if (g == 0) st.to_lds(ex + ((size_t)wave * ROWS + row) * Stat::kWords);
            }
            __syncthreads();
            if (tid < ROWS && tid < a.M) {
                Stat m;
                m.init();
                for (int w = 0; w < NW; ++w) m.merge_lds(ex + ((size_t)w * ROWS + tid) * Stat::kWords);
                m.store(a.hp, tid, (int)blockIdx.x);
            }
        };
        if (a.hp.topk <= 2) head_epilogue(std::integral_constant<int, 2>{});
        else head_epilogue(std::integral_constant<int, KT>{});
    } else if constexpr (EPI == EPI_SWIGLU) {
        static_assert((NW / 2) * MB * 4 * 64 * sizeof(float) <= BUFH * sizeof(uint16_t), "the exchange area must fit a chunk buffer");
        float* ex = reinterpret_cast<float*>(sx);             // [pair][mb][i][lane]; the loop's last barrier freed sx
        if (sel == 1) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int i = 0; i < 4; ++i) ex[(((wave >> 1) * MB + mb) * 4 + i) * 64 + lane] = v[mb][i];
        }
        __syncthreads();
        if (sel == 1 || !active) return;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int row = mb * 16 + r;
            if (row >= a.M) continue;
            Frag4 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float up = ex[(((wave >> 1) * MB + mb) * 4 + i) * 64 + lane];
                o.h[i] = f32_to_f16(v[mb][i] / (1.f + __expf(-v[mb][i])) * up);
            }
            *reinterpret_cast<uint2*>(a.outh + (size_t)row * a.N + n) = o.u;
        }
    } else {
        if (!active) return;
        float* const outf = S > 1 ? a.part + (size_t)ks * a.M * a.N : a.outf;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int row = mb * 16 + r;
            if (row >= a.M) continue;
            float4* p = reinterpret_cast<float4*>(outf + (size_t)row * a.N + n);
            float4 t = make_float4(v[mb][0], v[mb][1], v[mb][2], v[mb][3]);
            if (EPI == EPI_RESID && S == 1) { const float4 o = *p; t.x += o.x; t.y += o.y; t.z += o.z; t.w += o.w; }
            *p = t;
        }
    }
}

// Compute units of the device (asked once).
inline int gemm_mid_cu_count() {
    static const int n = [] {
        int v = 0;
        return hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, 0) == hipSuccess && v > 0 ? v : 256;
    }();
    return n;
}

struct GemmMidPlan { int NW, S; };

// Waves per workgroup and reduction parts for one launch: the pair with the fewest kilobytes entering the busiest
// compute unit (weights + activation chunks over its workgroups' steps, two steps' worth of start-up per
// workgroup -- five for the 8-wave form, whose deeper rings take longer to fill and drain --, plus its share of
// writing and re-reading the partial results). Parts only for store / accumulate
// epilogues with a workspace, each part at least two steps. A function of the launch shape only.
inline GemmMidPlan gemm_mid_plan(int M, int N, int Kd, int planes, bool swiglu, size_t part_floats, int force_nw = 0) {
    const int n_cu = gemm_mid_cu_count();
    const long vtiles = (long)(N / 16) * (swiglu ? 2 : 1), ksteps = Kd / kGemmKStep;
    const long xkb = (long)((M + 15) / 16) * 4 * planes;
    GemmMidPlan best{4, 1};
    double best_cost = 1e300;
    for (int nw = 4; nw <= 8; nw *= 2)
        for (int S = 1; S <= 8; S *= 2) {
            if (force_nw && nw != force_nw) break;
            if (S > 1 && (swiglu || ksteps / S < 2 || (size_t)S * M * N > part_floats)) break;
            const long n_wg = (vtiles + nw - 1) / nw * S;
            const long per_cu = (n_wg + n_cu - 1) / n_cu, steps = (ksteps + S - 1) / S;
            const double cost = (double)per_cu * (steps + (nw == 8 ? 5 : 2)) * (nw * 4 + xkb) +
                                (S > 1 ? 2.0 * S * M * N * 4 / 1024 / n_cu : 0.0);
            if (cost < best_cost) { best_cost = cost; best = {nw, S}; }
        }
    return best;
}

// Dynamic LDS of a launch: one chunk buffer (both planes, padded rows) for the 8-wave form, two for the 4-wave form.
constexpr size_t gemm_mid_lds_bytes(int mb, bool split, int nw, bool head = false) {
    const size_t chunks = (size_t)(nw == 8 ? 1 : 2) * (split ? 2 : 1) * mb * 16 * (kGemmKStep + 8) * sizeof(uint16_t);
    const size_t records = head ? (size_t)nw * mb * 16 * RowStat::kWords * sizeof(float) : 0;   // the head's merge over the waves
    return chunks > records ? chunks : records;
}

// Caller guarantees 16 < M <= 80, N % 16 == 0, Kd % 128 == 0, and a plan made for this shape.
template <int EPI, bool SPLIT>
inline void launch_gemm_mid(const GemmMidArgs& a, GemmMidPlan pl, hipStream_t stream) {
    const int vtiles = (EPI == EPI_SWIGLU ? 2 : 1) * (a.N / 16), mblocks = (a.M + 15) / 16;
    dim3 grid((unsigned)((vtiles + pl.NW - 1) / pl.NW), (unsigned)pl.S);
    constexpr bool kHead = EPI == EPI_HEAD;
    auto go = [&](auto mbc) {
        constexpr int mb = decltype(mbc)::value;
        // more than 64 KB of dynamic LDS has to be allowed per kernel, once
        static const bool allowed = [] {
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mid_kernel<mb, EPI, SPLIT, 8>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_mid_lds_bytes(mb, SPLIT, 8, kHead));
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mid_kernel<mb, EPI, SPLIT, 4>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_mid_lds_bytes(mb, SPLIT, 4, kHead));
            return true;
        }();
        (void)allowed;
        if (pl.NW == 8)
            hipLaunchKernelGGL((gemm_mid_kernel<mb, EPI, SPLIT, 8>), grid, dim3(512), gemm_mid_lds_bytes(mb, SPLIT, 8, kHead), stream, a);
        else
            hipLaunchKernelGGL((gemm_mid_kernel<mb, EPI, SPLIT, 4>), grid, dim3(256), gemm_mid_lds_bytes(mb, SPLIT, 4, kHead), stream, a);
    };
    switch (mblocks) {
        case 2: go(std::integral_constant<int, 2>{}); break;
        case 3: go(std::integral_constant<int, 3>{}); break;
        case 4: go(std::integral_constant<int, 4>{}); break;
        default: go(std::integral_constant<int, 5>{}); break;
    }
}

}  // namespace laser
