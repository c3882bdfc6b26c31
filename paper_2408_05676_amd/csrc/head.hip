// Fused output head + acceptance (Sec. 3.4 Eq. 7-8; greedy Eq. 4; correction rule of Sec. 2.1).
//
// Pass 1 (lm_head_kernel): every wavefront owns a contiguous chunk of the vocabulary, streams those
// rows of the head matrix once through the matrix cores against all verified rows, and keeps, per
// row, running softmax statistics (max, sum of exp), the arg-max (smaller id on ties), the logit of
// the row's draft token, and its chunk's best LASER_MAX_TOPK (logit, id) pairs -- all in registers.
// Logits are never written unless a debug buffer is passed.
// Pass 2 (accept_kernel): one block per sequence merges the per-chunk partials. The draft's rank is
// the number of partial-list entries ordered before it; if a chunk hides an entry that precedes the
// draft, that chunk already contributes >= LASER_MAX_TOPK >= k listed ones, so "rank < k" is exact.
// The block then scans the rows left to right and emits accepted drafts plus the correction token.
//
// More than 16 rows: the per-lane running statistics of pass 1 (one set per row tile) and the serial merge of
// pass 2 cost more than they save. Instead the logits are written to an fp32 workspace by a GEMM (17..80 rows:
// the weight-streaming kernel of gemm_mid.h, the head matrix read once; more: the LDS-tiled matrix-core GEMM;
// the logits are written and read once, 8 bytes each against the 2 * d flops they cost), head_stats_kernel
// reduces each row (max, sum of exp, arg-max, the draft's logit and its exact rank) and decides it,
// head_scan_kernel scans the rows.
#include <cmath>
#include <mutex>

#include "gemm_mfma.h"
#include "gemm_skinny.h"
#include "gemm_mid.h"
#include "state.h"

namespace laser {

constexpr int KT = LASER_MAX_TOPK;
constexpr int kHeadStreamMaxRows = 16;   // beyond this the logits are written out by a GEMM and reduced row by row
constexpr int kHeadMidMaxRows = 80;      // up to here that GEMM streams the head matrix once; beyond, the tiled one

struct HeadArgs {
    const uint16_t* W; const uint16_t* H; int M, V, d, tiles_per_wave, chunks;
    const int32_t* row_x;
    float* hp_max; float* hp_sum; int32_t* hp_arg; float* hp_topv; int32_t* hp_topi; float* hp_lx;
    float* logits_dbg;
};

__global__ void head_rows_kernel(const int32_t* drafts, const int32_t* draft_len, int B, int K, int vocab,
                                 int32_t* row_x, float* hp_lx) {
    const int m = blockIdx.x * blockDim.x + threadIdx.x, R = K + 1;
    if (m >= B * R) return;
    const int b = m / R, r = m % R;
    int x = (r < K && r < draft_len[b]) ? drafts[(size_t)b * K + r] : -1;
    if (x >= vocab) x = -1;
    row_x[m] = x;
    hp_lx[m] = -INFINITY;
}

// ordering of (logit, id): larger logit first, smaller id on ties
__device__ inline bool before(float v, int i, float w, int j) { return v > w || (v == w && i < j); }

struct RowStat {
    float mx, sum, lx;
    int arg;
    float tv[KT];
    int ti[KT];
    __device__ void init() {
        mx = -INFINITY; sum = 0.f; lx = -INFINITY; arg = 0x7FFFFFFF;
#pragma unroll
        for (int j = 0; j < KT; ++j) { tv[j] = -INFINITY; ti[j] = 0x7FFFFFFF; }
    }
    __device__ void push_top(float v, int n) {
        if (!before(v, n, tv[KT - 1], ti[KT - 1])) return;
        tv[KT - 1] = v; ti[KT - 1] = n;
#pragma unroll
        for (int j = KT - 1; j > 0; --j) {
            if (before(tv[j], ti[j], tv[j - 1], ti[j - 1])) {
                float fv = tv[j]; tv[j] = tv[j - 1]; tv[j - 1] = fv;
                int fi = ti[j]; ti[j] = ti[j - 1]; ti[j - 1] = fi;
            }
        }
    }
    __device__ void add(float v, int n) {
        if (v > mx) { sum = sum * __expf(mx - v) + 1.f; mx = v; arg = n; }   // ids arrive ascending per lane
        else sum += __expf(v - mx);
        push_top(v, n);
    }
    __device__ void merge_from_lane(int src_xor) {
        const float omx = __shfl_xor(mx, src_xor), osum = __shfl_xor(sum, src_xor), olx = __shfl_xor(lx, src_xor);
        const int oarg = __shfl_xor(arg, src_xor);
        float otv[KT]; int oti[KT];
#pragma unroll
        for (int j = 0; j < KT; ++j) { otv[j] = __shfl_xor(tv[j], src_xor); oti[j] = __shfl_xor(ti[j], src_xor); }
        const float M = fmaxf(mx, omx);
        if (M != -INFINITY) sum = sum * __expf(mx - M) + osum * __expf(omx - M);
        if (before(omx, oarg, mx, arg)) arg = oarg;
        mx = M;
        lx = fmaxf(lx, olx);
#pragma unroll
        for (int j = 0; j < KT; ++j) push_top(otv[j], oti[j]);
    }
};

template <int MB>
__global__ __launch_bounds__(256) void lm_head_kernel(HeadArgs a) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 15, g = lane >> 4;
    const int chunk = blockIdx.x * 4 + wave;
    if (chunk >= a.chunks) return;
    const int ntiles = a.V / 16;
    const int t0 = chunk * a.tiles_per_wave, t1 = min(ntiles, t0 + a.tiles_per_wave);
    const int row0 = blockIdx.y * MB * 16;

    RowStat st[MB];
    int x[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        st[mb].init();
        const int row = row0 + mb * 16 + r;
        x[mb] = row < a.M ? a.row_x[row] : -1;
    }
    for (int t = t0; t < t1; ++t) {
        float4_t acc[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[mb] = float4_t{0.f, 0.f, 0.f, 0.f};
        wave_gemm_tile<MB, false>(a.W + (size_t)t * 16 * a.d, (size_t)a.d, a.H, nullptr, a.d, a.M, row0, 0, a.d, acc);
        const int n = t * 16 + 4 * g;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                st[mb].add(acc[mb][i], n + i);
                if (n + i == x[mb]) st[mb].lx = acc[mb][i];
            }
            const int row = row0 + mb * 16 + r;
            if (a.logits_dbg && row < a.M)
                *reinterpret_cast<float4*>(a.logits_dbg + (size_t)row * a.V + n) =
                    make_float4(acc[mb][0], acc[mb][1], acc[mb][2], acc[mb][3]);
        }
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        st[mb].merge_from_lane(16);
        st[mb].merge_from_lane(32);
        const int row = row0 + mb * 16 + r;
        if (g == 0 && row < a.M) {
            const size_t o = (size_t)row * a.chunks + chunk;
            a.hp_max[o] = st[mb].mx; a.hp_sum[o] = st[mb].sum; a.hp_arg[o] = st[mb].arg;
#pragma unroll
            for (int j = 0; j < KT; ++j) { a.hp_topv[o * KT + j] = st[mb].tv[j]; a.hp_topi[o * KT + j] = st[mb].ti[j]; }
            if (st[mb].lx != -INFINITY) a.hp_lx[row] = st[mb].lx;
        }
    }
}

struct AcceptArgs {
    const float* hp_max; const float* hp_sum; const int32_t* hp_arg; const float* hp_topv; const int32_t* hp_topi;
    const float* hp_lx; const int32_t* row_x; const int32_t* drafts; const int32_t* draft_len;
    int K, chunks, topk, mode; float p;
    int32_t* accept_len; int32_t* out_tokens;
};

__global__ __launch_bounds__(256) void accept_kernel(AcceptArgs a) {
    __shared__ float s_f[4][3];
    __shared__ int s_i[4][2];
    __shared__ int row_ok[LASER_MAX_DRAFT + 1], row_arg[LASER_MAX_DRAFT + 1];
    const int b = blockIdx.x, R = a.K + 1;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int r = 0; r < R; ++r) {
        const int row = b * R + r;
        const int x = a.row_x[row];
        const float lx = a.hp_lx[row];
        float mx = -INFINITY, sum = 0.f;
        int arg = 0x7FFFFFFF, ahead = 0;
        for (int c = threadIdx.x; c < a.chunks; c += 256) {
            const size_t o = (size_t)row * a.chunks + c;
            const float cm = a.hp_max[o], cs = a.hp_sum[o];
            const int ca = a.hp_arg[o];
            const float M = fmaxf(mx, cm);
            sum = sum * __expf(mx - M) + cs * __expf(cm - M);
            if (before(cm, ca, mx, arg)) arg = ca;
            mx = M;
            if (x >= 0)
#pragma unroll
                for (int j = 0; j < KT; ++j) {
                    const float v = a.hp_topv[o * KT + j];
                    const int i = a.hp_topi[o * KT + j];
                    ahead += (i != x && before(v, i, lx, x)) ? 1 : 0;
                }
        }
        for (int off = 32; off > 0; off >>= 1) {
            const float omx = __shfl_xor(mx, off), osum = __shfl_xor(sum, off);
            const int oarg = __shfl_xor(arg, off);
            ahead += __shfl_xor(ahead, off);
            const float M = fmaxf(mx, omx);
            if (M != -INFINITY) sum = sum * __expf(mx - M) + osum * __expf(omx - M);
            if (before(omx, oarg, mx, arg)) arg = oarg;
            mx = M;
        }
        __syncthreads();
        if (lane == 0) { s_f[wave][0] = mx; s_f[wave][1] = sum; s_i[wave][0] = arg; s_i[wave][1] = ahead; }
        __syncthreads();
        if (threadIdx.x == 0) {
            float M = -INFINITY, S = 0.f; int A = 0x7FFFFFFF, rank = 0;
            for (int w = 0; w < 4; ++w) {
                const float wm = s_f[w][0];
                const float nm = fmaxf(M, wm);
                if (nm != -INFINITY) S = S * __expf(M - nm) + s_f[w][1] * __expf(wm - nm);
                if (before(wm, s_i[w][0], M, A)) A = s_i[w][0];
                M = nm;
                rank += s_i[w][1];
            }
            bool ok = false;
            if (x >= 0) {
                const float q = __expf(lx - M) / S;
                const bool in_k = rank < a.topk, above = q > a.p, top1 = rank == 0;
                ok = a.mode == LASER_MODE_RV ? (in_k && above)
                   : a.mode == LASER_MODE_RV_OR_TOP1 ? (top1 || (in_k && above))
                   : a.mode == LASER_MODE_TOPK_ONLY ? in_k : (top1 || above);
            }
            row_ok[r] = ok ? 1 : 0;
            row_arg[r] = A;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int dl = a.draft_len[b];
        dl = dl < 0 ? 0 : (dl > a.K ? a.K : dl);
        int n = 0;
        while (n < dl && row_ok[n]) ++n;
        a.accept_len[b] = n;
        int32_t* out = a.out_tokens + (size_t)b * R;
        for (int j = 0; j < R; ++j) out[j] = j < n ? a.drafts[(size_t)b * a.K + j] : (j == n ? row_arg[n] : -1);
    }
}

// One workgroup per row of the logits matrix: softmax statistics, arg-max (smaller id on ties), the
// draft's logit, the number of vocabulary entries ordered before the draft, and the row's decision.
struct StatsArgs {
    const float* logits; const int32_t* row_x; int V, topk, mode; float p;
    int32_t* row_ok; int32_t* row_arg;
};

__global__ __launch_bounds__(256) void head_stats_kernel(StatsArgs a) {
    __shared__ float s_f[4][2];
    __shared__ int s_i[4][2];
    const int row = blockIdx.x;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const float* l = a.logits + (size_t)row * a.V;
    const int x = a.row_x[row];
    const float lx = x >= 0 ? l[x] : -INFINITY;
    float mx = -INFINITY, sum = 0.f;
    int arg = 0x7FFFFFFF, ahead = 0;
    for (int n = threadIdx.x * 4; n < a.V; n += 256 * 4) {          // V is a multiple of 16
        const float4 v = *reinterpret_cast<const float4*>(l + n);
        const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (e[i] > mx) { sum = sum * __expf(mx - e[i]) + 1.f; mx = e[i]; arg = n + i; }   // ids ascend per thread
            else sum += __expf(e[i] - mx);
            ahead += (n + i != x && before(e[i], n + i, lx, x)) ? 1 : 0;
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        const float omx = __shfl_xor(mx, off), osum = __shfl_xor(sum, off);
        const int oarg = __shfl_xor(arg, off);
        ahead += __shfl_xor(ahead, off);
        const float M = fmaxf(mx, omx);
        if (M != -INFINITY) sum = sum * __expf(mx - M) + osum * __expf(omx - M);
        if (before(omx, oarg, mx, arg)) arg = oarg;
        mx = M;
    }
    if (lane == 0) { s_f[wave][0] = mx; s_f[wave][1] = sum; s_i[wave][0] = arg; s_i[wave][1] = ahead; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float M = -INFINITY, S = 0.f; int A = 0x7FFFFFFF, rank = 0;
        for (int w = 0; w < 4; ++w) {
            const float wm = s_f[w][0];
            const float nm = fmaxf(M, wm);
            if (nm != -INFINITY) S = S * __expf(M - nm) + s_f[w][1] * __expf(wm - nm);
            if (before(wm, s_i[w][0], M, A)) A = s_i[w][0];
            M = nm;
            rank += s_i[w][1];
        }
        bool ok = false;
        if (x >= 0) {
            const float q = __expf(lx - M) / S;
            const bool in_k = rank < a.topk, above = q > a.p, top1 = rank == 0;
            ok = a.mode == LASER_MODE_RV ? (in_k && above)
               : a.mode == LASER_MODE_RV_OR_TOP1 ? (top1 || (in_k && above))
               : a.mode == LASER_MODE_TOPK_ONLY ? in_k : (top1 || above);
        }
        a.row_ok[row] = ok ? 1 : 0;
        a.row_arg[row] = A;
    }
}

// One thread per sequence: longest accepted prefix, then the correction token (Sec. 2.1).
__global__ void head_scan_kernel(const int32_t* row_ok, const int32_t* row_arg, const int32_t* drafts,
                                 const int32_t* draft_len, int B, int K, int32_t* accept_len, int32_t* out_tokens) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x, R = K + 1;
    if (b >= B) return;
    int dl = draft_len[b];
    dl = dl < 0 ? 0 : (dl > K ? K : dl);
    int n = 0;
    while (n < dl && row_ok[b * R + n]) ++n;
    accept_len[b] = n;
    int32_t* out = out_tokens + (size_t)b * R;
    for (int j = 0; j < R; ++j) out[j] = j < n ? drafts[(size_t)b * K + j] : (j == n ? row_arg[b * R + n] : -1);
}

// Device buffers of the streaming head (at most 16 rows): the row's draft token, and per (row, vocabulary chunk) the
// partial statistics that lm_head_kernel leaves for accept_kernel.
struct HeadBufs {
    int32_t* row_x; float* hp_max; float* hp_sum; int32_t* hp_arg; float* hp_topv; int32_t* hp_topi; float* hp_lx;
};

// The streaming head: rows -> lm_head_kernel (every wave a vocabulary chunk) -> accept_kernel. Allocates nothing.
static int run_head_stream(Model* m, const uint16_t* h, const int32_t* drafts, const int32_t* draft_len, int B, int K,
                           int topk, float p, int mode, int32_t* accept_len, int32_t* out_tokens, float* logits_dbg,
                           const HeadBufs& hb, hipStream_t stream) {
    const int M = B * (K + 1);
    hipLaunchKernelGGL(head_rows_kernel, dim3((M + 255) / 256), dim3(256), 0, stream, drafts, draft_len, B, K,
                       m->d.vocab, hb.row_x, hb.hp_lx);
    const int ntiles = m->d.vocab / 16;
    const int tpw = (ntiles + 1023) / 1024;
    HeadArgs a{m->d.wlm, h, M, m->d.vocab, m->d.d_model, tpw, m->head_chunks, hb.row_x,
               hb.hp_max, hb.hp_sum, hb.hp_arg, hb.hp_topv, hb.hp_topi, hb.hp_lx, logits_dbg};
    dim3 grid((unsigned)((m->head_chunks + 3) / 4), 1u);         // at most 16 rows: one row tile
    hipLaunchKernelGGL(lm_head_kernel<1>, grid, dim3(256), 0, stream, a);
    AcceptArgs aa{hb.hp_max, hb.hp_sum, hb.hp_arg, hb.hp_topv, hb.hp_topi, hb.hp_lx, hb.row_x, drafts, draft_len,
                  K, m->head_chunks, topk, mode, p, accept_len, out_tokens};
    hipLaunchKernelGGL(accept_kernel, dim3(B), dim3(256), 0, stream, aa);
    LASER_HIP_CHECK(hipGetLastError());
    return LASER_OK;
}

int run_head(Model* m, const uint16_t* h, const int32_t* drafts, const int32_t* draft_len, int B, int K,
             int topk, float p, int mode, int32_t* accept_len, int32_t* out_tokens, float* logits_dbg,
             hipStream_t stream) {
    const int R = K + 1, M = B * R;
    if (M > kHeadStreamMaxRows) {
        hipLaunchKernelGGL(head_rows_kernel, dim3((M + 255) / 256), dim3(256), 0, stream, drafts, draft_len, B, K,
                           m->d.vocab, m->row_x, m->hp_lx);
        float* logits = logits_dbg;
        if (!logits) {                                   // workspace for max_rows x vocab logits, on first use
            if (!m->logits_ws) {
                const size_t bytes = (size_t)m->d.max_rows * m->d.vocab * sizeof(float);
                hipError_t e = hipMalloc((void**)&m->logits_ws, bytes);
                LASER_REQUIRE(e == hipSuccess, LASER_E_HIP, "hipMalloc of the %zu-byte logits workspace failed: %s", bytes,
                              hipGetErrorString(e));
            }
            logits = m->logits_ws;
        }
        if (M <= kHeadMidMaxRows && m->d.d_model % kGemmKStep == 0 && m->d.vocab % 16 == 0) {
            GemmMidArgs t{m->d.wlm, h, nullptr, M, m->d.vocab, m->d.d_model, logits, nullptr, nullptr};
            launch_gemm_mid<EPI_F32, false>(t, gemm_mid_plan(M, m->d.vocab, m->d.d_model, 1, false, 0), stream);
        } else {
            const int tiles_m = (M + GM_BM - 1) / GM_BM, tiles_n = (m->d.vocab + 127) / 128;
            GemmTileArgs t{m->d.wlm, h, nullptr, M, m->d.vocab, m->d.d_model, tiles_m, tiles_n, 1, logits, nullptr};
            hipLaunchKernelGGL((gemm_mfma_kernel<GEPI_F32, 128, false>), dim3(gemm_mfma_grid(tiles_m, tiles_n)), dim3(256), 0,
                               stream, t);
        }
        int32_t* row_ok = m->hp_arg;                     // per-row scratch: the streaming path's buffers are free here
        int32_t* row_arg = m->hp_arg + M;
        StatsArgs sa{logits, m->row_x, m->d.vocab, topk, mode, p, row_ok, row_arg};
        hipLaunchKernelGGL(head_stats_kernel, dim3(M), dim3(256), 0, stream, sa);
        hipLaunchKernelGGL(head_scan_kernel, dim3((B + 63) / 64), dim3(64), 0, stream, row_ok, row_arg, drafts, draft_len,
                           B, K, accept_len, out_tokens);
        LASER_HIP_CHECK(hipGetLastError());
        return LASER_OK;
    }
    HeadBufs hb{m->row_x, m->hp_max, m->hp_sum, m->hp_arg, m->hp_topv, m->hp_topi, m->hp_lx};
    return run_head_stream(m, h, drafts, draft_len, B, K, topk, p, mode, accept_len, out_tokens, logits_dbg, hb, stream);
}

// ---- the head without any allocation ------------------------------------------------------------------------
// The partial statistics live in a file-scope device array instead of the model handle's workspace. Each GPU holds
// its own copy of the array at its own address: the address is taken once per device with that device current.
constexpr int kStaticRows = kHeadStreamMaxRows;      // rows one call may verify
constexpr int kStaticChunks = 1024;                  // vocabulary chunks (laser_model_create never makes more)
struct HeadScratch {
    float hp_max[kStaticRows * kStaticChunks];
    float hp_sum[kStaticRows * kStaticChunks];
    int32_t hp_arg[kStaticRows * kStaticChunks];
    float hp_topv[kStaticRows * kStaticChunks * KT];
    int32_t hp_topi[kStaticRows * kStaticChunks * KT];
    float hp_lx[kStaticRows];
    int32_t row_x[kStaticRows];
};
static __device__ __align__(256) unsigned char scratch[sizeof(HeadScratch)];      // 1.19 MiB per GPU, for the life of the process

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kMaxDevices];             // device address of `scratch` on each GPU, once known

static int head_scratch(HeadScratch** out) {
    int dev = -1;
    LASER_HIP_CHECK(hipGetDevice(&dev));
    LASER_REQUIRE(dev >= 0 && dev < kMaxDevices, LASER_E_LIMIT, "device ordinal %d beyond %d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        LASER_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        LASER_REQUIRE(ptr != nullptr, LASER_E_HIP, "hipGetSymbolAddress returned no address for the head scratch");
        g_scratch_ptr[dev] = ptr;
    }
    *out = reinterpret_cast<HeadScratch*>(g_scratch_ptr[dev]);
    return LASER_OK;
}

int run_head_static(Model* m, const uint16_t* h, const int32_t* drafts, const int32_t* draft_len, int B, int K,
                    int topk, float p, int mode, int32_t* accept_len, int32_t* out_tokens, hipStream_t stream) {
    const int M = B * (K + 1);
    LASER_REQUIRE(M <= kStaticRows, LASER_E_LIMIT, "B*(K+1) = %d rows exceed the %d this entry point verifies per call", M, kStaticRows);
    LASER_REQUIRE(m->head_chunks <= kStaticChunks, LASER_E_LIMIT, "vocabulary of %d needs %d chunks, the static scratch holds %d",
                  m->d.vocab, m->head_chunks, kStaticChunks);
    HeadScratch* sc = nullptr;
    int rc = head_scratch(&sc);
    if (rc) return rc;
    // Nothing in the array has to start at zero: head_rows_kernel resets row_x and hp_lx for the call's rows, and
    // lm_head_kernel overwrites every (row, chunk) record that accept_kernel reads.
    HeadBufs hb{sc->row_x, sc->hp_max, sc->hp_sum, sc->hp_arg, sc->hp_topv, sc->hp_topi, sc->hp_lx};
    return run_head_stream(m, h, drafts, draft_len, B, K, topk, p, mode, accept_len, out_tokens, nullptr, hb, stream);
}

}  // namespace laser
