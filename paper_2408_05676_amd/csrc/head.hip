// Fused output head + acceptance (Sec. 3.4 Eq. 7-8; greedy Eq. 4; correction rule of Sec. 2.1). Logits are never
// stored (unless a debug buffer is passed): every kernel that produces them reduces them at once to per-(row,
// vocabulary chunk) partial statistics (head_part.h); accept_rows_kernel merges a row's chunks and ranks the row's
// candidates, and accept_scan_kernel walks the nodes of a sequence.
//
// Pass 1, by row count M = B*(K+1):
//   M <= 16   lm_head_kernel: every wavefront owns a contiguous chunk of the vocabulary, streams those rows of the
//             head matrix once through the matrix cores against all verified rows and keeps the running statistics
//             in registers (chunk = wavefront).
//   M <= 80   the weight-streaming kernel of gemm_mid.h with its head epilogue (chunk = workgroup, 64 or 128
//             vocabulary entries): the head matrix is read once.
//   more      the LDS-tiled matrix-core GEMM of gemm_mfma.h with its head epilogue (chunk = 128-column tile).
// Pass 2: a wavefront per row merges the per-chunk partials. The draft's rank is the number of partial-list entries
// ordered before it; if a chunk hides an entry that precedes the draft, that chunk already contributes
// >= LASER_MAX_TOPK >= k listed ones, so "rank < k" is exact. A thread per sequence then examines the nodes in order
// and emits accepted drafts plus the correction token.
#include <cmath>
#include <mutex>

#include "gemm_mfma.h"
#include "gemm_skinny.h"
#include "gemm_mid.h"
#include "state.h"

namespace laser {

int widen_copies(const uint16_t* const* src, const size_t* elems, int n, uint16_t** dst, hipStream_t stream);

constexpr int kHeadStreamMaxRows = 16;   // up to here lm_head_kernel; beyond, a GEMM with the head epilogue
constexpr int kHeadMidMaxRows = 80;      // up to here that GEMM streams the head matrix once; beyond, the tiled one

struct HeadArgs {
    const uint16_t* W; const uint16_t* H; int M, V, d, tiles_per_wave;
    HeadPart hp;
};

// One wavefront per sequence (lane i = node i): the candidates of every row. Node i of the pseudo-sequence (token
// tokens[b][i]) is a candidate of its parent's row (row parent + 1; row 0 is the pending token's): for a chain, node i
// of row i. Candidates of a row are stored next to each other, in pseudo-sequence order; nodes past n_nodes[b] and
// tokens outside the vocabulary are no candidates (node_cand = -1: never accepted).
__global__ __launch_bounds__(64) void head_cands_kernel(const int32_t* tokens, const int32_t* parent, const int32_t* n_nodes, int B, int K, int vocab,
                                                        int32_t* cand_beg, int32_t* cand_cnt, int32_t* cand_x, int32_t* node_cand, float* cand_lx) {
    __shared__ int prow[LASER_MAX_DRAFT + 1];          // parent row of node i, -1: no candidate
    __shared__ int cnt[LASER_MAX_DRAFT + 1], beg[LASER_MAX_DRAFT + 1];
    const int b = blockIdx.x, i = threadIdx.x, R = K + 1;
    int nn = n_nodes[b];
    nn = nn < 0 ? 0 : (nn > K ? K : nn);
    int x = -1, pr = -1;
    if (i < K) {
        x = tokens[(size_t)b * K + i];
        if (i < nn && x >= 0 && x < vocab) pr = tree_parent_of(parent, b, K, i, nn) + 1;
    }
    if (i < R) cnt[i] = 0;
    prow[i] = pr;
    __syncthreads();
    if (pr >= 0) atomicAdd(&cnt[pr], 1);
    __syncthreads();
    if (i == 0) {
        int off = b * K;
        for (int r = 0; r < R; ++r) { beg[r] = off; off += cnt[r]; }
    }
    __syncthreads();
    if (i < R) { cand_beg[(size_t)b * R + i] = beg[i]; cand_cnt[(size_t)b * R + i] = cnt[i]; }
    if (i < K) {
        int c = -1;
        if (pr >= 0) {
            int before_me = 0;                          // earlier nodes below the same row keep their order
            for (int j = 0; j < i; ++j) before_me += prow[j] == pr ? 1 : 0;
            c = beg[pr] + before_me;
            cand_x[c] = x;
            cand_lx[c] = -INFINITY;
        }
        node_cand[(size_t)b * K + i] = c;
    }
}

template <int MB>
__global__ __launch_bounds__(256) void lm_head_kernel(HeadArgs a) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 15, g = lane >> 4;
    const int chunk = blockIdx.x * 4 + wave;
    if (chunk >= a.hp.chunks) return;
    const int ntiles = a.V / 16;
    const int t0 = chunk * a.tiles_per_wave, t1 = min(ntiles, t0 + a.tiles_per_wave);
    const int row0 = blockIdx.y * MB * 16;

    RowStat st[MB];
    int cb[MB], cn[MB], x0[MB];           // the row's candidates; the first one's token is kept in a register
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        st[mb].init();
        const int row = row0 + mb * 16 + r;
        cb[mb] = row < a.M ? a.hp.cand_beg[row] : 0;
        cn[mb] = row < a.M ? a.hp.cand_cnt[row] : 0;
        x0[mb] = cn[mb] > 0 ? a.hp.cand_x[cb[mb]] : -1;
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
            for (int i = 0; i < 4; ++i) st[mb].add(acc[mb][i], n + i);
            auto pick = [&](int c) { return c == 0 ? acc[mb][0] : c == 1 ? acc[mb][1] : c == 2 ? acc[mb][2] : acc[mb][3]; };
            if (x0[mb] >= n && x0[mb] < n + 4) a.hp.cand_lx[cb[mb]] = pick(x0[mb] - n);
            for (int c = 1; c < cn[mb]; ++c) {                   // further children of a tree node
                const int x = a.hp.cand_x[cb[mb] + c];
                if (x >= n && x < n + 4) a.hp.cand_lx[cb[mb] + c] = pick(x - n);
            }
            const int row = row0 + mb * 16 + r;
            if (a.hp.logits_dbg && row < a.M)
                *reinterpret_cast<float4*>(a.hp.logits_dbg + (size_t)row * a.V + n) =
                    make_float4(acc[mb][0], acc[mb][1], acc[mb][2], acc[mb][3]);
        }
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        st[mb].merge_from_lane(16);
        st[mb].merge_from_lane(32);
        const int row = row0 + mb * 16 + r;
        if (g == 0 && row < a.M) st[mb].store(a.hp, row, chunk);
    }
}

struct AcceptArgs {
    const float* hp_max; const float* hp_sum; const int32_t* hp_arg; const float* hp_topv; const int32_t* hp_topi;
    const int32_t* cand_beg; const int32_t* cand_cnt; const int32_t* cand_x; const float* cand_lx; const int32_t* node_cand;
    const int32_t* tokens; const int32_t* parent; const int32_t* n_nodes;      // parent == NULL: a chain
    int M, B, K, chunks, topk, mode; float p;
    float* row_mx; float* row_sum; int32_t* row_arg; int32_t* cand_rank;       // between the two kernels
    int32_t* accept_len; int32_t* out_tokens; int32_t* accept_path;            // accept_path may be NULL
};

// Pass 2a, a wavefront per row: the row's chunks are merged (softmax statistics, arg-max) and every candidate of the
// row gets its rank, the number of vocabulary entries ahead of it. A chunk's list is read only when the chunk's
// largest entry is ahead of one of the candidates (otherwise nothing in the chunk is).
constexpr int kCandPass = 4;          // candidates ranked per pass over a row's chunks
__global__ __launch_bounds__(256) void accept_rows_kernel(AcceptArgs a) {
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (row >= a.M) return;
    const int cb = a.cand_beg[row], cn = a.cand_cnt[row];
    for (int c0 = 0; c0 < (cn > 0 ? cn : 1); c0 += kCandPass) {
        int x[kCandPass];
        float lx[kCandPass];
#pragma unroll
        for (int j = 0; j < kCandPass; ++j) {
            const bool have = c0 + j < cn;
            x[j] = have ? a.cand_x[cb + c0 + j] : -1;
            lx[j] = have ? a.cand_lx[cb + c0 + j] : -INFINITY;
        }
        float mx = -INFINITY, sum = 0.f;
        int arg = 0x7FFFFFFF, ahead[kCandPass] = {0, 0, 0, 0};
        for (int c = lane; c < a.chunks; c += 64) {
            const size_t o = (size_t)row * a.chunks + c;
            const float cm = a.hp_max[o], cs = a.hp_sum[o];
            const int ca = a.hp_arg[o];
            const float M = fmaxf(mx, cm);
            sum = sum * __expf(mx - M) + cs * __expf(cm - M);
            if (before(cm, ca, mx, arg)) arg = ca;
            mx = M;
            bool any = false;
#pragma unroll
            for (int j = 0; j < kCandPass; ++j) any |= x[j] >= 0 && ca != x[j] && before(cm, ca, lx[j], x[j]);
            if (any)
#pragma unroll
                for (int t = 0; t < KT; ++t) {
                    const float v = a.hp_topv[o * KT + t];
                    const int i = a.hp_topi[o * KT + t];
#pragma unroll
                    for (int j = 0; j < kCandPass; ++j) ahead[j] += (x[j] >= 0 && i != x[j] && before(v, i, lx[j], x[j])) ? 1 : 0;
                }
        }
        for (int off = 32; off > 0; off >>= 1) {
            const float omx = __shfl_xor(mx, off), osum = __shfl_xor(sum, off);
            const int oarg = __shfl_xor(arg, off);
#pragma unroll
            for (int j = 0; j < kCandPass; ++j) ahead[j] += __shfl_xor(ahead[j], off);
            const float M = fmaxf(mx, omx);
            if (M != -INFINITY) sum = sum * __expf(mx - M) + osum * __expf(omx - M);
            if (before(omx, oarg, mx, arg)) arg = oarg;
            mx = M;
        }
        if (lane == 0) {
            if (c0 == 0) { a.row_mx[row] = mx; a.row_sum[row] = sum; a.row_arg[row] = arg; }
#pragma unroll
            for (int j = 0; j < kCandPass; ++j)
                if (c0 + j < cn) a.cand_rank[cb + c0 + j] = ahead[j];
        }
    }
}

// Pass 2b, a thread per sequence: the nodes are examined in pseudo-sequence order (a node is verified iff its parent
// is and its token passes the rule against its parent's row), the deepest verified node -- the first one among
// equally deep -- ends the accepted branch, and the branch's tokens plus the arg-max of its last row are emitted
// (Sec. 3.4; Sec. 2.1 for the correction token). For a chain this is the longest accepted prefix.
__global__ __launch_bounds__(64) void accept_scan_kernel(AcceptArgs a) {
    const int b = blockIdx.x * 64 + threadIdx.x, R = a.K + 1;
    if (b >= a.B) return;
    int nn = a.n_nodes[b];
    nn = nn < 0 ? 0 : (nn > a.K ? a.K : nn);
    unsigned long long ver = 0;                           // bit i: node i is verified
    unsigned long long dpk[(LASER_MAX_DRAFT + 8) / 8] = {};   // depth of node i, a byte each
    int best = -1, best_depth = 0;
    for (int i = 0; i < nn; ++i) {
        const int par = tree_parent_of(a.parent, b, a.K, i, nn);
        const int c = a.node_cand[(size_t)b * a.K + i];
        bool ok = c >= 0 && (par < 0 || ((ver >> par) & 1ull));
        if (ok) {
            const int prow = b * R + par + 1, rank = a.cand_rank[c];
            const float q = __expf(a.cand_lx[c] - a.row_mx[prow]) / a.row_sum[prow];
            const bool in_k = rank < a.topk, above = q > a.p, top1 = rank == 0;
            ok = a.mode == LASER_MODE_RV ? (in_k && above)
               : a.mode == LASER_MODE_RV_OR_TOP1 ? (top1 || (in_k && above))
               : a.mode == LASER_MODE_TOPK_ONLY ? in_k : (top1 || above);
        }
        if (ok) {
            ver |= 1ull << i;
            int d = 1;
            if (par >= 0) {
                unsigned long long w = 0;
#pragma unroll
                for (int s = 0; s < (LASER_MAX_DRAFT + 8) / 8; ++s) w = s == (par >> 3) ? dpk[s] : w;
                d = (int)((w >> ((par & 7) * 8)) & 0xFF) + 1;
            }
#pragma unroll
            for (int s = 0; s < (LASER_MAX_DRAFT + 8) / 8; ++s)
                if (s == (i >> 3)) dpk[s] |= (unsigned long long)d << ((i & 7) * 8);
            if (d > best_depth) { best = i; best_depth = d; }
        }
    }
    a.accept_len[b] = best_depth;
    int32_t* out = a.out_tokens + (size_t)b * R;
    for (int j = best_depth + 1; j < R; ++j) out[j] = -1;
    out[best_depth] = a.row_arg[b * R + best + 1];
    for (int i = best, j = best_depth - 1; j >= 0; --j) {
        out[j] = a.tokens[(size_t)b * a.K + i];
        if (a.accept_path) a.accept_path[(size_t)b * a.K + j] = i;
        i = tree_parent_of(a.parent, b, a.K, i, nn);
    }
    if (a.accept_path)
        for (int j = best_depth; j < a.K; ++j) a.accept_path[(size_t)b * a.K + j] = -1;
}

// Device buffers of the head: the rows' candidate lists, and per (row, vocabulary chunk) the partial statistics that
// pass 1 leaves for the acceptance kernels, and the per-row results between those two.
struct HeadBufs {
    int32_t* cand_beg; int32_t* cand_cnt; int32_t* cand_x; int32_t* node_cand; float* cand_lx;
    float* hp_max; float* hp_sum; int32_t* hp_arg; float* hp_topv; int32_t* hp_topi;
    float* row_mx; float* row_sum; int32_t* row_arg; int32_t* cand_rank;
};

// Chunks per row of the pass-1 kernel a row count takes (the partial arrays must hold rows x this many records).
static int head_chunks_for(const Model* m, int M) {
    if (M <= kHeadStreamMaxRows) return m->head_chunks;
    if (M <= kHeadMidMaxRows && m->d.d_model % kGemmKStep == 0)
        return (m->d.vocab / 16 + 3) / 4;                          // at most: the 4-wave form has the most workgroups
    return (m->d.vocab + 127) / 128;
}
int head_chunks_cap(const Model* m) {
    return std::max(m->head_chunks, std::max(head_chunks_for(m, kHeadMidMaxRows), head_chunks_for(m, kHeadMidMaxRows + 1)));
}

// candidates -> pass 1 -> acceptance. Allocates nothing. tokens / parent / n_nodes: the drafts as a pseudo-sequence
// (parent == NULL: a chain, n_nodes = draft_len).
static int run_head_bufs(Model* m, const uint16_t* h, const int32_t* tokens, const int32_t* parent, const int32_t* n_nodes, int B, int K,
                         int topk, float p, int mode, int32_t* accept_len, int32_t* out_tokens, int32_t* accept_path, float* logits_dbg,
                         const HeadBufs& hb, hipStream_t stream) {
    const int M = B * (K + 1), V = m->d.vocab, dm = m->d.d_model;
    hipLaunchKernelGGL(head_cands_kernel, dim3(B), dim3(64), 0, stream, tokens, parent, n_nodes, B, K, V,
                       hb.cand_beg, hb.cand_cnt, hb.cand_x, hb.node_cand, hb.cand_lx);
    HeadPart hp{hb.cand_beg, hb.cand_cnt, hb.cand_x, hb.cand_lx, hb.hp_max, hb.hp_sum, hb.hp_arg, hb.hp_topv, hb.hp_topi, 0, topk, logits_dbg};
    if (M <= kHeadStreamMaxRows) {
        const int ntiles = V / 16;
        const int tpw = (ntiles + 1023) / 1024;
        hp.chunks = m->head_chunks;
        HeadArgs a{m->d.wlm, h, M, V, dm, tpw, hp};
        dim3 grid((unsigned)((m->head_chunks + 3) / 4), 1u);         // at most 16 rows: one row tile
        hipLaunchKernelGGL(lm_head_kernel<1>, grid, dim3(256), 0, stream, a);
    } else if (M <= kHeadMidMaxRows && dm % kGemmKStep == 0) {
        const GemmMidPlan pl = gemm_mid_plan(M, V, dm, 1, false, 0);
        hp.chunks = (V / 16 + pl.NW - 1) / pl.NW;                     // = workgroups of the launch
        GemmMidArgs t{m->d.wlm, h, nullptr, M, V, dm, nullptr, nullptr, nullptr, hp};
        launch_gemm_mid<EPI_HEAD, false>(t, pl, stream);
    } else {
        const int tiles_m = (M + GM_BM - 1) / GM_BM, tiles_n = (V + 127) / 128;
        hp.chunks = tiles_n;
        if (m->f16_copies && !m->wlm16) {          // first many-row head: widen the head matrix to fp16 once
            const uint16_t* src[1] = {m->d.wlm};
            const size_t n[1] = {(size_t)V * dm};
            const int rc = widen_copies(src, n, 1, &m->wlm16, stream);
            if (rc) return rc;
        }
        GemmTileArgs t{m->wlm16 ? m->wlm16 : m->d.wlm, h, nullptr, M, V, dm, tiles_m, tiles_n, 1, nullptr, nullptr, hp};
        const dim3 grid(gemm_mfma_grid(tiles_m, tiles_n));
        if (m->wlm16) hipLaunchKernelGGL((gemm_mfma_kernel<GEPI_HEAD, 128, false, true>), grid, dim3(256), 0, stream, t);
        else hipLaunchKernelGGL((gemm_mfma_kernel<GEPI_HEAD, 128, false, false>), grid, dim3(256), 0, stream, t);
    }
    AcceptArgs aa{hb.hp_max, hb.hp_sum, hb.hp_arg, hb.hp_topv, hb.hp_topi, hb.cand_beg, hb.cand_cnt, hb.cand_x, hb.cand_lx, hb.node_cand,
                  tokens, parent, n_nodes, M, B, K, hp.chunks, topk, mode, p, hb.row_mx, hb.row_sum, hb.row_arg, hb.cand_rank,
                  accept_len, out_tokens, accept_path};
    hipLaunchKernelGGL(accept_rows_kernel, dim3((M + 3) / 4), dim3(256), 0, stream, aa);
    hipLaunchKernelGGL(accept_scan_kernel, dim3((B + 63) / 64), dim3(64), 0, stream, aa);
    LASER_HIP_CHECK(hipGetLastError());
    return LASER_OK;
}

int run_head(Model* m, const uint16_t* h, const int32_t* tokens, const int32_t* parent, const int32_t* n_nodes, int B, int K,
             int topk, float p, int mode, int32_t* accept_len, int32_t* out_tokens, int32_t* accept_path, float* logits_dbg,
             hipStream_t stream) {
    HeadBufs hb{m->cand_beg, m->cand_cnt, m->cand_x, m->node_cand, m->cand_lx, m->hp_max, m->hp_sum, m->hp_arg, m->hp_topv, m->hp_topi,
                m->row_mx, m->row_sum, m->row_arg, m->cand_rank};
    return run_head_bufs(m, h, tokens, parent, n_nodes, B, K, topk, p, mode, accept_len, out_tokens, accept_path, logits_dbg, hb, stream);
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
    int32_t cand_beg[kStaticRows], cand_cnt[kStaticRows], cand_x[kStaticRows], node_cand[kStaticRows];
    float cand_lx[kStaticRows];
    float row_mx[kStaticRows], row_sum[kStaticRows];
    int32_t row_arg[kStaticRows], cand_rank[kStaticRows];
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
    // Nothing in the array has to start at zero: head_cands_kernel rewrites the candidate lists of the call's rows, and
    // lm_head_kernel overwrites every (row, chunk) record that the acceptance kernels read.
    HeadBufs hb{sc->cand_beg, sc->cand_cnt, sc->cand_x, sc->node_cand, sc->cand_lx, sc->hp_max, sc->hp_sum, sc->hp_arg, sc->hp_topv, sc->hp_topi,
                sc->row_mx, sc->row_sum, sc->row_arg, sc->cand_rank};
    return run_head_bufs(m, h, drafts, nullptr, draft_len, B, K, topk, p, mode, accept_len, out_tokens, nullptr, nullptr, hb, stream);
}

}  // namespace laser
