// The generation loop (Sec. 3.1 overview; Sec. 2.1: draft, verify, keep the accepted tokens, repeat until the text
// is complete): retrieve drafts -> verify -> bookkeeping -> commit, step after step on one stream,
// for a whole batch, until every sequence has emitted max_new_tokens tokens or its end-of-sequence token. The host
// enqueues the steps and never reads device state on the step path; once every `check_every` steps it looks at a
// device counter of finished sequences (one stream synchronisation) to stop early. A finished sequence stays in
// the batch (its rows are computed and dropped): its commit adds nothing and its outputs are not appended.
#include <algorithm>
#include <vector>

#include "state.h"

namespace laser {

struct GenArgs {
    const int32_t* accept_len; const int32_t* out_tokens; const int32_t* draft_len;
    int32_t* accept_eff;                 // out: tokens this step really keeps - 1; -1 for a sequence that was finished before it
    int32_t* ctx_tail; int32_t* pending; // in/out
    int32_t* gen_tokens; int32_t* gen_len; int32_t* counters; int32_t* done; int32_t* n_done;
    int B, K, n_max, max_new, eos;
};

// One thread per sequence: what the step's emitted tokens (accepted drafts + the correction / bonus token) mean for
// the text -- cut at the end-of-sequence token and at max_new tokens --, the context tail and the pending token.
__global__ void gen_bookkeep_kernel(GenArgs a) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= a.B) return;
    if (a.done[b]) { a.accept_eff[b] = -1; return; }
    int acc = a.accept_len[b];
    acc = acc < 0 ? 0 : (acc > a.K ? a.K : acc);
    const int32_t* out = a.out_tokens + (size_t)b * (a.K + 1);
    const int have = a.gen_len[b];
    int n_emit = min(acc + 1, a.max_new - have);
    bool finished = false;
    for (int j = 0; j < n_emit; ++j)
        if (out[j] == a.eos) { n_emit = j + 1; finished = true; break; }
    for (int j = 0; j < n_emit; ++j) a.gen_tokens[(size_t)b * a.max_new + have + j] = out[j];
    a.gen_len[b] = have + n_emit;
    int32_t* tail = a.ctx_tail + (size_t)b * a.n_max;
    int32_t tmp[LASER_MAX_NGRAM];
    for (int i = 0; i < a.n_max; ++i) {
        const int src = i + n_emit;                   // index into old tail ++ emitted
        tmp[i] = src < a.n_max ? tail[src] : out[src - a.n_max];
    }
    for (int i = 0; i < a.n_max; ++i) tail[i] = tmp[i];
    a.pending[b] = out[n_emit - 1];
    a.accept_eff[b] = n_emit - 1;
    int32_t* c = a.counters + (size_t)b * 4;
    c[0] += 1;                                        // steps
    c[1] += min(max(a.draft_len[b], 0), a.K);         // draft tokens offered
    c[2] += n_emit - 1;                               // draft tokens kept
    c[3] += acc;                                      // draft tokens accepted by the rule (before the cut)
    if (finished || have + n_emit >= a.max_new) {
        a.done[b] = 1;
        atomicAdd(a.n_done, 1);
    }
}

__global__ void gen_fill_kernel(int32_t* p, int32_t v, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

}  // namespace laser

using namespace laser;

extern "C" int laser_generate(laser_model* mh, laser_kv* kh, const laser_pool* pool, const int32_t* seq_ids, const int64_t* keys,
                              int32_t* ctx_tail, int32_t* pending, int32_t* own_tokens, int32_t* own_len, int B,
                              const laser_generate_opts* opts, int32_t* gen_tokens, int32_t* gen_len, int32_t* counters,
                              int* steps_run, float* retrieve_ms, void* stream_) {
    Model* m = reinterpret_cast<Model*>(mh);
    KV* kv = reinterpret_cast<KV*>(kh);
    hipStream_t stream = (hipStream_t)stream_;
    LASER_REQUIRE(m && kv && opts && steps_run, LASER_E_INVALID_ARG, "NULL argument");
    const laser_generate_opts& o = *opts;
    LASER_REQUIRE(B >= 0 && B <= m->d.max_batch && B <= kv->d.max_seqs, LASER_E_INVALID_ARG, "B %d outside 0..max_batch", B);
    LASER_REQUIRE(o.K >= 0 && o.K <= (o.tree ? LASER_MAX_TREE : LASER_MAX_DRAFT), LASER_E_INVALID_ARG, "K %d out of range", o.K);
    LASER_REQUIRE(o.n_max >= 1 && o.n_max <= LASER_MAX_NGRAM && o.n_min >= 1 && o.n_min <= o.n_max, LASER_E_INVALID_ARG, "bad n_min / n_max");
    LASER_REQUIRE(o.max_new_tokens >= 1 && o.check_every >= 1, LASER_E_INVALID_ARG, "max_new_tokens and check_every must be >= 1");
    LASER_REQUIRE(!(o.tree && o.own_cap > 0), LASER_E_INVALID_ARG, "the temporary branch is searched with chain drafts only");
    *steps_run = 0;
    if (retrieve_ms) *retrieve_ms = 0.f;
    if (B == 0) return LASER_OK;
    LASER_REQUIRE(seq_ids && ctx_tail && pending && gen_tokens && gen_len && counters, LASER_E_INVALID_ARG, "NULL buffer");
    LASER_REQUIRE(!pool || keys, LASER_E_INVALID_ARG, "keys is NULL");
    LASER_REQUIRE(o.own_cap <= 0 || (own_tokens && own_len && pool), LASER_E_INVALID_ARG, "the temporary branch needs own_tokens, own_len and a pool");
    const int K = pool ? o.K : 0, R = K + 1;
    // capacity: a sequence grows by at most max_new_tokens tokens in total, and a step writes R rows behind that
    std::vector<int> ub0(B);
    for (int b = 0; b < B; ++b) {
        const int s = seq_ids[b];
        LASER_REQUIRE(s >= 0 && s < kv->d.max_seqs, LASER_E_INVALID_ARG, "sequence slot %d out of range", s);
        ub0[b] = kv->h_len_ub[s];
        LASER_REQUIRE(ub0[b] + o.max_new_tokens + R <= kv->h_npages[s] * kPageSize, LASER_E_OOM_PAGES,
                      "slot %d: length bound %d + %d new tokens + %d rows exceeds the %d tokens reserved", s, ub0[b], o.max_new_tokens, R,
                      kv->h_npages[s] * kPageSize);
    }
    // per-call device state
    int32_t* ws = nullptr;
    const size_t n_ws = (size_t)B * (3 * (size_t)K + (size_t)R + 8) + 16;
    LASER_HIP_CHECK(hipMalloc((void**)&ws, n_ws * 4 + (size_t)B * 8 + 8));
    int32_t* drafts = ws; int32_t* parent = drafts + (size_t)B * K; int32_t* path = parent + (size_t)B * K;
    int32_t* out_tokens = path + (size_t)B * K;
    int32_t* draft_len = out_tokens + (size_t)B * R; int32_t* match_n = draft_len + B; int32_t* accept_len = match_n + B;
    int32_t* accept_eff = accept_len + B; int32_t* done = accept_eff + B; int32_t* n_done = done + B;
    int64_t* pool_index = reinterpret_cast<int64_t*>(ws + ((n_ws + 1) & ~(size_t)1));
    int* h_done = nullptr;
    std::vector<hipEvent_t> ev;
    int rc = LASER_OK;
    auto cleanup = [&](int code) {
        (void)hipStreamSynchronize(stream);
        (void)hipFree(ws);
        if (h_done) (void)hipHostFree(h_done);
        for (hipEvent_t e : ev) (void)hipEventDestroy(e);
        return code;
    };
#define G_TRY(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) { set_error("%s: %s", #expr, hipGetErrorString(e_)); return cleanup(LASER_E_HIP); } } while (0)
#define G_RC(expr) do { if ((rc = (expr)) != LASER_OK) return cleanup(rc); } while (0)
    G_TRY(hipHostMalloc((void**)&h_done, sizeof(int)));
    G_TRY(hipMemsetAsync(ws, 0, n_ws * 4 + (size_t)B * 8 + 8, stream));       // no drafts, nothing done
    G_TRY(hipMemsetAsync(gen_len, 0, (size_t)B * 4, stream));
    G_TRY(hipMemsetAsync(counters, 0, (size_t)B * 16, stream));
    hipLaunchKernelGGL(gen_fill_kernel, dim3((B * o.max_new_tokens + 255) / 256), dim3(256), 0, stream, gen_tokens, -1, B * o.max_new_tokens);

    GenArgs g{accept_len, out_tokens, draft_len, accept_eff, ctx_tail, pending, gen_tokens, gen_len, counters, done, n_done,
              B, K, o.n_max, o.max_new_tokens, o.eos_token};
    int steps = 0;
    for (; steps < o.max_new_tokens; ++steps) {
        for (int b = 0; b < B; ++b)       // a true bound: a step adds at most R tokens, the whole call at most max_new_tokens
            kv->h_len_ub[seq_ids[b]] = ub0[b] + std::min(steps * R, o.max_new_tokens);
        if (pool && K > 0) {
            if (retrieve_ms) {
                hipEvent_t e0, e1;
                G_TRY(hipEventCreate(&e0)); ev.push_back(e0);
                G_TRY(hipEventCreate(&e1)); ev.push_back(e1);
                G_TRY(hipEventRecord(e0, stream));
            }
            if (o.tree)
                G_RC(laser_retrieve_tree(pool, keys, ctx_tail, B, o.n_min, o.n_max, K, o.min_tokens, drafts, parent, nullptr, draft_len, match_n, stream));
            else if (o.own_cap > 0)
                G_RC(laser_retrieve_drafts_temp(pool, keys, ctx_tail, own_tokens, own_len, o.own_cap, B, o.n_min, o.n_max, K, o.min_tokens,
                                                drafts, draft_len, match_n, pool_index, stream));
            else
                G_RC(laser_retrieve_drafts(pool, keys, ctx_tail, B, o.n_min, o.n_max, K, o.min_tokens, drafts, draft_len, match_n, pool_index, stream));
            if (retrieve_ms) G_TRY(hipEventRecord(ev.back(), stream));
        }
        if (o.tree && K > 0)
            G_RC(laser_verify_tree(mh, kh, seq_ids, pending, drafts, parent, draft_len, B, K, o.topk, o.p, o.mode, accept_len, out_tokens, path,
                                   nullptr, stream));
        else
            G_RC(laser_verify_step(mh, kh, seq_ids, pending, drafts, draft_len, B, K, o.topk, o.p, o.mode, accept_len, out_tokens, nullptr, stream));
        hipLaunchKernelGGL(gen_bookkeep_kernel, dim3((B + 63) / 64), dim3(64), 0, stream, g);
        if (o.own_cap > 0)
            G_RC(laser_own_text_append(own_tokens, own_len, o.own_cap, out_tokens, accept_eff, B, K, stream));
        if (o.tree && K > 0) G_RC(laser_kv_commit_tree(kh, seq_ids, accept_eff, path, B, K, stream));
        else G_RC(laser_kv_commit(kh, seq_ids, accept_eff, B, stream));
        if ((steps + 1) % o.check_every == 0) {
            G_TRY(hipMemcpyAsync(h_done, n_done, sizeof(int), hipMemcpyDeviceToHost, stream));
            G_TRY(hipStreamSynchronize(stream));
            if (*h_done >= B) { ++steps; break; }
        }
    }
    G_TRY(hipStreamSynchronize(stream));
    for (int b = 0; b < B; ++b) kv->h_len_ub[seq_ids[b]] = ub0[b] + std::min(steps * R, o.max_new_tokens);
    *steps_run = steps;
    if (retrieve_ms) {
        double tot = 0.0;
        for (size_t i = 0; i + 1 < ev.size(); i += 2) {
            float ms = 0.f;
            G_TRY(hipEventElapsedTime(&ms, ev[i], ev[i + 1]));
            tot += ms;
        }
        *retrieve_ms = (float)tot;
    }
#undef G_TRY
#undef G_RC
    return cleanup(LASER_OK);
}
