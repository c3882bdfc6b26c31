// Retrieval pool: host-side construction of the regrouped pool and its suffix index, and the
// per-context lookup + frequency-greedy chain kernel (Sec. 3.2 pool construction, Sec. 3.3 Eq. 5).
//
// Index layout (all device resident, immutable after the build):
//   P[N]        int32   tokens, sub-pools laid out by ascending key
//   seq_end[N]  uint32  per position: one past the last position of its sequence
//   sa[Ne]      uint32  every position that has an in-sequence successor, sorted inside its
//                       sub-pool by the text read backwards from it (P[e], P[e-1], ... up to n_max
//                       tokens, "before the sequence start" ordering first), then by position.
//                       All occurrences of any n-gram (n <= n_max) are therefore one contiguous run of
//                       sa. Only the runs of n_max-grams are position-ascending: inside the run of a shorter
//                       n-gram the order is set by the tokens further back first, so the smallest position
//                       of a run has to be searched for (the lookup takes an explicit minimum).
//   table[cap]  16 B    open addressing (linear probing, load <= 0.5): (key, n, n-gram) -> run in sa
// A lookup hashes (key, n, suffix), probes, and confirms a hit by comparing key, n and the actual
// tokens at the run's first occurrence, so hash collisions cannot produce a false match.
#include <algorithm>
#include <cstring>
#include <numeric>
#include <thread>
#include <vector>

#include "common.h"

namespace laser {

struct Pool {
    int32_t* P = nullptr;
    uint32_t* seq_end = nullptr;
    uint32_t* sa = nullptr;
    IndexEntry* table = nullptr;
    uint64_t cap_mask = 0;
    int64_t n_tokens = 0, n_keys = 0, n_entries = 0, n_sa = 0, device_bytes = 0;
    int n_max = 0;
};

// ------------------------------------------------------------------------------------ kernel
constexpr int kCand = 512;         // occurrences a wave keeps in LDS (more: streamed from the index, re-checked against the chain)
constexpr int kVote = 512;         // vote-table slots (power of two; wider votes are partitioned)
constexpr int kEmptyTok = -1;
constexpr int kOwnMax = LASER_MAX_OWN_TEXT;   // tokens of a sequence's own text (temporary branch) a lookup can take

__device__ inline uint32_t fmix32(uint32_t h) {   // bijective 32-bit mixer
    h ^= h >> 16; h *= 0x85EBCA6Bu; h ^= h >> 13; h *= 0xC2B2AE35u; h ^= h >> 16;
    return h;
}

struct RetrieveArgs {
    const int32_t* P; const uint32_t* seq_end; const uint32_t* sa; const IndexEntry* table;
    uint64_t cap_mask;
    const int64_t* keys; const int32_t* ctx_tail;
    int B, n_min, n_max, K, min_tokens;
    int32_t* drafts; int32_t* draft_len; int32_t* match_n; int64_t* pool_index;
    // temporary branch (Sec. 3.2): the sequence's own text, searched as one more sequence of its key's sub-pool,
    // placed after the pool's sequences; NULL = none
    const int32_t* own; const int32_t* own_len; int own_cap;
};

// One wavefront (= one workgroup of 64 lanes) per context. OWN: with the temporary branch. Occurrences in the own
// text are found by a scan of it (it is at most kOwnMax tokens and the wave has it in L2 anyway), always kept
// in LDS (own_cand, position-ascending) and take part in every vote and filter next to the pool's.
template <bool OWN>
__global__ __launch_bounds__(64) void retrieve_kernel(RetrieveArgs a) {
    __shared__ uint32_t cand[kCand];
    // Beside each occurrence kept in LDS: the end of its sequence, and the successor token the current vote read for
    // it (-1: none). The filter that follows a vote then needs no memory round trip at all, the vote one instead of
    // two -- the lookup is a chain of dependent round trips, and these were three of the four per chain step.
    __shared__ uint32_t cand_end[kCand];
    __shared__ int cand_tok[kCand];
    __shared__ uint32_t own_cand[OWN ? kOwnMax : 1];
    __shared__ int vote_tok[kVote];
    __shared__ int vote_cnt[kVote];
    __shared__ int chain[LASER_MAX_DRAFT + 1];
    __shared__ int best_chain[LASER_MAX_DRAFT + 1];
    __shared__ int sh_distinct;

    const int b = blockIdx.x;
    const int lane = threadIdx.x;
    const int64_t key = a.keys[b];
    const int32_t* tail = a.ctx_tail + (size_t)b * a.n_max;

    int valid = 0;
    while (valid < a.n_max && tail[a.n_max - 1 - valid] >= 0) ++valid;
    const int32_t* own = OWN ? a.own + (size_t)b * a.own_cap : nullptr;
    const uint32_t own_len = OWN ? (uint32_t)min(max(a.own_len[b], 0), a.own_cap) : 0u;

    int best_len = 0, best_n = 0;
    long long best_idx = -1;
    int res_len = 0, res_n = 0;
    long long res_idx = -1;
    bool done = false;

    const int n_hi = valid < a.n_max ? valid : a.n_max;
    for (int n = n_hi; n >= a.n_min && !done && a.K > 0; --n) {
        // ---- index probe (every lane does the same probe; addresses are uniform) ----
        const int32_t* w = tail + (a.n_max - n);
        uint64_t slot = ngram_hash(key, n, w) & a.cap_mask;
        uint32_t start = 0, count = 0;
        for (;;) {
            IndexEntry e = a.table[slot];
            if (e.count_n == 0) break;
            if (e.key == key && (int)(e.count_n >> 28) == n) {
                uint32_t e0 = a.sa[e.start];
                bool same = true;
                for (int i = 0; i < n; ++i) same = same && (a.P[e0 - (n - 1) + i] == w[i]);
                if (same) { start = e.start; count = e.count_n & 0x0FFFFFFFu; break; }
            }
            slot = (slot + 1) & a.cap_mask;
        }
        // ---- occurrences in the own text: positions e with own[e-n+1..e] == w and a successor e+1 < own_len ----
        uint32_t mo = 0;
        if constexpr (OWN) {
            for (uint32_t e0 = (uint32_t)(n - 1); e0 + 1 < own_len; e0 += 64) {
                const uint32_t e = e0 + lane;
                bool hit = e + 1 < own_len;
                for (int i = 0; i < n && hit; ++i) hit = own[e - (n - 1) + i] == w[i];
                const uint64_t mask = __ballot(hit);
                if (hit) own_cand[mo + __popcll(mask & ((1ull << lane) - 1ull))] = e;
                mo += __popcll(mask);
            }
            __syncthreads();
        }
        if (count == 0 && mo == 0) continue;

        // ---- frequency-greedy chain over the occurrences sa[start .. start+count) ----
        // Survivors are either materialised in LDS (m <= kCand) or, while there are too many,
        // re-derived from the run by re-checking the chain so far.
        bool in_lds = count <= (uint32_t)kCand;
        uint32_t m = count;
        if (in_lds)
            for (uint32_t i = lane; i < count; i += 64) {
                const uint32_t e = a.sa[start + i];
                cand[i] = e;
                cand_end[i] = a.seq_end[e];
            }
        __syncthreads();

        int len = 0;
        for (int j = 1; j <= a.K; ++j) {
            int win_tok = -1, win_cnt = 0;
            // The table is only as large as this vote can need (4 slots per voter, 64..kVote): clearing and scanning
            // 1024 slots with one wave cost more than the votes of the few dozen occurrences a typical lookup has.
            const uint32_t voters = (in_lds ? m : count) + mo;
            int vsz = 64;
            while (vsz < kVote && (uint32_t)vsz < 4u * voters) vsz *= 2;
            const int vfill = vsz / 4 * 3;             // distinct tokens beyond which a vote pass is split
            // The vote may need several passes when too many distinct successors show up.
            for (uint32_t nparts = 1;; nparts *= 2) {
                win_tok = -1; win_cnt = 0;
                bool overflow = false;
                for (uint32_t part = 0; part < nparts && !overflow; ++part) {
                    for (int i = lane; i < vsz; i += 64) { vote_tok[i] = kEmptyTok; vote_cnt[i] = 0; }
                    if (lane == 0) sh_distinct = 0;
                    __syncthreads();
                    const uint32_t total_pool = in_lds ? m : count;
                    const uint32_t total = total_pool + mo;
                    for (uint32_t i0 = 0; i0 < total; i0 += 64) {
                        uint32_t i = i0 + lane;
                        if (i < total) {
                            bool ok;
                            int tok = 0;
                            if (i < total_pool) {
                                uint32_t e = in_lds ? cand[i] : a.sa[start + i];
                                ok = (e + (uint32_t)j) < (in_lds ? cand_end[i] : a.seq_end[e]);
                                if (ok && !in_lds)
                                    for (int c = 1; c < j; ++c) ok = ok && (a.P[e + c] == chain[c - 1]);
                                if (ok) tok = a.P[e + j];
                                if (in_lds) cand_tok[i] = ok ? tok : -1;
                            } else {
                                const uint32_t e = own_cand[OWN ? i - total_pool : 0];
                                ok = e + (uint32_t)j < own_len;
                                if (ok) tok = own[e + j];
                            }
                            if (ok) {
                                uint32_t hh = fmix32((uint32_t)tok);
                                if (nparts == 1 || (hh / kVote) % nparts == part) {
                                    uint32_t s = hh & (vsz - 1);
                                    for (int probe = 0; probe < vsz; ++probe) {
                                        int cur = vote_tok[s];
                                        if (cur == kEmptyTok) {
                                            int prev = atomicCAS(&vote_tok[s], kEmptyTok, tok);
                                            if (prev == kEmptyTok) { atomicAdd(&sh_distinct, 1); cur = tok; }
                                            else cur = prev;
                                        }
                                        if (cur == tok) { atomicAdd(&vote_cnt[s], 1); break; }
                                        s = (s + 1) & (vsz - 1);
                                    }
                                }
                            }
                        }
                        // stop feeding a table that is getting too full; the pass will be split
                        if ((i0 & 1023u) == 960u) {
                            __syncthreads();
                            if (sh_distinct > vfill) break;
                        }
                    }
                    __syncthreads();
                    overflow = sh_distinct > vfill;
                    __syncthreads();               // everyone has read the counter before it is reset
                    if (overflow) break;
                    // best of this part: larger count, then smaller token id
                    int bt = -1, bc = 0;
                    for (int i = lane; i < vsz; i += 64) {
                        int c = vote_cnt[i], t = vote_tok[i];
                        if (c > bc || (c == bc && c > 0 && t < bt)) { bc = c; bt = t; }
                    }
                    for (int off = 32; off > 0; off >>= 1) {
                        int oc = __shfl_xor(bc, off), ot = __shfl_xor(bt, off);
                        if (oc > bc || (oc == bc && oc > 0 && ot < bt)) { bc = oc; bt = ot; }
                    }
                    if (bc > win_cnt || (bc == win_cnt && bc > 0 && bt < win_tok)) { win_cnt = bc; win_tok = bt; }
                    __syncthreads();
                }
                if (!overflow) break;
            }
            if (win_cnt == 0) break;       // no survivor has a successor left
            if (lane == 0) chain[j - 1] = win_tok;
            len = j;
            // ---- keep the occurrences that agree with the winner ----
            if (in_lds) {
                uint32_t out = 0;
                for (uint32_t i0 = 0; i0 < m; i0 += 64) {
                    uint32_t i = i0 + lane;
                    uint32_t e = 0, end = 0; bool keep = false;
                    if (i < m) {
                        e = cand[i];
                        end = cand_end[i];
                        keep = cand_tok[i] == win_tok;     // what the vote just read for this occurrence (tokens are >= 0)
                    }
                    uint64_t mask = __ballot(keep);
                    uint32_t pos = out + __popcll(mask & ((1ull << lane) - 1ull));
                    __syncthreads();               // all reads of this chunk precede the writes
                    if (keep) { cand[pos] = e; cand_end[pos] = end; }   // pos <= i: never overtakes unread entries
                    out += __popcll(mask);
                }
                m = out;
                __syncthreads();
            } else {
                __syncthreads();
                if ((uint32_t)win_cnt <= (uint32_t)kCand) {   // few enough now: materialise
                    uint32_t out = 0;
                    for (uint32_t i0 = 0; i0 < count; i0 += 64) {
                        uint32_t i = i0 + lane;
                        uint32_t e = 0, end = 0; bool keep = false;
                        if (i < count) {
                            e = a.sa[start + i];
                            end = a.seq_end[e];
                            keep = (e + (uint32_t)j) < end;
                            for (int c = 1; c <= j && keep; ++c) keep = (a.P[e + c] == chain[c - 1]);
                        }
                        uint64_t mask = __ballot(keep);
                        uint32_t pos = out + __popcll(mask & ((1ull << lane) - 1ull));
                        if (keep) { cand[pos] = e; cand_end[pos] = end; }
                        out += __popcll(mask);
                    }
                    m = out;
                    in_lds = true;
                    __syncthreads();
                }
            }
            if constexpr (OWN) {
                uint32_t out = 0;
                for (uint32_t i0 = 0; i0 < mo; i0 += 64) {
                    const uint32_t i = i0 + lane;
                    uint32_t e = 0; bool keep = false;
                    if (i < mo) {
                        e = own_cand[i];
                        keep = e + (uint32_t)j < own_len && own[e + j] == win_tok;
                    }
                    const uint64_t mask = __ballot(keep);
                    const uint32_t pos = out + __popcll(mask & ((1ull << lane) - 1ull));
                    __syncthreads();               // all reads of this chunk precede the writes
                    if (keep) own_cand[pos] = e;   // pos <= i: never overtakes unread entries
                    out += __popcll(mask);
                }
                mo = out;
                __syncthreads();
            }
        }
        // ---- smallest surviving position ----
        uint32_t mn = 0xFFFFFFFFu;
        if (in_lds) {
            for (uint32_t i = lane; i < m; i += 64) mn = min(mn, cand[i]);
        } else {
            for (uint32_t i = lane; i < count; i += 64) {
                uint32_t e = a.sa[start + i];
                bool keep = (e + (uint32_t)len) < a.seq_end[e];
                for (int c = 1; c <= len && keep; ++c) keep = (a.P[e + c] == chain[c - 1]);
                if (keep) mn = min(mn, e);
            }
        }
        for (int off = 32; off > 0; off >>= 1) mn = min(mn, (uint32_t)__shfl_xor((int)mn, off));
        __syncthreads();
        // pool positions precede the own text's; a result that survives only there is reported as -2 - position
        // (own_cand stays position-ascending through the filters, so its first entry is the smallest)
        long long idx = (long long)mn;
        if (OWN && mn == 0xFFFFFFFFu) idx = mo > 0 ? -2ll - (long long)own_cand[0] : -1ll;

        if (len >= a.min_tokens) {
            res_len = len; res_n = n; res_idx = idx; done = true;
        } else if (len > best_len) {
            best_len = len; best_n = n; best_idx = idx;
            for (int i = lane; i < len; i += 64) best_chain[i] = chain[i];
            __syncthreads();
        }
    }
    const int* src = chain;
    if (!done) { res_len = best_len; res_n = best_n; res_idx = best_idx; src = best_chain; }
    __syncthreads();
    for (int i = lane; i < a.K; i += 64) a.drafts[(size_t)b * a.K + i] = i < res_len ? src[i] : -1;
    if (lane == 0) {
        a.draft_len[b] = res_len;
        a.match_n[b] = res_len > 0 ? res_n : 0;
        a.pool_index[b] = res_len > 0 ? res_idx : -1;
    }
}

// ---------------------------------------------------------------------------------------------- token trees
// Tree-based drafting (Sec. 3.3): the sub-tree of the key's trie below the node the context suffix reaches, cut to
// its K most frequent nodes. A node is a path of successor tokens; its frequency is the number of occurrences of the
// suffix whose continuation starts with that path. Nodes are taken best first: always the best node not yet taken
// whose parent is taken (higher frequency, then smaller depth, then the parent taken earlier, then the smaller token
// id); a child is never more frequent than its parent, so these are the K best nodes of the whole sub-tree.
// One wavefront per context. Taking a node means one vote over the occurrences that continue with its path
// (re-checked against the path, so any number of occurrences works) to find its children and their frequencies;
// the best K - (taken) of them join the frontier. The pseudo-sequence lists the taken nodes depth-first, siblings
// in the order taken.
constexpr int kTreeMax = LASER_MAX_TREE;                       // nodes of one tree
constexpr int kFrontier = kTreeMax * (kTreeMax + 1) / 2 + 16;  // every expansion adds at most K - taken children

struct TreeArgs {
    const int32_t* P; const uint32_t* seq_end; const uint32_t* sa; const IndexEntry* table;
    uint64_t cap_mask;
    const int64_t* keys; const int32_t* ctx_tail;
    int B, n_min, n_max, K, min_tokens;
    int32_t* tree_tokens; int32_t* tree_parent; int32_t* tree_freq; int32_t* tree_len; int32_t* match_n;
};

__global__ __launch_bounds__(64) void retrieve_tree_kernel(TreeArgs a) {
    __shared__ uint32_t cand[kCand];
    __shared__ uint32_t cand_end[kCand];
    __shared__ int vote_tok[kVote];
    __shared__ int vote_cnt[kVote];
    __shared__ int sh_distinct;
    __shared__ int t_tok[kTreeMax], t_par[kTreeMax], t_depth[kTreeMax], t_cnt[kTreeMax];     // taken nodes, in the order taken
    __shared__ int f_tok[kFrontier], f_cnt[kFrontier], f_par[kFrontier], f_depth[kFrontier];
    __shared__ int ch_tok[kTreeMax], ch_cnt[kTreeMax];                                       // best children of one expansion
    __shared__ int path[kTreeMax];
    __shared__ int b_tok[kTreeMax], b_par[kTreeMax], b_cnt[kTreeMax];                        // best tree seen (pseudo-sequence form)
    __shared__ int o_tok[kTreeMax], o_par[kTreeMax], o_cnt[kTreeMax], dfs_pos[kTreeMax], stack[kTreeMax];

    const int b = blockIdx.x, lane = threadIdx.x;
    const int64_t key = a.keys[b];
    const int32_t* tail = a.ctx_tail + (size_t)b * a.n_max;
    int valid = 0;
    while (valid < a.n_max && tail[a.n_max - 1 - valid] >= 0) ++valid;

    int best_len = 0, best_n = 0, res_len = 0, res_n = 0;
    bool done = false;
    const int n_hi = valid < a.n_max ? valid : a.n_max;
    for (int n = n_hi; n >= a.n_min && !done && a.K > 0; --n) {
        // ---- index probe (as in retrieve_kernel) ----
        const int32_t* w = tail + (a.n_max - n);
        uint64_t slot = ngram_hash(key, n, w) & a.cap_mask;
        uint32_t start = 0, count = 0;
        for (;;) {
            IndexEntry e = a.table[slot];
            if (e.count_n == 0) break;
            if (e.key == key && (int)(e.count_n >> 28) == n) {
                uint32_t e0 = a.sa[e.start];
                bool same = true;
                for (int i = 0; i < n; ++i) same = same && (a.P[e0 - (n - 1) + i] == w[i]);
                if (same) { start = e.start; count = e.count_n & 0x0FFFFFFFu; break; }
            }
            slot = (slot + 1) & a.cap_mask;
        }
        if (count == 0) continue;
        const bool in_lds = count <= (uint32_t)kCand;
        if (in_lds)
            for (uint32_t i = lane; i < count; i += 64) {
                const uint32_t e = a.sa[start + i];
                cand[i] = e;
                cand_end[i] = a.seq_end[e];
            }
        __syncthreads();

        int taken = 0, fsize = 0;
        // children of taken node `node` (-1: the root) at depth d: the best K - taken of them go to the frontier
        auto expand = [&](int node, int d) {
            for (int i = node, j = d - 1; j >= 0; --j) {           // every lane walks the same path (LDS broadcast reads)
                if (lane == 0) path[j] = t_tok[i];
                i = t_par[i];
            }
            const int want = a.K - taken;
            int n_ch = 0;                                            // uniform: entries of ch_*
            __syncthreads();
            int vsz = 64;
            while (vsz < kVote && (uint32_t)vsz < 4u * count) vsz *= 2;
            const int vfill = vsz / 4 * 3;
            for (uint32_t nparts = 1;; nparts *= 2) {
                bool overflow = false;
                n_ch = 0;
                for (uint32_t part = 0; part < nparts && !overflow; ++part) {
                    for (int i = lane; i < vsz; i += 64) { vote_tok[i] = kEmptyTok; vote_cnt[i] = 0; }
                    if (lane == 0) sh_distinct = 0;
                    __syncthreads();
                    for (uint32_t i0 = 0; i0 < count; i0 += 64) {
                        const uint32_t i = i0 + lane;
                        if (i < count) {
                            const uint32_t e = in_lds ? cand[i] : a.sa[start + i];
                            bool ok = (e + (uint32_t)d + 1u) < (in_lds ? cand_end[i] : a.seq_end[e]);
                            for (int c = 0; c < d && ok; ++c) ok = a.P[e + 1 + c] == path[c];
                            if (ok) {
                                const int tok = a.P[e + d + 1];
                                const uint32_t hh = fmix32((uint32_t)tok);
                                if (nparts == 1 || (hh / kVote) % nparts == part) {
                                    uint32_t s = hh & (vsz - 1);
                                    for (int probe = 0; probe < vsz; ++probe) {
                                        int cur = vote_tok[s];
                                        if (cur == kEmptyTok) {
                                            const int prev = atomicCAS(&vote_tok[s], kEmptyTok, tok);
                                            if (prev == kEmptyTok) { atomicAdd(&sh_distinct, 1); cur = tok; }
                                            else cur = prev;
                                        }
                                        if (cur == tok) { atomicAdd(&vote_cnt[s], 1); break; }
                                        s = (s + 1) & (vsz - 1);
                                    }
                                }
                            }
                        }
                        if ((i0 & 1023u) == 960u) {
                            __syncthreads();
                            if (sh_distinct > vfill) break;
                        }
                    }
                    __syncthreads();
                    overflow = sh_distinct > vfill;
                    __syncthreads();
                    if (overflow) break;
                    // this part's best `want` (count desc, token asc), merged into the sorted child list
                    for (int round = 0; round < want; ++round) {
                        int bc = 0, bt = 0x7FFFFFFF, bs = -1;
                        for (int i = lane; i < vsz; i += 64) {
                            const int c = vote_cnt[i], t = vote_tok[i];
                            if (c > bc || (c == bc && c > 0 && t < bt)) { bc = c; bt = t; bs = i; }
                        }
                        for (int off = 32; off > 0; off >>= 1) {
                            const int oc = __shfl_xor(bc, off), ot = __shfl_xor(bt, off), os = __shfl_xor(bs, off);
                            if (oc > bc || (oc == bc && oc > 0 && ot < bt)) { bc = oc; bt = ot; bs = os; }
                        }
                        if (bc == 0) break;                          // uniform
                        // insert (bt, bc) into ch_* (sorted, at most `want` entries); lane 0 does the shifting
                        int pos = n_ch;
                        while (pos > 0 && (ch_cnt[pos - 1] < bc || (ch_cnt[pos - 1] == bc && ch_tok[pos - 1] > bt))) --pos;
                        if (pos < want) {
                            if (lane == 0) {
                                const int last = n_ch < want ? n_ch : want - 1;
                                for (int q = last; q > pos; --q) { ch_tok[q] = ch_tok[q - 1]; ch_cnt[q] = ch_cnt[q - 1]; }
                                ch_tok[pos] = bt; ch_cnt[pos] = bc;
                                vote_cnt[bs] = 0;
                            }
                            if (n_ch < want) ++n_ch;
                        } else if (lane == 0) {
                            vote_cnt[bs] = 0;
                        }
                        __syncthreads();
                        if (pos >= want) break;                      // nothing later in this part can enter either
                    }
                    __syncthreads();
                }
                if (!overflow) break;
            }
            for (int i = lane; i < n_ch; i += 64) {
                f_tok[fsize + i] = ch_tok[i]; f_cnt[fsize + i] = ch_cnt[i]; f_par[fsize + i] = node; f_depth[fsize + i] = d + 1;
            }
            fsize += n_ch;
            __syncthreads();
        };
        expand(-1, 0);
        while (taken < a.K && fsize > 0) {
            // best frontier entry: count desc, depth asc, parent asc, token asc
            int bi = -1, bc = 0, bd = 0, bp = 0, bt = 0;
            auto better = [](int c, int d, int p, int t, int c2, int d2, int p2, int t2) {
                return c != c2 ? c > c2 : (d != d2 ? d < d2 : (p != p2 ? p < p2 : t < t2));
            };
            for (int i = lane; i < fsize; i += 64)
                if (bi < 0 || better(f_cnt[i], f_depth[i], f_par[i], f_tok[i], bc, bd, bp, bt)) {
                    bi = i; bc = f_cnt[i]; bd = f_depth[i]; bp = f_par[i]; bt = f_tok[i];
                }
            for (int off = 32; off > 0; off >>= 1) {
                const int oi = __shfl_xor(bi, off), oc = __shfl_xor(bc, off), od = __shfl_xor(bd, off), op = __shfl_xor(bp, off),
                          ot = __shfl_xor(bt, off);
                if (oi >= 0 && (bi < 0 || better(oc, od, op, ot, bc, bd, bp, bt))) { bi = oi; bc = oc; bd = od; bp = op; bt = ot; }
            }
            __syncthreads();
            if (lane == 0) {
                t_tok[taken] = bt; t_par[taken] = bp; t_depth[taken] = bd; t_cnt[taken] = bc;
                const int last = fsize - 1;
                f_tok[bi] = f_tok[last]; f_cnt[bi] = f_cnt[last]; f_par[bi] = f_par[last]; f_depth[bi] = f_depth[last];
            }
            --fsize;
            ++taken;
            __syncthreads();
            if (taken < a.K) expand(taken - 1, bd);
        }
        // ---- pseudo-sequence: depth-first, siblings in the order taken ----
        if (lane == 0) {
            int sp = 0, n_out = 0;
            for (int i = taken - 1; i >= 0; --i) if (t_par[i] < 0) stack[sp++] = i;
            while (sp > 0) {
                const int i = stack[--sp];
                dfs_pos[i] = n_out;
                o_tok[n_out] = t_tok[i]; o_cnt[n_out] = t_cnt[i];
                o_par[n_out] = t_par[i] < 0 ? -1 : dfs_pos[t_par[i]];
                ++n_out;
                for (int c = taken - 1; c > i; --c) if (t_par[c] == i) stack[sp++] = c;
            }
        }
        __syncthreads();
        if (taken >= a.min_tokens) {
            res_len = taken; res_n = n; done = true;
        } else if (taken > best_len) {
            best_len = taken; best_n = n;
            for (int i = lane; i < taken; i += 64) { b_tok[i] = o_tok[i]; b_par[i] = o_par[i]; b_cnt[i] = o_cnt[i]; }
            __syncthreads();
        }
    }
    const int *s_tok = o_tok, *s_par = o_par, *s_cnt = o_cnt;
    if (!done) { res_len = best_len; res_n = best_n; s_tok = b_tok; s_par = b_par; s_cnt = b_cnt; }
    __syncthreads();
    for (int i = lane; i < a.K; i += 64) {
        a.tree_tokens[(size_t)b * a.K + i] = i < res_len ? s_tok[i] : -1;
        a.tree_parent[(size_t)b * a.K + i] = i < res_len ? s_par[i] : -1;
        if (a.tree_freq) a.tree_freq[(size_t)b * a.K + i] = i < res_len ? s_cnt[i] : 0;
    }
    if (lane == 0) {
        a.tree_len[b] = res_len;
        a.match_n[b] = res_len > 0 ? res_n : 0;
    }
}

// Appends the tokens a step emitted (out_tokens[b][0 .. accept_len[b]]) to row b of the own-text buffer; a full row
// drops its oldest tokens (sliding window of `cap`). One workgroup per sequence.
__global__ __launch_bounds__(256) void own_text_append_kernel(int32_t* own, int32_t* own_len, int cap, const int32_t* out_tokens,
                                                              const int32_t* accept_len, int K) {
    const int b = blockIdx.x, tid = threadIdx.x;
    if (accept_len[b] < 0) return;                     // nothing was emitted for this sequence (it had finished before the step)
    int32_t* row = own + (size_t)b * cap;
    const int32_t* nw = out_tokens + (size_t)b * (K + 1);
    int n_new = min(accept_len[b], K) + 1;
    int len = min(max(own_len[b], 0), cap);
    const int skip = max(n_new - cap, 0);              // more new tokens than the row holds: keep the newest
    n_new -= skip;
    const int shift = max(len + n_new - cap, 0);
    if (shift > 0) {
        const int keep = len - shift;                  // row[shift .. len) moves to row[0 .. keep)
        for (int base = 0; base < keep; base += 256) {
            const int i = base + tid;
            const int32_t v = i < keep ? row[i + shift] : 0;
            __syncthreads();                           // every read of this chunk precedes its writes; later chunks read beyond them
            if (i < keep) row[i] = v;
        }
        len = max(keep, 0);
    }
    for (int i = tid; i < n_new; i += 256) row[len + i] = nw[skip + i];
    if (tid == 0) own_len[b] = len + n_new;
}

// ------------------------------------------------------------------------------------ host build
namespace {

struct SubPool { int64_t key; uint32_t begin, end; };

}  // namespace

static int build_pool(const int32_t* tokens, const int64_t* seq_off, const int64_t* seq_key,
                      int64_t n_seq, int n_max, hipStream_t stream, Pool** out) {
    const int64_t n_tok = n_seq > 0 ? seq_off[n_seq] : 0;
    LASER_REQUIRE(n_tok < 0xFFFFFFFFll, LASER_E_LIMIT, "pool of %lld tokens exceeds 2^32-2", (long long)n_tok);
    for (int64_t s = 0; s < n_seq; ++s)
        LASER_REQUIRE(seq_off[s + 1] >= seq_off[s], LASER_E_INVALID_ARG, "seq_off not ascending at %lld", (long long)s);

    // 1. regroup: ascending key, supply order inside a key
    std::vector<int64_t> order(n_seq);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int64_t x, int64_t y) { return seq_key[x] < seq_key[y]; });

    std::vector<int32_t> P((size_t)n_tok);
    std::vector<uint32_t> seq_begin((size_t)n_tok), seq_end((size_t)n_tok);
    std::vector<SubPool> subs;
    {
        uint32_t pos = 0;
        for (int64_t i = 0; i < n_seq; ++i) {
            const int64_t s = order[i];
            const uint32_t len = (uint32_t)(seq_off[s + 1] - seq_off[s]);
            if (subs.empty() || subs.back().key != seq_key[s]) subs.push_back({seq_key[s], pos, pos});
            for (uint32_t t = 0; t < len; ++t) {
                const int32_t tok = tokens[seq_off[s] + t];
                LASER_REQUIRE(tok >= 0, LASER_E_INVALID_ARG, "negative token in sequence %lld", (long long)s);
                P[pos + t] = tok;
                seq_begin[pos + t] = pos;
                seq_end[pos + t] = pos + len;
            }
            pos += len;
            subs.back().end = pos;
        }
    }

    // 2. sorted occurrence array: per sub-pool, positions with a successor, by reversed text
    std::vector<uint32_t> sa;
    sa.reserve((size_t)n_tok);
    std::vector<uint32_t> sub_sa_begin(subs.size() + 1);
    for (size_t g = 0; g < subs.size(); ++g) {
        sub_sa_begin[g] = (uint32_t)sa.size();
        for (uint32_t e = subs[g].begin; e < subs[g].end; ++e)
            if (e + 1 < seq_end[e]) sa.push_back(e);
    }
    sub_sa_begin[subs.size()] = (uint32_t)sa.size();

    auto back_tok = [&](uint32_t e, int i) -> int64_t {       // i-th token back from e, or -1 before the sequence
        return (e - seq_begin[e] >= (uint32_t)i) ? (int64_t)P[e - i] : -1;
    };
    auto less = [&](uint32_t x, uint32_t y) {
        for (int i = 0; i < n_max; ++i) {
            const int64_t a = back_tok(x, i), b = back_tok(y, i);
            if (a != b) return a < b;
        }
        return x < y;
    };
    {
        const unsigned hw = std::max(1u, std::min(16u, std::thread::hardware_concurrency()));
        const size_t G = subs.size();
        if (G <= 1 || hw == 1) {
            for (size_t g = 0; g < G; ++g)
                std::sort(sa.begin() + sub_sa_begin[g], sa.begin() + sub_sa_begin[g + 1], less);
        } else {
            // split the sub-pools into hw contiguous chunks of roughly equal size
            std::vector<std::thread> th;
            std::vector<size_t> cut(hw + 1, G);
            cut[0] = 0;
            const uint64_t total = sa.size();
            size_t g = 0;
            for (unsigned t = 1; t < hw; ++t) {
                const uint64_t target = total * t / hw;
                while (g < G && sub_sa_begin[g] < target) ++g;
                cut[t] = g;
            }
            for (unsigned t = 0; t < hw; ++t)
                th.emplace_back([&, t] {
                    for (size_t q = cut[t]; q < cut[t + 1]; ++q)
                        std::sort(sa.begin() + sub_sa_begin[q], sa.begin() + sub_sa_begin[q + 1], less);
                });
            for (auto& x : th) x.join();
        }
    }

    // 3. runs of equal n-grams -> table entries
    auto same_ngram = [&](uint32_t x, uint32_t y, int n) {
        for (int i = 0; i < n; ++i) {
            const int64_t a = back_tok(x, i), b = back_tok(y, i);
            if (a < 0 || a != b) return false;
        }
        return true;
    };
    auto has_n = [&](uint32_t e, int n) { return e - seq_begin[e] >= (uint32_t)(n - 1); };

    // two passes over the runs (count, then insert) keep the host footprint at the table itself
    auto for_each_run = [&](auto&& fn) -> bool {
        for (size_t g = 0; g < subs.size(); ++g) {
            const uint32_t lo = sub_sa_begin[g], hi = sub_sa_begin[g + 1];
            for (int n = 1; n <= n_max; ++n) {
                uint32_t i = lo;
                while (i < hi) {
                    if (!has_n(sa[i], n)) { ++i; continue; }
                    uint32_t j = i + 1;
                    while (j < hi && same_ngram(sa[i], sa[j], n)) ++j;
                    if (!fn(g, n, i, j - i)) return false;
                    i = j;
                }
            }
        }
        return true;
    };
    uint64_t n_runs = 0;
    uint32_t longest = 0;
    for_each_run([&](size_t, int, uint32_t, uint32_t c) { ++n_runs; longest = std::max(longest, c); return true; });
    LASER_REQUIRE(longest < (1u << 28), LASER_E_LIMIT, "an n-gram occurs %u times (limit 2^28-1)", longest);
    uint64_t cap = 16;
    while (cap < 2 * n_runs) cap <<= 1;
    std::vector<IndexEntry> table(cap);
    std::memset(table.data(), 0, cap * sizeof(IndexEntry));
    for_each_run([&](size_t g, int n, uint32_t start, uint32_t c) {
        int32_t w[LASER_MAX_NGRAM];
        const uint32_t e0 = sa[start];
        for (int i = 0; i < n; ++i) w[i] = P[e0 - (n - 1) + i];
        uint64_t slot = ngram_hash(subs[g].key, n, w) & (cap - 1);
        while (table[slot].count_n != 0) slot = (slot + 1) & (cap - 1);
        table[slot] = {subs[g].key, start, c | ((uint32_t)n << 28)};
        return true;
    });

    // 4. upload
    Pool* p = new Pool();
    p->n_tokens = n_tok; p->n_keys = (int64_t)subs.size(); p->n_entries = (int64_t)n_runs;
    p->n_sa = (int64_t)sa.size(); p->n_max = n_max; p->cap_mask = cap - 1;
    auto up = [&](void** dst, const void* src, size_t bytes) -> int {
        const size_t alloc = bytes ? bytes : 16;
        LASER_HIP_CHECK(hipMalloc(dst, alloc));
        p->device_bytes += (int64_t)alloc;
        if (bytes) LASER_HIP_CHECK(hipMemcpyAsync(*dst, src, bytes, hipMemcpyHostToDevice, stream));
        return LASER_OK;
    };
    int rc;
    if ((rc = up((void**)&p->P, P.data(), P.size() * 4)) || (rc = up((void**)&p->seq_end, seq_end.data(), seq_end.size() * 4)) ||
        (rc = up((void**)&p->sa, sa.data(), sa.size() * 4)) || (rc = up((void**)&p->table, table.data(), cap * sizeof(IndexEntry)))) {
        (void)hipFree(p->P); (void)hipFree(p->seq_end); (void)hipFree(p->sa); (void)hipFree(p->table);
        delete p;
        return rc;
    }
    LASER_HIP_CHECK(hipStreamSynchronize(stream));
    *out = p;
    return LASER_OK;
}

}  // namespace laser

using namespace laser;

extern "C" int laser_pool_build(const int32_t* tokens, const int64_t* seq_off, const int64_t* seq_key,
                                int64_t n_seq, int n_max, void* stream, laser_pool** out) {
    LASER_REQUIRE(out != nullptr, LASER_E_INVALID_ARG, "out is NULL");
    LASER_REQUIRE(n_seq >= 0, LASER_E_INVALID_ARG, "n_seq < 0");
    LASER_REQUIRE(n_seq == 0 || (tokens && seq_off && seq_key), LASER_E_INVALID_ARG, "NULL input array");
    LASER_REQUIRE(n_max >= 1 && n_max <= LASER_MAX_NGRAM, LASER_E_INVALID_ARG, "n_max %d outside 1..%d", n_max, LASER_MAX_NGRAM);
    LASER_REQUIRE(n_seq == 0 || seq_off[0] == 0, LASER_E_INVALID_ARG, "seq_off[0] != 0");
    Pool* p = nullptr;
    int rc = build_pool(tokens, seq_off, seq_key, n_seq, n_max, (hipStream_t)stream, &p);
    if (rc == LASER_OK) *out = reinterpret_cast<laser_pool*>(p);
    return rc;
}

extern "C" int laser_pool_destroy(laser_pool* pool) {
    if (!pool) return LASER_OK;
    Pool* p = reinterpret_cast<Pool*>(pool);
    (void)hipFree(p->P); (void)hipFree(p->seq_end); (void)hipFree(p->sa); (void)hipFree(p->table);
    delete p;
    return LASER_OK;
}

extern "C" int laser_pool_info(const laser_pool* pool, int64_t* n_tokens, int64_t* n_keys,
                               int64_t* n_index_entries, int64_t* device_bytes) {
    LASER_REQUIRE(pool != nullptr, LASER_E_INVALID_ARG, "pool is NULL");
    const Pool* p = reinterpret_cast<const Pool*>(pool);
    if (n_tokens) *n_tokens = p->n_tokens;
    if (n_keys) *n_keys = p->n_keys;
    if (n_index_entries) *n_index_entries = p->n_entries;
    if (device_bytes) *device_bytes = p->device_bytes;
    return LASER_OK;
}

extern "C" int laser_pool_read_tokens(const laser_pool* pool, int64_t start, int64_t count, int32_t* out_host) {
    LASER_REQUIRE(pool != nullptr && out_host != nullptr, LASER_E_INVALID_ARG, "NULL argument");
    const Pool* p = reinterpret_cast<const Pool*>(pool);
    LASER_REQUIRE(start >= 0 && count >= 0 && start + count <= p->n_tokens, LASER_E_INVALID_ARG,
                  "range [%lld, +%lld) outside the pool", (long long)start, (long long)count);
    if (count) LASER_HIP_CHECK(hipMemcpy(out_host, p->P + start, (size_t)count * 4, hipMemcpyDeviceToHost));
    return LASER_OK;
}

static int retrieve_impl(const laser_pool* pool, const int64_t* keys, const int32_t* ctx_tail, const int32_t* own,
                         const int32_t* own_len, int own_cap, int B, int n_min, int n_max, int K, int min_tokens,
                         int32_t* drafts, int32_t* draft_len, int32_t* match_n, int64_t* pool_index, void* stream) {
    LASER_REQUIRE(pool != nullptr, LASER_E_INVALID_ARG, "pool is NULL");
    const Pool* p = reinterpret_cast<const Pool*>(pool);
    LASER_REQUIRE(B >= 0, LASER_E_INVALID_ARG, "B < 0");
    LASER_REQUIRE(K >= 0 && K <= LASER_MAX_DRAFT, LASER_E_INVALID_ARG, "K %d outside 0..%d", K, LASER_MAX_DRAFT);
    LASER_REQUIRE(n_max >= 1 && n_max <= p->n_max, LASER_E_INVALID_ARG, "n_max %d outside 1..%d (the pool's)", n_max, p->n_max);
    LASER_REQUIRE(n_min >= 1 && n_min <= n_max, LASER_E_INVALID_ARG, "n_min %d outside 1..n_max", n_min);
    if (B == 0) return LASER_OK;
    LASER_REQUIRE(keys && ctx_tail && draft_len && match_n && pool_index && (drafts || K == 0),
                  LASER_E_INVALID_ARG, "NULL device buffer");
    RetrieveArgs a{p->P, p->seq_end, p->sa, p->table, p->cap_mask, keys, ctx_tail,
                   B, n_min, n_max, K, min_tokens < 1 ? 1 : min_tokens, drafts, draft_len, match_n, pool_index,
                   own, own_len, own_cap};
    if (own) hipLaunchKernelGGL(retrieve_kernel<true>, dim3(B), dim3(64), 0, (hipStream_t)stream, a);
    else hipLaunchKernelGGL(retrieve_kernel<false>, dim3(B), dim3(64), 0, (hipStream_t)stream, a);
    LASER_HIP_CHECK(hipGetLastError());
    return LASER_OK;
}

extern "C" int laser_retrieve_drafts(const laser_pool* pool, const int64_t* keys, const int32_t* ctx_tail,
                                     int B, int n_min, int n_max, int K, int min_tokens,
                                     int32_t* drafts, int32_t* draft_len, int32_t* match_n,
                                     int64_t* pool_index, void* stream) {
    return retrieve_impl(pool, keys, ctx_tail, nullptr, nullptr, 0, B, n_min, n_max, K, min_tokens, drafts, draft_len,
                         match_n, pool_index, stream);
}

extern "C" int laser_retrieve_drafts_temp(const laser_pool* pool, const int64_t* keys, const int32_t* ctx_tail,
                                          const int32_t* own_tokens, const int32_t* own_len, int own_cap,
                                          int B, int n_min, int n_max, int K, int min_tokens,
                                          int32_t* drafts, int32_t* draft_len, int32_t* match_n,
                                          int64_t* pool_index, void* stream) {
    LASER_REQUIRE(own_cap >= 1 && own_cap <= LASER_MAX_OWN_TEXT, LASER_E_INVALID_ARG, "own_cap %d outside 1..%d", own_cap,
                  LASER_MAX_OWN_TEXT);
    LASER_REQUIRE(B <= 0 || (own_tokens && own_len), LASER_E_INVALID_ARG, "NULL own-text buffer");
    return retrieve_impl(pool, keys, ctx_tail, own_tokens, own_len, own_cap, B, n_min, n_max, K, min_tokens, drafts,
                         draft_len, match_n, pool_index, stream);
}

extern "C" int laser_retrieve_tree(const laser_pool* pool, const int64_t* keys, const int32_t* ctx_tail, int B, int n_min, int n_max,
                                   int K, int min_tokens, int32_t* tree_tokens, int32_t* tree_parent, int32_t* tree_freq,
                                   int32_t* tree_len, int32_t* match_n, void* stream) {
    LASER_REQUIRE(pool != nullptr, LASER_E_INVALID_ARG, "pool is NULL");
    const Pool* p = reinterpret_cast<const Pool*>(pool);
    LASER_REQUIRE(B >= 0, LASER_E_INVALID_ARG, "B < 0");
    LASER_REQUIRE(K >= 0 && K <= LASER_MAX_TREE, LASER_E_INVALID_ARG, "K %d outside 0..%d", K, LASER_MAX_TREE);
    LASER_REQUIRE(n_max >= 1 && n_max <= p->n_max, LASER_E_INVALID_ARG, "n_max %d outside 1..%d (the pool's)", n_max, p->n_max);
    LASER_REQUIRE(n_min >= 1 && n_min <= n_max, LASER_E_INVALID_ARG, "n_min %d outside 1..n_max", n_min);
    if (B == 0) return LASER_OK;
    LASER_REQUIRE(keys && ctx_tail && tree_len && match_n && ((tree_tokens && tree_parent) || K == 0), LASER_E_INVALID_ARG,
                  "NULL device buffer");
    TreeArgs a{p->P, p->seq_end, p->sa, p->table, p->cap_mask, keys, ctx_tail, B, n_min, n_max, K, min_tokens < 1 ? 1 : min_tokens,
               tree_tokens, tree_parent, tree_freq, tree_len, match_n};
    hipLaunchKernelGGL(retrieve_tree_kernel, dim3(B), dim3(64), 0, (hipStream_t)stream, a);
    LASER_HIP_CHECK(hipGetLastError());
    return LASER_OK;
}

extern "C" int laser_own_text_append(int32_t* own_tokens, int32_t* own_len, int own_cap, const int32_t* out_tokens,
                                     const int32_t* accept_len, int B, int K, void* stream) {
    LASER_REQUIRE(B >= 0 && K >= 0 && K <= LASER_MAX_DRAFT, LASER_E_INVALID_ARG, "B < 0 or K outside 0..%d", LASER_MAX_DRAFT);
    LASER_REQUIRE(own_cap >= 1 && own_cap <= LASER_MAX_OWN_TEXT, LASER_E_INVALID_ARG, "own_cap %d outside 1..%d", own_cap,
                  LASER_MAX_OWN_TEXT);
    if (B == 0) return LASER_OK;
    LASER_REQUIRE(own_tokens && own_len && out_tokens && accept_len, LASER_E_INVALID_ARG, "NULL device buffer");
    hipLaunchKernelGGL(own_text_append_kernel, dim3(B), dim3(256), 0, (hipStream_t)stream, own_tokens, own_len, own_cap,
                       out_tokens, accept_len, K);
    LASER_HIP_CHECK(hipGetLastError());
    return LASER_OK;
}
