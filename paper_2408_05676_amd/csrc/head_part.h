// Per-row partial statistics of the output head (Sec. 3.4 Eq. 7-8): what every kernel that produces logits keeps of
// them INSTEAD of the logits -- per (row, vocabulary chunk) the softmax statistics (running maximum, sum of
// exponentials), the arg-max (smaller id on ties) and the chunk's best LASER_MAX_TOPK (logit, id) pairs; beside them
// the logit of every CANDIDATE token of the row, written by the one chunk that holds it. A row's candidates are the
// draft tokens that would follow its token: one for a chain of drafts, the row's children for a token tree (Sec. 3.3).
// accept_kernel merges the chunks of a row: a candidate's rank is the number of listed entries ordered before it; a
// chunk that hides an entry preceding the candidate already lists LASER_MAX_TOPK >= k such entries, so "rank < k" is
// decided exactly.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cmath>

#include "../../include/laser.h"

namespace laser {

constexpr int KT = LASER_MAX_TOPK;

// where the records go: [row][chunk] arrays of the model handle (or of the static scratch)
struct HeadPart {
    const int32_t* cand_beg; // [rows] first candidate of the row (index into cand_x / cand_lx)
    const int32_t* cand_cnt; // [rows] its number of candidates
    const int32_t* cand_x;   // [candidates] token id
    float* cand_lx;          // [candidates] out: the candidate's logit in its row
    float* hp_max; float* hp_sum; int32_t* hp_arg; float* hp_topv; int32_t* hp_topi;   // [rows][chunks] (x KT)
    int chunks;              // records per row
    int topk;                // the call's k (1..LASER_MAX_TOPK): list entries beyond the k-th are never needed
    float* logits_dbg;       // optional [rows][V] copy of the logits (debug), else NULL
};

// Parent of node i of sequence b's pseudo-sequence (-1: child of the root, i.e. it follows the pending token).
// parent == NULL: the drafts are a chain. Padding nodes (i >= n_nodes) hang off the node before them; an entry that
// does not name an earlier node counts as -1. Every kernel that needs the tree's shape reads it through this.
__device__ inline int tree_parent_of(const int32_t* parent, int b, int K, int i, int n_nodes) {
    if (!parent || i >= n_nodes) return i - 1;
    const int p = parent[(size_t)b * K + i];
    return (p < -1 || p >= i) ? -1 : p;
}

// The candidates of row `row` whose token lies in [n0, n0 + count): their logits are vals[token - n0].
template <class Get>
__device__ inline void store_candidates(const HeadPart& hp, int row, int n0, int count, Get&& get) {
    const int cb = hp.cand_beg[row], cn = hp.cand_cnt[row];
    for (int c = 0; c < cn; ++c) {
        const int x = hp.cand_x[cb + c];
        if (x >= n0 && x < n0 + count) hp.cand_lx[cb + c] = get(x - n0);
    }
}

// ordering of (logit, id): larger logit first, smaller id on ties
__device__ inline bool before(float v, int i, float w, int j) { return v > w || (v == w && i < j); }

// KD: entries of the list the statistics keep, topk <= KD <= KT (a shorter list is all a call with a small k needs,
// and costs a fraction of the full one to maintain); the stored record is padded to KT entries.
template <int KD>
struct RowStatT {
    static_assert(KD >= 1 && KD <= KT, "list depth");
    float mx, sum;
    int arg;
    float tv[KD];
    int ti[KD];
    __device__ void init() {
        mx = -INFINITY; sum = 0.f; arg = 0x7FFFFFFF;
#pragma unroll
        for (int j = 0; j < KD; ++j) { tv[j] = -INFINITY; ti[j] = 0x7FFFFFFF; }
    }
    __device__ void push_top(float v, int n) {
        if (!before(v, n, tv[KD - 1], ti[KD - 1])) return;
        tv[KD - 1] = v; ti[KD - 1] = n;
#pragma unroll
        for (int j = KD - 1; j > 0; --j) {
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
    __device__ void merge(float omx, float osum, int oarg, const float (&otv)[KD], const int (&oti)[KD]) {
        const float M = fmaxf(mx, omx);
        if (M != -INFINITY) sum = sum * __expf(mx - M) + osum * __expf(omx - M);
        if (before(omx, oarg, mx, arg)) arg = oarg;
        mx = M;
#pragma unroll
        for (int j = 0; j < KD; ++j) push_top(otv[j], oti[j]);
    }
    __device__ void merge_from_lane(int src_xor) {
        const float omx = __shfl_xor(mx, src_xor), osum = __shfl_xor(sum, src_xor);
        const int oarg = __shfl_xor(arg, src_xor);
        float otv[KD]; int oti[KD];
#pragma unroll
        for (int j = 0; j < KD; ++j) { otv[j] = __shfl_xor(tv[j], src_xor); oti[j] = __shfl_xor(ti[j], src_xor); }
        merge(omx, osum, oarg, otv, oti);
    }
    // record (row, chunk) of the partial arrays
    __device__ void store(const HeadPart& hp, int row, int chunk) const {
        const size_t o = (size_t)row * hp.chunks + chunk;
        hp.hp_max[o] = mx; hp.hp_sum[o] = sum; hp.hp_arg[o] = arg;
#pragma unroll
        for (int j = 0; j < KT; ++j) {
            hp.hp_topv[o * KT + j] = j < KD ? tv[j < KD ? j : 0] : -INFINITY;
            hp.hp_topi[o * KT + j] = j < KD ? ti[j < KD ? j : 0] : 0x7FFFFFFF;
        }
    }
    // the same record in LDS for a merge across the waves of a workgroup
    static constexpr int kWords = 3 + 2 * KD;
    __device__ void to_lds(float* p) const {
        p[0] = mx; p[1] = sum; p[2] = __int_as_float(arg);
#pragma unroll
        for (int j = 0; j < KD; ++j) { p[3 + j] = tv[j]; p[3 + KD + j] = __int_as_float(ti[j]); }
    }
    __device__ void merge_lds(const float* p) {
        float otv[KD]; int oti[KD];
#pragma unroll
        for (int j = 0; j < KD; ++j) { otv[j] = p[3 + j]; oti[j] = __float_as_int(p[3 + KD + j]); }
        merge(p[0], p[1], __float_as_int(p[2]), otv, oti);
    }
};
using RowStat = RowStatT<KT>;

}  // namespace laser
