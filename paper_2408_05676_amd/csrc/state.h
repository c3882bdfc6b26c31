// Host-side state behind the opaque laser_model / laser_kv handles.
#pragma once

#include <vector>

#include "common.h"

namespace laser {

constexpr int kPageSize = 16;     // tokens per KV page (fixed: one MFMA token tile)
constexpr int kIdSlots = 64;      // ring of staged seq-id vectors

// KV page layouts (fp16), per layer l, page g, head h:
//   kpages[((l * n_pages + g) * H + h) * 16 * dh + t * dh + c]     token-major  (t = slot in page)
//   vpages[((l * n_pages + g) * H + h) * dh * 16 + c * 16 + t]     channel-major (transposed)
// so that a 16-token page of one head is one contiguous 4 KiB block (dh = 128) in either pool and
// both feed the matrix cores without an in-kernel transpose. Keys are stored split (see mfma.h):
// klpages holds their 8-bit low plane, one byte per element, indexed like kpages.
struct KV {
    laser_kv_desc d{};
    uint16_t* kpages = nullptr;
    uint8_t* klpages = nullptr;       // 8-bit low plane of the split keys, indexed like kpages: k = kpages + klpages / 4096
    uint16_t* vpages = nullptr;
    int32_t* block_table = nullptr;   // [dev] [max_seqs][max_pages_per_seq]
    int32_t* len = nullptr;           // [dev] [max_seqs] committed tokens
    // host bookkeeping
    std::vector<int32_t> h_block_table;
    std::vector<int32_t> h_npages;    // pages owned per slot
    std::vector<int32_t> h_len_ub;    // upper bound of len per slot
    std::vector<int32_t> h_last_rows; // R of the last verify per slot (commit adds at most this)
    std::vector<int32_t> free_pages;
    // staging ring for per-call seq-id vectors
    int32_t* ids_pinned = nullptr;    // [kIdSlots][max_seqs]
    int32_t* ids_dev = nullptr;       // [kIdSlots][max_seqs]
    hipEvent_t ids_ev[kIdSlots]{};
    bool ids_used[kIdSlots]{};
    int ids_last = -1, ids_last_n = 0;            // most recently staged slot, its id count and stream
    hipStream_t ids_last_stream = nullptr;
    int ids_next = 0;

    int stage_ids(const int32_t* host_ids, int B, hipStream_t stream, const int32_t** dev_out);
    size_t page_elems() const { return (size_t)d.n_heads * kPageSize * d.head_dim; }
};

struct Model {
    laser_model_desc d{};
    int dh = 0;
    // workspace (device)
    float* x = nullptr;          // [max_rows][d]   residual stream
    uint16_t* xn = nullptr;      // [max_rows][d]   normed activations (fp16, high plane)
    uint16_t* xn_lo = nullptr;   // [max_rows][d]   their low plane (x = xn + xn_lo / 4096); likewise q_lo, attn_lo
    uint16_t* q_lo = nullptr;
    uint16_t* attn_lo = nullptr;
    float* qkv = nullptr;        // [max_rows][3d]
    uint16_t* q = nullptr;       // [max_rows][d]   rotated queries (fp16)
    uint16_t* attn = nullptr;    // [max_rows][d]
    uint16_t* act = nullptr;     // [max_rows][F]
    int32_t* row_pos = nullptr;  // [max_rows] position of the row's token: committed length + depth in the token tree (chain: + row number)
    int32_t* row_slot = nullptr; // [max_rows] cache slot of the row's key/value: committed length + row number
    unsigned long long* row_anc = nullptr;   // [max_rows] bit j: row j of the same sequence is this row or one of its ancestors
    float* att_part = nullptr;   // attention split partials
    size_t att_part_floats = 0;
    float2* rope = nullptr;      // [max_pos][dh/2] (cos, sin)
    // output-head partials
    int head_chunks = 0;
    float* hp_max = nullptr;     // [max_rows][most chunks any row count produces]
    float* hp_sum = nullptr;
    int32_t* hp_arg = nullptr;
    float* hp_topv = nullptr;    // [max_rows][chunks][LASER_MAX_TOPK]
    int32_t* hp_topi = nullptr;
    // candidate lists of the rows (head_part.h): [max_rows] each
    int32_t* cand_beg = nullptr;
    int32_t* cand_cnt = nullptr;
    int32_t* cand_x = nullptr;
    int32_t* node_cand = nullptr;
    float* cand_lx = nullptr;
    // acceptance, between its per-row and its per-sequence kernel: [max_rows] each
    float* row_mx = nullptr;
    float* row_sum = nullptr;
    int32_t* row_arg = nullptr;
    int32_t* cand_rank = nullptr;
    // optional timing of the dominant kernel (laser_profile_begin / laser_profile_end)
    std::vector<hipEvent_t> prof_ev;   // start/stop pairs
    int prof_cap = 0, prof_n = 0;
    bool prof_on = false;
    void* fused_ws = nullptr;          // workspace of the persistent few-row kernel (fused.hip)
    int use_fused = 1;                 // 0 forces the generic multi-kernel path
    int fused_trace = 0;               // 1: thread 0 of every workgroup stamps the wall clock at phase edges
    uint16_t* w16[4] = {nullptr, nullptr, nullptr, nullptr};   // fp16 copies of wqkv, wo, wgu, wdown for the tiled many-row
                                                               // kernels, made at the first step with more than 80 rows
    uint16_t* wlm16 = nullptr;         // fp16 copy of the head matrix, made at the first head call with more than 80 rows
    int f16_copies = 1;                // 0: the tiled kernels stream the bf16 weights and widen them in the loop (no copies)
    float* kpart = nullptr;            // partial results of reduction-split tiled GEMMs (many-row path), [parts][rows][N]
    size_t kpart_floats = 0;
    int ksplit_opt[3] = {0, 0, 0};     // forced reduction parts for QKV, O, down (0 = choose from the tile count)
    int mid_waves = 0;                 // 17..80 rows: waves per workgroup of the weight-streaming GEMM, 0 = chosen per launch shape
    int attn_whole_min = 0;            // attention takes a context unsplit from this many (sequence, head, query tile) triples on; 0: half the number of compute units
    int attn_waves = 0;                // unsplit attention: waves per workgroup that share a context's pages (4 or 8), 0 = chosen per launch shape
    int split_ffn = 0;                 // 1: the many-row (tiled) gate/up product also takes split activations
};

}  // namespace laser
