// Paged KV cache bookkeeping: page reservation on the host (no device reads), the commit of
// accepted tokens and the between-step context update on the device.
#include <algorithm>
#include <cstring>

#include "state.h"

namespace laser {

int KV::stage_ids(const int32_t* host_ids, int B, hipStream_t stream, const int32_t** dev_out) {
    // The same ids on the same stream as the staging before (the steady state of a decoding loop, where verify and
    // commit alternate over one batch): that device copy is still intact and ordered before this call.
    if (ids_last >= 0 && ids_last_n == B && ids_last_stream == stream &&
        std::memcmp(ids_pinned + (size_t)ids_last * d.max_seqs, host_ids, (size_t)B * sizeof(int32_t)) == 0) {
        *dev_out = ids_dev + (size_t)ids_last * d.max_seqs;
        return LASER_OK;
    }
    const int s = ids_next;
    ids_next = (ids_next + 1) % kIdSlots;
    if (ids_used[s]) LASER_HIP_CHECK(hipEventSynchronize(ids_ev[s]));   // slot's last copy has been consumed
    int32_t* pin = ids_pinned + (size_t)s * d.max_seqs;
    int32_t* dev = ids_dev + (size_t)s * d.max_seqs;
    std::memcpy(pin, host_ids, (size_t)B * sizeof(int32_t));
    LASER_HIP_CHECK(hipMemcpyAsync(dev, pin, (size_t)B * sizeof(int32_t), hipMemcpyHostToDevice, stream));
    LASER_HIP_CHECK(hipEventRecord(ids_ev[s], stream));
    ids_used[s] = true;
    ids_last = s; ids_last_n = B; ids_last_stream = stream;
    *dev_out = dev;
    return LASER_OK;
}

__global__ void fill_i32_kernel(int32_t* p, int32_t v, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// max_accept: the most drafts any of the call's sequences had in the verify step before it. The host has already
// raised its bound of every length by that step's rows; a value outside -1..max_accept (a caller's mistake) is cut
// to that range so that a length never passes the bound the pages were reserved against.
__global__ void commit_kernel(int32_t* len, const int32_t* seq_ids, const int32_t* accept_len, int B, int max_accept) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) len[seq_ids[b]] += min(max(accept_len[b], -1), max_accept) + 1;
}

// Token trees (Sec. 3.3-3.4): the rows of a verify step sit in slots len + 1 + (node index); the accepted branch's
// rows (accept_path[b][0 .. accept_len[b]), ascending node indices) move to slots len + 1, len + 2, .. behind the
// pending token before the length grows. A thread owns one channel of one (sequence, layer, head) and moves its
// elements branch position by branch position: sources never lie before their destinations (path[j] >= j), and a
// destination is never a later source, so the in-place order j = 0, 1, .. is safe.
__global__ void kv_compact_kernel(uint16_t* kpages, uint8_t* klpages, uint16_t* vpages, const int32_t* block_table,
                                  const int32_t* len, const int32_t* seq_ids, const int32_t* accept_len,
                                  const int32_t* accept_path, int K, int H, int dh, int mpps, int n_pages) {
    const int h = blockIdx.x, l = blockIdx.y, b = blockIdx.z, c = threadIdx.x;
    const int slot = seq_ids[b], len0 = len[slot];
    int a = accept_len[b];
    a = a < 0 ? 0 : (a > K ? K : a);
    const int32_t* bt = block_table + (size_t)slot * mpps;
    for (int j = 0; j < a; ++j) {
        const int i = accept_path[(size_t)b * K + j];
        if (i < j || i >= K) break;                     // not a branch of this step's tree: nothing more to move
        if (i == j) continue;
        const int src = len0 + 1 + i, dst = len0 + 1 + j;
        const size_t sb = (((size_t)l * n_pages + bt[src / kPageSize]) * H + h) * kPageSize * dh;
        const size_t db = (((size_t)l * n_pages + bt[dst / kPageSize]) * H + h) * kPageSize * dh;
        const int st = src % kPageSize, dt = dst % kPageSize;
        kpages[db + (size_t)dt * dh + c] = kpages[sb + (size_t)st * dh + c];
        klpages[db + (size_t)dt * dh + c] = klpages[sb + (size_t)st * dh + c];
        vpages[db + (size_t)c * kPageSize + dt] = vpages[sb + (size_t)c * kPageSize + st];
    }
}

__global__ void ctx_advance_kernel(int32_t* ctx_tail, int32_t* pending, const int32_t* out_tokens,
                                   const int32_t* accept_len, int B, int K, int n_max) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int a = accept_len[b];
    a = a < 0 ? 0 : (a > K ? K : a);
    const int n_new = a + 1;
    int32_t* tail = ctx_tail + (size_t)b * n_max;
    const int32_t* out = out_tokens + (size_t)b * (K + 1);
    int32_t tmp[LASER_MAX_NGRAM];
    for (int i = 0; i < n_max; ++i) {                 // i-th entry of the new tail
        const int src = i + n_new;                    // index into old tail ++ emitted
        tmp[i] = src < n_max ? tail[src] : out[src - n_max];
    }
    for (int i = 0; i < n_max; ++i) tail[i] = tmp[i];
    pending[b] = out[a];
}

// k, v: [n_tokens][H][dh] -> pages of one layer
__global__ void kv_import_kernel(uint16_t* kpages, uint8_t* klpages, uint16_t* vpages, const int32_t* block_row,
                                 const uint16_t* k, const uint16_t* v, int n_tokens, int H, int dh,
                                 int layer, int n_pages) {
    const size_t total = (size_t)n_tokens * H * dh;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int c = (int)(i % dh);
    const int h = (int)((i / dh) % H);
    const int t = (int)(i / ((size_t)dh * H));
    const int pg = block_row[t / kPageSize], tp = t % kPageSize;
    const size_t base = (((size_t)layer * n_pages + pg) * H + h) * kPageSize * dh;
    kpages[base + (size_t)tp * dh + c] = k[i];
    klpages[base + (size_t)tp * dh + c] = 0;          // imported keys are plain fp16
    vpages[base + (size_t)c * kPageSize + tp] = v[i];
}

}  // namespace laser

using namespace laser;

extern "C" int laser_kv_create(const laser_kv_desc* desc, void* stream_, laser_kv** out) {
    LASER_REQUIRE(desc && out, LASER_E_INVALID_ARG, "NULL argument");
    hipStream_t stream = (hipStream_t)stream_;
    const laser_kv_desc& d = *desc;
    LASER_REQUIRE(d.n_layers >= 0 && d.n_heads > 0 && d.n_pages > 0 && d.max_seqs > 0 && d.max_pages_per_seq > 0,
                  LASER_E_INVALID_ARG, "non-positive size in laser_kv_desc");
    LASER_REQUIRE(d.page_size == kPageSize, LASER_E_SHAPE, "page_size must be %d", kPageSize);
    LASER_REQUIRE(d.head_dim == 64 || d.head_dim == 128, LASER_E_SHAPE, "head_dim %d unsupported (64 or 128)", d.head_dim);
    KV* kv = new KV();
    kv->d = d;
    const size_t pool_elems = (size_t)std::max(d.n_layers, 1) * d.n_pages * kv->page_elems();
    const size_t bt = (size_t)d.max_seqs * d.max_pages_per_seq;
    auto fail = [&](int rc) { laser_kv_destroy(reinterpret_cast<laser_kv*>(kv)); return rc; };
#define KV_TRY(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) { set_error("%s: %s", #expr, hipGetErrorString(e_)); return fail(LASER_E_HIP); } } while (0)
    KV_TRY(hipMalloc((void**)&kv->kpages, pool_elems * 2));
    KV_TRY(hipMalloc((void**)&kv->klpages, pool_elems));
    KV_TRY(hipMalloc((void**)&kv->vpages, pool_elems * 2));
    KV_TRY(hipMalloc((void**)&kv->block_table, bt * 4));
    KV_TRY(hipMalloc((void**)&kv->len, (size_t)d.max_seqs * 4));
    KV_TRY(hipMalloc((void**)&kv->ids_dev, (size_t)kIdSlots * d.max_seqs * 4));
    KV_TRY(hipHostMalloc((void**)&kv->ids_pinned, (size_t)kIdSlots * d.max_seqs * 4));
    for (int i = 0; i < kIdSlots; ++i) KV_TRY(hipEventCreateWithFlags(&kv->ids_ev[i], hipEventDisableTiming));
    // Pages start as zeros: masked-out cache slots are multiplied by probability 0 in the value
    // product, which must not meet NaN/Inf bit patterns left in fresh memory.
    KV_TRY(hipMemsetAsync(kv->kpages, 0, pool_elems * 2, stream));
    KV_TRY(hipMemsetAsync(kv->klpages, 0, pool_elems, stream));
    KV_TRY(hipMemsetAsync(kv->vpages, 0, pool_elems * 2, stream));
    KV_TRY(hipMemsetAsync(kv->block_table, 0, bt * 4, stream));
    KV_TRY(hipMemsetAsync(kv->len, 0, (size_t)d.max_seqs * 4, stream));
    KV_TRY(hipStreamSynchronize(stream));
#undef KV_TRY
    kv->h_block_table.assign(bt, 0);
    kv->h_npages.assign(d.max_seqs, 0);
    kv->h_len_ub.assign(d.max_seqs, 0);
    kv->h_last_rows.assign(d.max_seqs, 0);
    kv->free_pages.resize(d.n_pages);
    for (int i = 0; i < d.n_pages; ++i) kv->free_pages[i] = d.n_pages - 1 - i;   // pop_back hands out 0,1,2,...
    *out = reinterpret_cast<laser_kv*>(kv);
    return LASER_OK;
}

extern "C" int laser_kv_destroy(laser_kv* h) {
    if (!h) return LASER_OK;
    KV* kv = reinterpret_cast<KV*>(h);
    (void)hipFree(kv->kpages); (void)hipFree(kv->klpages); (void)hipFree(kv->vpages); (void)hipFree(kv->block_table);
    (void)hipFree(kv->len); (void)hipFree(kv->ids_dev);
    if (kv->ids_pinned) (void)hipHostFree(kv->ids_pinned);
    for (int i = 0; i < kIdSlots; ++i) if (kv->ids_ev[i]) (void)hipEventDestroy(kv->ids_ev[i]);
    delete kv;
    return LASER_OK;
}

static int check_seq(const KV* kv, int seq) {
    LASER_REQUIRE(kv != nullptr, LASER_E_INVALID_ARG, "kv is NULL");
    LASER_REQUIRE(seq >= 0 && seq < kv->d.max_seqs, LASER_E_INVALID_ARG, "sequence slot %d outside 0..%d", seq, kv->d.max_seqs - 1);
    return LASER_OK;
}

extern "C" int laser_kv_seq_reserve(laser_kv* h, int seq, int n_tokens, void* stream) {
    KV* kv = reinterpret_cast<KV*>(h);
    int rc = check_seq(kv, seq);
    if (rc) return rc;
    LASER_REQUIRE(n_tokens >= 0, LASER_E_INVALID_ARG, "n_tokens < 0");
    const int need = (n_tokens + kPageSize - 1) / kPageSize;
    const int have = kv->h_npages[seq];
    if (need <= have) return LASER_OK;
    LASER_REQUIRE(need <= kv->d.max_pages_per_seq, LASER_E_OOM_PAGES, "slot %d needs %d pages, max_pages_per_seq is %d", seq, need, kv->d.max_pages_per_seq);
    LASER_REQUIRE((size_t)(need - have) <= kv->free_pages.size(), LASER_E_OOM_PAGES, "page pool exhausted: need %d more, %zu free", need - have, kv->free_pages.size());
    int32_t* row = kv->h_block_table.data() + (size_t)seq * kv->d.max_pages_per_seq;
    for (int p = have; p < need; ++p) { row[p] = kv->free_pages.back(); kv->free_pages.pop_back(); }
    kv->h_npages[seq] = need;
    // pageable source: the runtime stages it before returning, and the row is not modified again
    // until the next reserve/release of this slot, which enqueue behind this copy
    LASER_HIP_CHECK(hipMemcpyAsync(kv->block_table + (size_t)seq * kv->d.max_pages_per_seq + have, row + have,
                                   (size_t)(need - have) * 4, hipMemcpyHostToDevice, (hipStream_t)stream));
    return LASER_OK;
}

extern "C" int laser_kv_seq_release(laser_kv* h, int seq, void* stream) {
    KV* kv = reinterpret_cast<KV*>(h);
    int rc = check_seq(kv, seq);
    if (rc) return rc;
    int32_t* row = kv->h_block_table.data() + (size_t)seq * kv->d.max_pages_per_seq;
    for (int p = kv->h_npages[seq] - 1; p >= 0; --p) kv->free_pages.push_back(row[p]);
    kv->h_npages[seq] = 0;
    kv->h_len_ub[seq] = 0;
    kv->h_last_rows[seq] = 0;
    hipLaunchKernelGGL(fill_i32_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, kv->len + seq, 0, (size_t)1);
    LASER_HIP_CHECK(hipGetLastError());
    return LASER_OK;
}

extern "C" int laser_kv_seq_set_len(laser_kv* h, int seq, int len, void* stream) {
    KV* kv = reinterpret_cast<KV*>(h);
    int rc = check_seq(kv, seq);
    if (rc) return rc;
    LASER_REQUIRE(len >= 0 && len <= kv->h_npages[seq] * kPageSize, LASER_E_OOM_PAGES,
                  "length %d exceeds the %d tokens reserved for slot %d", len, kv->h_npages[seq] * kPageSize, seq);
    kv->h_len_ub[seq] = len;
    kv->h_last_rows[seq] = 0;
    hipLaunchKernelGGL(fill_i32_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, kv->len + seq, len, (size_t)1);
    LASER_HIP_CHECK(hipGetLastError());
    return LASER_OK;
}

extern "C" int laser_kv_import(laser_kv* h, int seq, int layer, const uint16_t* k, const uint16_t* v,
                               int n_tokens, void* stream) {
    KV* kv = reinterpret_cast<KV*>(h);
    int rc = check_seq(kv, seq);
    if (rc) return rc;
    LASER_REQUIRE(layer >= 0 && layer < kv->d.n_layers, LASER_E_INVALID_ARG, "layer %d out of range", layer);
    LASER_REQUIRE(n_tokens >= 0 && n_tokens <= kv->h_npages[seq] * kPageSize, LASER_E_OOM_PAGES,
                  "%d tokens exceed the capacity reserved for slot %d", n_tokens, seq);
    if (n_tokens == 0) return LASER_OK;
    LASER_REQUIRE(k && v, LASER_E_INVALID_ARG, "NULL k/v");
    const size_t total = (size_t)n_tokens * kv->d.n_heads * kv->d.head_dim;
    hipLaunchKernelGGL(kv_import_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       kv->kpages, kv->klpages, kv->vpages, kv->block_table + (size_t)seq * kv->d.max_pages_per_seq, k, v,
                       n_tokens, kv->d.n_heads, kv->d.head_dim, layer, kv->d.n_pages);
    LASER_HIP_CHECK(hipGetLastError());
    return LASER_OK;
}

extern "C" int laser_kv_read_lens(laser_kv* h, const int32_t* seq_ids, int B, int32_t* lens_out, void* stream) {
    KV* kv = reinterpret_cast<KV*>(h);
    LASER_REQUIRE(kv && (B == 0 || (seq_ids && lens_out)) && B >= 0, LASER_E_INVALID_ARG, "bad argument");
    for (int b = 0; b < B; ++b) { int rc = check_seq(kv, seq_ids[b]); if (rc) return rc; }
    std::vector<int32_t> all(kv->d.max_seqs);
    LASER_HIP_CHECK(hipMemcpyAsync(all.data(), kv->len, all.size() * 4, hipMemcpyDeviceToHost, (hipStream_t)stream));
    LASER_HIP_CHECK(hipStreamSynchronize((hipStream_t)stream));
    for (int b = 0; b < B; ++b) {
        lens_out[b] = all[seq_ids[b]];
        kv->h_len_ub[seq_ids[b]] = all[seq_ids[b]];
        kv->h_last_rows[seq_ids[b]] = 0;
    }
    return LASER_OK;
}

// laser_kv_commit and laser_kv_commit_tree (accept_path != NULL: compact the accepted branch first)
static int commit_impl(laser_kv* h, const int32_t* seq_ids, const int32_t* accept_len, const int32_t* accept_path, int B, int K,
                       void* stream) {
    KV* kv = reinterpret_cast<KV*>(h);
    LASER_REQUIRE(kv != nullptr && B >= 0, LASER_E_INVALID_ARG, "bad argument");
    if (B == 0) return LASER_OK;
    LASER_REQUIRE(seq_ids && accept_len, LASER_E_INVALID_ARG, "NULL argument");
    LASER_REQUIRE(B <= kv->d.max_seqs, LASER_E_INVALID_ARG, "B exceeds max_seqs");
    for (int b = 0; b < B; ++b) { int rc = check_seq(kv, seq_ids[b]); if (rc) return rc; }
    for (int b = 0; b < B; ++b) {
        // the device adds accept_len + 1 <= rows of the verify step before it
        LASER_REQUIRE(kv->h_last_rows[seq_ids[b]] > 0, LASER_E_INVALID_ARG,
                      "commit on slot %d without a verify step before it", seq_ids[b]);
        LASER_REQUIRE(!accept_path || kv->h_last_rows[seq_ids[b]] == K + 1, LASER_E_INVALID_ARG,
                      "slot %d: the verify step before this commit had %d rows, not K + 1 = %d", seq_ids[b], kv->h_last_rows[seq_ids[b]], K + 1);
    }
    const int32_t* ids_dev = nullptr;
    int rc = kv->stage_ids(seq_ids, B, (hipStream_t)stream, &ids_dev);
    if (rc) return rc;
    int max_rows = 0;
    for (int b = 0; b < B; ++b) {
        max_rows = std::max(max_rows, kv->h_last_rows[seq_ids[b]]);
        kv->h_len_ub[seq_ids[b]] += kv->h_last_rows[seq_ids[b]];
        kv->h_last_rows[seq_ids[b]] = 0;
    }
    if (accept_path && K > 0 && kv->d.n_layers > 0)
        hipLaunchKernelGGL(kv_compact_kernel, dim3(kv->d.n_heads, kv->d.n_layers, B), dim3(kv->d.head_dim), 0, (hipStream_t)stream,
                           kv->kpages, kv->klpages, kv->vpages, kv->block_table, kv->len, ids_dev, accept_len, accept_path, K,
                           kv->d.n_heads, kv->d.head_dim, kv->d.max_pages_per_seq, kv->d.n_pages);
    hipLaunchKernelGGL(commit_kernel, dim3((B + 63) / 64), dim3(64), 0, (hipStream_t)stream, kv->len, ids_dev, accept_len, B, max_rows - 1);
    LASER_HIP_CHECK(hipGetLastError());
    return LASER_OK;
}

extern "C" int laser_kv_commit(laser_kv* h, const int32_t* seq_ids, const int32_t* accept_len, int B, void* stream) {
    return commit_impl(h, seq_ids, accept_len, nullptr, B, 0, stream);
}

extern "C" int laser_kv_commit_tree(laser_kv* h, const int32_t* seq_ids, const int32_t* accept_len, const int32_t* accept_path,
                                    int B, int K, void* stream) {
    LASER_REQUIRE(K >= 0 && K <= LASER_MAX_DRAFT, LASER_E_INVALID_ARG, "K %d outside 0..%d", K, LASER_MAX_DRAFT);
    LASER_REQUIRE(B <= 0 || K == 0 || accept_path, LASER_E_INVALID_ARG, "accept_path is NULL");
    return commit_impl(h, seq_ids, accept_len, K > 0 ? accept_path : nullptr, B, K, stream);
}

extern "C" int laser_ctx_advance(int32_t* ctx_tail, int32_t* pending, const int32_t* out_tokens,
                                 const int32_t* accept_len, int B, int K, int n_max, void* stream) {
    LASER_REQUIRE(B >= 0 && K >= 0 && K <= LASER_MAX_DRAFT && n_max >= 1 && n_max <= LASER_MAX_NGRAM,
                  LASER_E_INVALID_ARG, "bad size");
    if (B == 0) return LASER_OK;
    LASER_REQUIRE(ctx_tail && pending && out_tokens && accept_len, LASER_E_INVALID_ARG, "NULL argument");
    hipLaunchKernelGGL(ctx_advance_kernel, dim3((B + 63) / 64), dim3(64), 0, (hipStream_t)stream,
                       ctx_tail, pending, out_tokens, accept_len, B, K, n_max);
    LASER_HIP_CHECK(hipGetLastError());
    return LASER_OK;
}
