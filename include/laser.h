/*
 * laser.h -- C ABI of the MI355X (gfx950) library for the per-step hot path of
 * retrieval-based Draft-then-Verify decoding with a Customized Retrieval Pool and Relaxed
 * Verification (arxiv 2408.05676, "LASER").
 *
 * One decoding step of one batch is
 *     laser_retrieve_drafts -> laser_verify_step -> laser_kv_commit (-> laser_ctx_advance)
 * all asynchronous on one HIP stream, with no device->host traffic.
 *
 * Conventions
 *   - Pointers are tagged [host] or [dev]. [dev] buffers are owned by the caller (for example
 *     PyTorch tensors) and only borrowed for the duration of the stream-ordered call.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream). Calls enqueue work and
 *     return; they synchronise only where stated.
 *   - Every function returns LASER_OK (0) or a negative LASER_E_* code; laser_last_error() gives a
 *     thread-local message for the last failure. Data-dependent outcomes (unknown key, no match,
 *     nothing accepted) are results, not errors.
 *   - Token ids are int32 >= 0; -1 pads. bf16 / fp16 = bfloat16 / IEEE half bit patterns in uint16.
 *   - Numerics: weights bf16 as given; activations that feed matrix products and the KV cache are
 *     fp16; accumulation, softmax, norms and the residual stream are fp32.
 *   - A handle must not be used from two streams or two host threads at the same time (the model
 *     handle owns activation workspace, the KV handle owns host-side page bookkeeping).
 */
#ifndef LASER_H
#define LASER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LASER_OK             0
#define LASER_E_INVALID_ARG (-1) /* null pointer, negative size, value out of its documented range */
#define LASER_E_SHAPE       (-2) /* model/cache shape the kernels do not support */
#define LASER_E_OOM_PAGES   (-3) /* KV page pool or a sequence's reserved capacity exhausted */
#define LASER_E_HIP         (-4) /* a HIP runtime call failed */
#define LASER_E_LIMIT       (-5) /* size beyond a documented maximum */

#define LASER_MAX_NGRAM   8      /* longest context suffix that can be indexed (n_max)            */
#define LASER_MAX_DRAFT   63     /* largest K (drafts per sequence per step); R = K+1 <= 64 rows    */
#define LASER_MAX_TOPK    8      /* largest k of the top-k condition                                */
#define LASER_MAX_TREE    32     /* largest K of laser_retrieve_tree (nodes of one retrieved token tree)           */
#define LASER_MAX_OWN_TEXT 4096  /* tokens of a sequence's own text a temporary-branch lookup takes */

/* acceptance rule selector (Sec. 3.4). rank = number of vocabulary entries ordered before the draft
 * (higher logit first, smaller id on ties); q = softmax probability of the draft at temperature 1. */
#define LASER_MODE_RV          0 /* Eq. 8: rank < k  and  q > p   (Eq. 4 greedy = k 1, p < 0)       */
#define LASER_MODE_RV_OR_TOP1  1 /* rank == 0  or  Eq. 8                                             */
#define LASER_MODE_TOPK_ONLY   2 /* Eq. 7 alone: rank < k                                            */
#define LASER_MODE_TOPP_ONLY   3 /* threshold-only ablation: rank == 0  or  q > p                    */

typedef struct laser_pool  laser_pool;   /* regrouped token pool + suffix index, device memory, library-owned */
typedef struct laser_model laser_model;  /* borrowed weight views + library-owned workspace and RoPE table     */
typedef struct laser_kv    laser_kv;     /* paged fp16 KV cache: page pool, block tables, lengths; library-owned */

const char* laser_last_error(void);
const char* laser_version(void);

/* ------------------------------------------------------------------------------------------------
 * Retrieval pool (Sec. 3.2: one pool per group of users/items, built from their earlier texts;
 * Sec. 3.3 Eq. 5: Retrieve(D, last n tokens, K)).
 *
 * laser_pool_build: groups the sequences by key (ascending key; supply order kept inside a key) into
 * one flat "regrouped pool" and indexes, for every key and every n in 1..n_max, each n-gram that
 * lies inside one sequence and is followed by at least one token of that sequence.
 *   tokens  [host] int32[seq_off[n_seq]]   all sequences back to back
 *   seq_off [host] int64[n_seq+1]          start of each sequence, ascending, seq_off[0] = 0
 *   seq_key [host] int64[n_seq]            opaque key (user / item / group id) of each sequence
 *   n_max   1..LASER_MAX_NGRAM
 * Host work (sorting, hashing) runs inside the call; device copies are enqueued on `stream` and the
 * call synchronises that stream before returning. Total tokens must stay below 2^32 - 1.
 * The pool is immutable afterwards. *out is written only on success.
 */
int laser_pool_build(const int32_t* tokens, const int64_t* seq_off, const int64_t* seq_key,
                     int64_t n_seq, int n_max, void* stream, laser_pool** out);
int laser_pool_destroy(laser_pool* pool);

/* Sizes of a built pool; any out pointer may be NULL. */
int laser_pool_info(const laser_pool* pool, int64_t* n_tokens, int64_t* n_keys,
                    int64_t* n_index_entries, int64_t* device_bytes);
/* Copy regrouped tokens [start, start+count) to host memory (synchronous; for checks and tools). */
int laser_pool_read_tokens(const laser_pool* pool, int64_t start, int64_t count, int32_t* out_host);

/* laser_retrieve_drafts (Sec. 3.3): for each of B contexts, try n = min(n_max, valid tail length)
 * down to n_min; at the first n whose n-gram occurs in the key's sub-pool, follow the most frequent
 * successor (ties -> smaller token id) among the surviving occurrences for up to K tokens; accept
 * that n if the chain has >= min_tokens tokens, otherwise keep the longest chain seen (ties ->
 * larger n).
 *   keys       [dev] int64[B]
 *   ctx_tail   [dev] int32[B][n_max]  last n_max context tokens, right-aligned, -1 padded on the left
 *   drafts     [dev] int32[B][K]      out: chain, -1 padded
 *   draft_len  [dev] int32[B]         out: 0..K
 *   match_n    [dev] int32[B]         out: suffix length used, 0 if nothing was found
 *   pool_index [dev] int64[B]         out: smallest regrouped-pool position e of a surviving occurrence
 *                                          (tokens e+1 .. e+draft_len are the drafts), -1 if none
 * n_max must not exceed the pool's n_max; 1 <= n_min <= n_max; 0 <= K <= LASER_MAX_DRAFT; B >= 0.
 * Results are exact (no hash false positives) and independent of scheduling.
 */
int laser_retrieve_drafts(const laser_pool* pool, const int64_t* keys, const int32_t* ctx_tail,
                          int B, int n_min, int n_max, int K, int min_tokens,
                          int32_t* drafts, int32_t* draft_len, int32_t* match_n,
                          int64_t* pool_index, void* stream);

/* laser_retrieve_drafts_temp: the same lookup with the temporary branch of Sec. 3.2 (the current prompt and
 * the text generated so far join the group's trie while this text is being generated, and leave it afterwards).
 * Row b of own_tokens counts as ONE MORE SEQUENCE of keys[b]'s sub-pool, placed after all of its pool sequences;
 * every rule of laser_retrieve_drafts applies unchanged to the enlarged sub-pool (occurrences need a successor
 * inside their sequence, so the context suffix at the very end of the own text is not one). Nothing is added to
 * the pool itself: the "branch" lives in the caller's buffer and ends with it. An unknown key searches the own
 * text alone.
 *   own_tokens [dev] int32[B][own_cap]  the sequence's text, oldest token first, left-aligned; normally its
 *                                       last tokens are ctx_tail
 *   own_len    [dev] int32[B]           tokens in each row (clamped to 0..own_cap)
 *   own_cap    1..LASER_MAX_OWN_TEXT    (longer texts: keep the most recent tokens, see laser_own_text_append)
 *   pool_index out: as above; if no surviving occurrence lies in the pool, -2 - (position in the own text row)
 * The own text is scanned by the lookup (no index): O(own_len * n) token compares per tried n. */
int laser_retrieve_drafts_temp(const laser_pool* pool, const int64_t* keys, const int32_t* ctx_tail,
                               const int32_t* own_tokens, const int32_t* own_len, int own_cap,
                               int B, int n_min, int n_max, int K, int min_tokens,
                               int32_t* drafts, int32_t* draft_len, int32_t* match_n,
                               int64_t* pool_index, void* stream);

/* laser_retrieve_tree (Sec. 3.3, tree-based drafting): like laser_retrieve_drafts, but instead of one chain the
 * sub-tree of the key's trie below the node the suffix reaches is returned, cut to its K most frequent nodes (the
 * paper's rule for a retrieval that returns more than K tokens: keep those of highest frequency). A node is a path of
 * successor tokens; its frequency is the number of occurrences of the suffix that continue with that path. Nodes are
 * taken best first among those whose parent is taken: higher frequency, then smaller depth, then the parent taken
 * earlier, then the smaller token id. The pseudo-sequence lists the taken nodes depth-first, the children of a node
 * in the order taken (higher frequency first).
 *   tree_tokens [dev] int32[B][K]  out: token of node i, -1 padded
 *   tree_parent [dev] int32[B][K]  out: pseudo-sequence index of node i's parent (< i), -1 for a child of the root
 *                                       (it follows the pending token) and for padding
 *   tree_freq   [dev] int32[B][K]  out, may be NULL: frequency of node i
 *   tree_len    [dev] int32[B]     out: nodes 0..K
 *   match_n     [dev] int32[B]     out: suffix length used (the first n from n_max down whose tree has >= min_tokens
 *                                       nodes, else the n of the largest tree seen), 0 if nothing was found
 * 0 <= K <= LASER_MAX_TREE; other arguments and limits as for laser_retrieve_drafts. */
int laser_retrieve_tree(const laser_pool* pool, const int64_t* keys, const int32_t* ctx_tail,
                        int B, int n_min, int n_max, int K, int min_tokens,
                        int32_t* tree_tokens, int32_t* tree_parent, int32_t* tree_freq,
                        int32_t* tree_len, int32_t* match_n, void* stream);

/* Device-side bookkeeping for the own text: appends the tokens a step emitted,
 * out_tokens[b][0..accept_len[b]] (as written by laser_verify_step), to row b; a row that would overflow drops
 * its oldest tokens first (sliding window of own_cap tokens). own_tokens / own_len [dev] in/out. A negative
 * accept_len[b] leaves row b unchanged. */
int laser_own_text_append(int32_t* own_tokens, int32_t* own_len, int own_cap, const int32_t* out_tokens,
                          const int32_t* accept_len, int B, int K, void* stream);

/* ------------------------------------------------------------------------------------------------
 * Target model (Sec. 2.1 Eq. 1/3, Sec. 3.4 Eq. 6: the LLM that yields K+1 distributions per pass).
 * Pre-norm decoder: RMSNorm, rotary positions (element i paired with i + head_dim/2), multi-head
 * causal attention, SwiGLU FFN, no biases, untied embedding / output head.
 * All weight pointers are [dev], row-major [out_features][in_features], bf16 unless noted, and
 * must stay valid and unchanged while the handle lives.
 */
typedef struct laser_model_desc {
    int32_t n_layers, d_model, n_heads, ffn, vocab;
    int32_t max_rows;       /* largest B*(K+1) any call will use (sizes the workspace)            */
    int32_t max_batch;      /* largest B                                                          */
    int32_t max_pos;        /* positions 0..max_pos-1 get a RoPE table entry                      */
    float   eps;            /* RMSNorm epsilon                                                    */
    float   rope_base;
    const uint16_t* wqkv;   /* [L][3d][d]  rows: query | key | value projection                   */
    const uint16_t* wo;     /* [L][d][d]                                                          */
    const uint16_t* wgu;    /* [L][2F][d]  rows: gate | up projection                             */
    const uint16_t* wdown;  /* [L][d][F]                                                          */
    const float*    g1;     /* [L][d] float32 pre-attention norm gain                             */
    const float*    g2;     /* [L][d] float32 pre-FFN norm gain                                   */
    const uint16_t* emb;    /* [V][d]                                                             */
    const uint16_t* wlm;    /* [V][d]                                                             */
    const float*    gf;     /* [d] float32 final norm gain                                        */
} laser_model_desc;

/* Supported: head_dim 64 or 128; d_model, ffn multiples of 128; vocab multiple of 16 (else
 * LASER_E_SHAPE). Allocates workspace and the RoPE table; synchronises `stream`. n_layers may be 0
 * (head-only use). Further allocations happen lazily, inside the first call that needs them:
 * with more than 16 rows a workspace for reduction-split partial results (max_rows * d_model * 32 bytes);
 * with more than 80 rows fp16 copies of the four projection matrices and of the head matrix (2 bytes per parameter:
 * the weight memory doubles) for the tiled many-row kernels. That call synchronises the stream; it fails with
 * LASER_E_HIP if the memory is not there and with LASER_E_LIMIT if a weight exceeds the fp16 range (|w| > 65280).
 * Option "f16_copies" = 0 makes no copies: the tiled kernels then widen the bf16 weights on the fly (slower). */
int laser_model_create(const laser_model_desc* desc, void* stream, laser_model** out);
int laser_model_destroy(laser_model* model);

/* ------------------------------------------------------------------------------------------------
 * Paged KV cache. A sequence slot owns a list of pages (page_size tokens each); `len` tokens are
 * committed, the next R slots are scratch for the step in flight. Pages are reserved from the host
 * without reading device state: the library keeps, per slot, an upper bound of `len`.
 * Storage per token, layer and channel: key fp16 + an 8-bit low part (the key is kept to about 14
 * significant bits, which the logit tolerance needs at 32 layers), value fp16: 5 bytes.
 */
typedef struct laser_kv_desc {
    int32_t n_layers, n_heads, head_dim;
    int32_t page_size;          /* tokens per page: 16                                            */
    int32_t n_pages;            /* pages in the pool (each page spans all layers and heads)       */
    int32_t max_seqs;           /* sequence slots 0..max_seqs-1                                   */
    int32_t max_pages_per_seq;
} laser_kv_desc;

int laser_kv_create(const laser_kv_desc* desc, void* stream, laser_kv** out);
int laser_kv_destroy(laser_kv* kv);
/* Make slot `seq` able to hold n_tokens tokens (committed + in flight). Grows only.
 * LASER_E_OOM_PAGES if the pool or max_pages_per_seq cannot cover it (nothing changes then). */
int laser_kv_seq_reserve(laser_kv* kv, int seq, int n_tokens, void* stream);
/* Return the slot's pages to the pool and set its length to 0. */
int laser_kv_seq_release(laser_kv* kv, int seq, void* stream);
/* Load externally produced keys/values (already rotated) for tokens [0, n_tokens) of one layer:
 * k, v [dev] fp16 [n_tokens][n_heads][head_dim]. Needs reserved capacity; does not change `len`. */
int laser_kv_import(laser_kv* kv, int seq, int layer, const uint16_t* k, const uint16_t* v,
                    int n_tokens, void* stream);
/* Set the committed length of a slot (after laser_kv_import, or to roll back). */
int laser_kv_seq_set_len(laser_kv* kv, int seq, int len, void* stream);
/* Read back the committed lengths of B slots (synchronises `stream`) and tighten the host bounds. */
int laser_kv_read_lens(laser_kv* kv, const int32_t* seq_ids /*[host] B*/, int B,
                       int32_t* lens_out /*[host] B*/, void* stream);

/* laser_verify_step (Eq. 3 / Eq. 6 forward, Eq. 4 / 7 / 8 acceptance, correction rule of Sec. 2.1).
 * For sequence b, rows r = 0..K hold the tokens [pending[b], drafts[b][0..K-1]] at positions
 * len+r; their keys/values go to cache slots len..len+K; row r attends to slots 0..len+r. The
 * output head and the acceptance rule are fused for every row count: logits are reduced to per-(row, vocabulary
 * chunk) partial statistics by the kernel that produces them and are never stored unless logits_dbg is given.
 * With B*(K+1) <= 16 the whole step is one
 * persistent cooperative kernel (see laser_model_set_option). Drafts j >= draft_len[b] are padding
 * (fed as token 0, never accepted).
 *   seq_ids    [host] int32[B]      KV slots, all different
 *   pending    [dev]  int32[B]      last emitted token of each sequence (not yet in the cache)
 *   drafts     [dev]  int32[B][K]
 *   draft_len  [dev]  int32[B]      0..K
 *   topk 1..LASER_MAX_TOPK, p, mode: see LASER_MODE_*
 *   accept_len [dev]  int32[B]      out: a = number of leading drafts accepted
 *   out_tokens [dev]  int32[B][K+1] out: drafts 0..a-1, then argmax of row a (smallest id on ties),
 *                                   then -1
 *   logits_dbg [dev]  float[B][K+1][V] or NULL
 * Needs (host bound of len) + K+1 <= reserved capacity for every slot, else LASER_E_OOM_PAGES.
 * Does not change `len`: call laser_kv_commit.
 */
int laser_verify_step(laser_model* model, laser_kv* kv, const int32_t* seq_ids,
                      const int32_t* pending, const int32_t* drafts, const int32_t* draft_len,
                      int B, int K, int topk, float p, int mode,
                      int32_t* accept_len, int32_t* out_tokens, float* logits_dbg, void* stream);

/* laser_verify_tree (Sec. 3.3 tree attention; Sec. 3.4: of the verified branches the longest one is accepted):
 * laser_verify_step for a token tree. Rows r = 1..K hold the nodes of the pseudo-sequence in order (row 0 the pending
 * token); node i sits at position len + depth(i), its key/value go to cache slot len + 1 + i, and it attends to the
 * committed cache, the pending token, its ancestors and itself -- never to a node of another branch. Node i is verified
 * iff its parent is (children of the root: always) and its token passes the acceptance rule against the distribution
 * of its parent's row; the accepted branch ends at the deepest verified node (the first in the pseudo-sequence among
 * equally deep ones).
 *   tree_tokens, tree_parent, tree_len  [dev] as written by laser_retrieve_tree (an entry of tree_parent that does
 *                not name an earlier node counts as -1; nodes past tree_len[b] are padding)
 *   accept_len  [dev] int32[B]      out: a = nodes on the accepted branch
 *   out_tokens  [dev] int32[B][K+1] out: the branch's tokens, then argmax of its last node's row (of row 0 if a = 0), then -1
 *   accept_path [dev] int32[B][K]   out: pseudo-sequence indices of the branch's nodes, root side first, then -1
 * A tree whose parent[i] = i - 1 is a chain and gives the results of laser_verify_step bit for bit: both calls choose
 * their path by the row count alone (at most 16 rows in all, B (K + 1) <= 16: the persistent few-row kernel, unless
 * option "fused" is 0). Follow with laser_kv_commit_tree. */
int laser_verify_tree(laser_model* model, laser_kv* kv, const int32_t* seq_ids,
                      const int32_t* pending, const int32_t* tree_tokens, const int32_t* tree_parent,
                      const int32_t* tree_len, int B, int K, int topk, float p, int mode,
                      int32_t* accept_len, int32_t* out_tokens, int32_t* accept_path,
                      float* logits_dbg, void* stream);

/* Output head + acceptance alone, on given final-normed hidden states h [dev] fp16 [B][K+1][d]. */
int laser_verify_head(laser_model* model, const uint16_t* h, const int32_t* drafts,
                      const int32_t* draft_len, int B, int K, int topk, float p, int mode,
                      int32_t* accept_len, int32_t* out_tokens, float* logits_dbg, void* stream);

/* laser_verify_head_static: laser_verify_head for callers that cannot allocate device memory -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc. Same inputs, outputs and results as
 * laser_verify_head with up to 16 rows (no logits_dbg), but the per-(row, vocabulary chunk) partial statistics that
 * pass from the streaming kernel to the acceptance kernel live in a device array that is part of the library image
 * (1.19 MiB on every GPU the library runs on, until the process ends) instead of the model handle's workspace; the
 * call itself allocates and frees nothing. Limits: B*(K+1) <= 16 rows and at most 1024 vocabulary chunks (every
 * model handle satisfies the second); beyond them LASER_E_LIMIT. All calls on one GPU share that
 * array: calls that overlap on one GPU (two streams, two threads) race; calls on one stream are ordered. */
int laser_verify_head_static(laser_model* model, const uint16_t* h, const int32_t* drafts,
                             const int32_t* draft_len, int B, int K, int topk, float p, int mode,
                             int32_t* accept_len, int32_t* out_tokens, void* stream);

/* laser_kv_commit (Sec. 2.1: drafts behind the first failing position are dropped):
 * len[seq_ids[b]] += accept_len[b] + 1, i.e. the pending token and the accepted drafts become
 * permanent; later slots are dead and get overwritten by the next step.
 *   seq_ids [host] int32[B];  accept_len [dev] int32[B] (values 0..K of the verify call before it; -1 commits
 *   nothing for that sequence, which is how a finished sequence idles in laser_generate; values outside -1..K are
 *   cut to that range on the device, so that a length never passes the bound its pages were reserved against)
 * A commit without a verify step on the same slots before it returns LASER_E_INVALID_ARG.
 */
int laser_kv_commit(laser_kv* kv, const int32_t* seq_ids, const int32_t* accept_len, int B,
                    void* stream);

/* laser_kv_commit_tree: laser_kv_commit after laser_verify_tree. The keys/values of the accepted branch's nodes are
 * moved from their slots len + 1 + accept_path[b][j] to len + 1 + j (every layer and head) -- their rotary positions
 * already are len + 1 + j --, then len[seq_ids[b]] += accept_len[b] + 1. K must be the K of that verify call. */
int laser_kv_commit_tree(laser_kv* kv, const int32_t* seq_ids, const int32_t* accept_len,
                         const int32_t* accept_path, int B, int K, void* stream);

/* Device-side bookkeeping between steps: append the emitted tokens out_tokens[b][0..accept_len[b]]
 * to the context tail (keeping the last n_max tokens) and make the last of them the new pending
 * token.  ctx_tail [dev] int32[B][n_max] in/out, pending [dev] int32[B] out. */
int laser_ctx_advance(int32_t* ctx_tail, int32_t* pending, const int32_t* out_tokens,
                      const int32_t* accept_len, int B, int K, int n_max, void* stream);

/* laser_generate: the whole generation of a batch (Sec. 3.1: retrieval, drafting and verification repeated until the
 * text is complete; Sec. 2.1 for what a step keeps). Every step is laser_retrieve_drafts (or laser_retrieve_tree /
 * laser_retrieve_drafts_temp) -> laser_verify_step (or laser_verify_tree) -> device-side bookkeeping -> laser_kv_commit
 * (or laser_kv_commit_tree), enqueued on `stream` without any device->host traffic; only once every
 * opts->check_every steps the host waits for the stream and reads a counter of finished sequences to stop early. A
 * sequence finishes when it has emitted max_new_tokens tokens or eos_token (which is kept); it then stays in the batch
 * without changing. Tokens a step emits beyond either limit are dropped (and not committed).
 *   pool        may be NULL: plain one-token-per-step decoding (K is ignored)
 *   seq_ids     [host] int32[B]; every slot needs reserved capacity >= its length bound + max_new_tokens + K + 1
 *   keys        [dev] int64[B]; ctx_tail [dev] int32[B][n_max] and pending [dev] int32[B] in/out (as laser_ctx_advance)
 *   own_tokens / own_len [dev] in/out, with opts->own_cap > 0: the temporary branch (chain drafts only); else NULL
 *   gen_tokens  [dev] int32[B][max_new_tokens] out: the emitted tokens, -1 padded;  gen_len [dev] int32[B] out
 *   counters    [dev] int32[B][4] out: steps taken, draft tokens offered, draft tokens kept, draft tokens accepted
 *   steps_run   [host] out: steps enqueued;  retrieve_ms [host] out, may be NULL: summed time of the retrieval kernels
 * Synchronises `stream` before returning; allocates and frees its own small device buffers. */
typedef struct laser_generate_opts {
    int32_t K, n_min, n_max, min_tokens;   /* drafting (see laser_retrieve_drafts)                              */
    int32_t tree;                          /* 0: chain drafts, 1: token trees (K <= LASER_MAX_TREE)             */
    int32_t topk; float p; int32_t mode;   /* acceptance rule (LASER_MODE_*)                                    */
    int32_t max_new_tokens, eos_token;     /* eos_token -1: none                                                */
    int32_t check_every;                   /* steps between two looks at the finished counter, >= 1             */
    int32_t own_cap;                       /* > 0: capacity of own_tokens rows (temporary branch)               */
} laser_generate_opts;
int laser_generate(laser_model* model, laser_kv* kv, const laser_pool* pool, const int32_t* seq_ids,
                   const int64_t* keys, int32_t* ctx_tail, int32_t* pending, int32_t* own_tokens,
                   int32_t* own_len, int B, const laser_generate_opts* opts, int32_t* gen_tokens,
                   int32_t* gen_len, int32_t* counters, int* steps_run, float* retrieve_ms, void* stream);

/* Options: "fused" = 1 (default) lets laser_verify_step use the persistent whole-step kernel when
 * B*(K+1) <= 16; 0 forces the general multi-kernel path. Both compute the same function.
 * "split_ffn" = 1 makes the many-row (more than 80 rows) gate/up product take its input rows as two
 * fp16 planes like the other products (default 0: single fp16 there, which halves that product's
 * matrix work; with up to 80 rows the input is always split).
 * "ksplit_qkv", "ksplit_o", "ksplit_down" = 0 (default), 1, 2 or 4: number of parts the reduction of
 * that projection is cut into on the many-row path (0: chosen from the launch shape; a value the
 * shape or the workspace cannot take falls back to 1). The parts are added in a fixed order by the
 * kernel that follows, so a given setting is deterministic; different settings may differ in the
 * last bits. Tuning and test knobs: the default is what the benchmark measures.
 * "f16_copies" = 1 (default) or 0: see laser_model_create.
 * "mid_waves" = 0 (default: chosen per launch shape), 4 or 8: waves per workgroup of the weight-streaming
 * GEMM used with 17..80 rows.
 * "attn_whole_min" = 0 (default: half the number of compute units) or a count: from this many (sequence, head,
 * 16-row query tile) triples on, the general path's attention walks a context in one workgroup instead of
 * splitting it into 256-token parts that a second kernel merges.
 * "attn_waves" = 0 (default: eight when an unsplit launch has fewer than two workgroups per compute unit, else four),
 * 4 or 8: waves of a workgroup that share the pages of an unsplit context.
 * Unknown names and out-of-range values return LASER_E_INVALID_ARG. */
int laser_model_set_option(laser_model* model, const char* name, int value);
/* Phase trace of the persistent kernel (option "fused_trace" = 1): thread 0 of every workgroup stamps
 * the 100 MHz wall clock before and after every grid barrier. Copies the stamps of the most recent
 * launch to out[nwg][cap] (host, int64) and synchronises `stream`. */
int laser_model_read_trace(laser_model* model, void* stream, long long* out, int max_elems, int* nwg, int* cap);
/* Synchronises `stream` and reports whether a bounded wait inside the persistent kernel ever gave up
 * (*aborted = 1): results after that are invalid and the handle must be destroyed. */
int laser_model_status(laser_model* model, void* stream, int* aborted);

/* Timing of the dominant kernel of laser_verify_step (the gate/up projection GEMM, which streams the
 * largest weight matrix of every layer): between begin and end, HIP events are recorded on the
 * call's stream right before and after each of its launches, up to max_records launches.
 * laser_profile_end synchronises `stream` and returns the summed kernel time and the launch count. */
int laser_profile_begin(laser_model* model, int max_records);
int laser_profile_end(laser_model* model, void* stream, float* total_ms, int* n_launches);

/* Measured peaks of the device, so that roofline fractions can be quoted against what the chip delivers as well
 * as against its datasheet. Neither touches any model state; both synchronise `stream` before they return.
 * laser_probe_hbm: buf [dev] is caller-owned scratch of `bytes` bytes (a multiple of 32, at least 1 MiB; use
 *   more than the 256 MiB last-level cache). The read probe streams all of it `reps` times (read_gbs = bytes
 *   read per second / 1e9); the copy probe copies its first half onto its second half `reps` times
 *   (copy_gbs = bytes read + written per second / 1e9). The buffer's second half is overwritten.
 * laser_probe_mfma_f16: a register-resident loop of 32x32x16 fp16 matrix instructions on every SIMD (16 waves per
 *   compute unit, four independent accumulators each); scratch [dev] is any device buffer of at least 4 bytes
 *   (not written); tflops = executed flops per second / 1e12. */
int laser_probe_hbm(void* buf, size_t bytes, int reps, void* stream, float* read_gbs, float* copy_gbs);
int laser_probe_mfma_f16(void* scratch, int reps, void* stream, float* tflops);
/* laser_probe_launch: the floor under a latency-bound kernel such as the draft lookup -- the mean time of `reps`
 * back-to-back launches of a kernel of `blocks` wavefronts that does nothing (microseconds per launch). */
int laser_probe_launch(int blocks, int reps, void* stream, float* us_per_launch);
/* laser_probe_exchange: what one all-to-all exchange between the phases of the persistent few-row kernel costs on this
 * device: a cooperative launch of one workgroup per compute unit repeats `iters` times { write-through store into a
 * fresh region; wait for it; grid barrier (counter + flag); read values other workgroups stored } and the mean time of
 * one round is returned in microseconds. *errors counts stale values read and expired (bounded) waits: it must be 0.
 * scratch [dev]: caller-owned, at least 4096 + iters * 2048 * (compute units) bytes; it is overwritten. */
int laser_probe_exchange(void* scratch, size_t bytes, int iters, void* stream, float* us_per_exchange, int* errors);

#ifdef __cplusplus
}
#endif
#endif /* LASER_H */
