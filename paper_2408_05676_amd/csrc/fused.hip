// Persistent whole-step kernel for the few-row regime (M = B*(K+1) <= 16 rows): one cooperative
// launch runs embedding, every decoder layer, the final norm, the output head and the acceptance
// rule (Eq. 3/6 forward; Eq. 4/7/8 + correction rule). It exists because at these shapes a layer's
// weights stream in ~60 us, so kernel boundaries and latency-bound helper kernels would cost as much
// as the streaming itself.
//
// Structure: grid = one workgroup of 8 waves per compute unit. Phases are separated by a grid
// barrier (one agent-scope atomic counter + a separate flag line); per layer:
//     QKV(+RoPE) | attention | O-proj(+residual) | gate/up(+SwiGLU) | down(+residual)
// * Weight streaming: a GEMM unit is a 16-feature tile (or a pair of tiles); the 8 waves of a
//   workgroup split its reduction dimension, the four lanes of a weight row reading 64 contiguous bytes
//   per instruction (the MFMA operands of weights and activations take the same k order), partial sums meet in LDS. Each wave keeps 12-16 KiB of weights in
//   flight in a register ring and issues the first steps of the NEXT phase while the barrier
//   resolves, so HBM stays busy (weights never depend on activations). The few activation rows are
//   staged into LDS once per workgroup and phase instead of being re-read per step.
// * RMSNorm never materialises: producers publish x*gain (fp16) plus per-workgroup partial sums of
//   squares; consumers multiply their accumulators by rsqrt(mean square) (a per-row scalar commutes
//   with the product).
// * Cross-workgroup exchange without cache flushes: the chip has one L2 per XCD and agent-scope
//   fences cost ~18 us here. Instead every exchanged buffer is WRITE-ONCE per launch (a fresh
//   address range per layer and phase), written with agent-scope (write-through) stores and read
//   with ordinary cached loads after the barrier: no L2 can hold a stale copy of a line it has never
//   read, and kernel boundaries clean the caches between launches.
// * Attention reads committed cache pages (slots < len) with ordinary loads and the R new rows from
//   the exchange buffers; the wave that owns the new tile also copies it into the cache pages.
//   Context splits are merged by the last workgroup to arrive (per-(sequence, head) counter).
// Every wait is bounded: a barrier that does not resolve within ~5 s raises the abort flag and all
// workgroups leave the kernel.
#include <algorithm>
#include <cmath>

#include "head_part.h"
#include "mfma.h"
#include "state.h"

namespace laser {

constexpr int FT = 512;             // threads per workgroup
constexpr int FWAVES = 8;
constexpr int AW = 8;               // waves per workgroup that take attention pages
constexpr int PPW = 2;              // consecutive pages per wave and context split (16 pages = 256 tokens per split)
constexpr int KTOP = LASER_MAX_TOPK;

struct FusedArgs {
    const uint16_t *wqkv, *wo, *wgu, *wdown, *emb, *wlm;
    const float *g1, *g2, *gf;
    int L, d, H, dh, F, V;
    float eps;
    const float2* rope;
    uint16_t *kpages, *vpages;
    uint8_t* klpages;
    const int32_t *block_table, *lens;
    int mpps, n_pages;
    const int32_t *seq_ids, *pending, *drafts, *draft_len;
    // Token trees (Sec. 3.3): parent != NULL. drafts / draft_len then hold the nodes of the pseudo-sequence and their
    // count, parent[b][i] the node's parent (tree_parent_of), row_pos_g / row_anc_g [M] each row's position (committed
    // length + depth) and the rows of its sequence it attends to (bit j: row j), accept_path the third output.
    const int32_t* parent;
    const int32_t* row_pos_g;
    const unsigned long long* row_anc_g;
    int32_t* accept_path;
    int B, K, R, M;
    // exchange buffers (write-once per launch)
    float* xbuf;        // [2L+1][16][d]
    uint16_t* xgbuf;    // [2L+1][16][d]   high plane of x * gain
    uint8_t* xglbuf;    // [2L+1][16][d]   8-bit low plane: x * gain = xgbuf + xglbuf / 4096 (split operands, see mfma.h)
    float* ssbuf;       // [2L+1][nwg][16]
    uint16_t *qbuf, *knew, *attn;          // [L][16][d]
    uint16_t* vnew;     // [L][16][H][dh][16]  new values in the cache's page layout (channel-major): entry
                        // (b * npp + i) holds the new rows of sequence b that fall into its i-th page from len / 16
                        // on (npp = 1 if R == 1, else 2; B * npp <= 16 because B * R <= 16)
    uint16_t* qlbuf;                       // [L][16][d]      fp16 low plane of the queries
    uint8_t *knewl, *attnl;                // [L][16][d]      8-bit low planes of the new keys and of the attention output
    uint16_t* act;      // [L][16][F]
    float* apart;       // [L][B*H][nsplit][32 + 16*dh]
    int* acount;        // [L][B*H]   (self-resetting)
    int nsplit;
    int xs_steps;       // reduction steps (of 128) whose activations fit the LDS staging area, single plane
    int xs_steps2;      // the same for split activations (fp16 high plane + 8-bit low plane)
    // head
    float *hp_max, *hp_sum; int32_t* hp_arg; float* hp_topv; int32_t* hp_topi; float* hp_lx;
    int topk, mode; float p;
    int32_t *accept_len, *out_tokens; float* logits_dbg;
    // sync
    unsigned long long *bar_count, *bar_flag; unsigned long long epoch0;
    int* abort_flag;
    long long* trace;     // optional [nwg][trace_cap] wall-clock stamps (100 MHz) of thread 0
    int trace_cap;
};

// ---- agent-scope (write-through) stores for exchanged data ----------------------------------------
__device__ inline void st_u32(void* p, uint32_t v) {
    __hip_atomic_store(reinterpret_cast<uint32_t*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_f32(float* p, float v) { st_u32(p, __float_as_uint(v)); }
// two neighbouring floats (8-byte aligned) as one store
__device__ inline void st_f32x2(float* p, float v0, float v1) {
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(p),
                       (unsigned long long)__float_as_uint(v0) | ((unsigned long long)__float_as_uint(v1) << 32),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_i32(int* p, int v) { st_u32(p, (uint32_t)v); }
__device__ inline void st_u16(void* p, uint16_t v) {
    __hip_atomic_store(reinterpret_cast<uint16_t*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline uint32_t pack_h2(float a, float b) { return (uint32_t)f32_to_f16(a) | ((uint32_t)f32_to_f16(b) << 16); }

constexpr int MAX_UNITS = 6;         // 16-row weight tiles one wave slot can accumulate per phase
struct Shared {
    float att_m[AW][16], att_l[AW][16];
    float rs[16];                         // rsqrt(mean square) per row
    float ss_acc[16][32];
    int row_pos[16], row_b[16];
    int seq_slot[16], seq_len[16];        // per sequence of the batch: cache slot, committed length
    int flag;                             // barrier outcome / last-arriver broadcast
    int row_ok[LASER_MAX_DRAFT + 1], row_arg[LASER_MAX_DRAFT + 1];
    union alignas(16) {
        float red[MAX_UNITS][FWAVES][4][64];   // per (unit slot, wave) partial tiles   48 KiB
        float att_o[AW][16][128];                  // attention wave merge                  64 KiB
    };
};
// Staged activations start right behind `red` and run to the end of the launch's dynamic LDS; they
// overlap the tail of att_o, which is never live at the same time.
constexpr size_t XS_OFFSET = offsetof(Shared, red) + sizeof(float) * MAX_UNITS * FWAVES * 4 * 64;

// optional finer stamps inside the GEMM phases of layer `layer`: slot = 3 * phase + {0: staged, 1: streamed, 2: epilogue done}
// Stamps exist only in the TR = true instantiation of the kernel: even a never-taken branch around a
// store makes the compiler's wait counters conservative at its join, which would stall the streaming.
template <bool TR>
__device__ inline void stamp_fine(const FusedArgs& a, int layer, int slot) {
    if constexpr (!TR) return;
    if (a.trace && threadIdx.x == 0 && layer >= 0) {
        const int i = 2 * (5 * a.L + 2) + 4 + 16 * layer + slot;
        if (i < a.trace_cap) a.trace[(size_t)blockIdx.x * a.trace_cap + i] = wall_clock64();
    }
}
template <bool TR>
__device__ inline void stamp(const FusedArgs& a, int& n) {
    if constexpr (!TR) return;
    if (a.trace && threadIdx.x == 0) {
        if (n < a.trace_cap) a.trace[(size_t)blockIdx.x * a.trace_cap + n] = wall_clock64();
        ++n;
    }
}

// Every wave waits until its own exchange stores have completed (the workgroup barrier alone only
// orders LDS; completion of a write-through store takes a full memory round trip), then thread 0
// arrives. `prefetch` issues the next phase's first weight steps right after the arrival, so they
// travel while the barrier resolves without delaying the arrival itself.
// The flag every workgroup polls exists BAR_FLAGS times, 256 bytes apart, workgroup w polling copy w % BAR_FLAGS:
// 256 pollers of one address measured 1 % slower per step than 8 per address.
constexpr int BAR_FLAGS = 32;
template <class Prefetch>
__device__ inline bool grid_sync(const FusedArgs& a, Shared& sh, unsigned long long& epoch, Prefetch&& prefetch) {
    ++epoch;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const unsigned long long e = a.epoch0 + epoch;
    bool last = false;
    if (threadIdx.x < 64) {                 // wave 0: lane 0 arrives; the last arriver's lanes raise the flags
        int lastf = 0;
        if (threadIdx.x == 0) {
            const unsigned long long old = __hip_atomic_fetch_add(a.bar_count, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            lastf = old + 1 == e * (unsigned long long)gridDim.x;
        }
        lastf = __shfl(lastf, 0);
        last = lastf != 0;
        if (last)
            for (int x = threadIdx.x; x < BAR_FLAGS; x += 64)
                __hip_atomic_store(a.bar_flag + 32 * x, e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    prefetch();
    if (threadIdx.x == 0) {
        int ok = 1;
        if (!last) {
            long spins = 0;
            while (__hip_atomic_load(a.bar_flag + 32 * (blockIdx.x % BAR_FLAGS), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < e) {
                __builtin_amdgcn_s_sleep(1);
                if ((++spins & 1023) == 0) {
                    if (spins > 8000000L || __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
                        __hip_atomic_store(a.abort_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        ok = 0;
                        break;
                    }
                }
            }
        }
        sh.flag = ok;
    }
    __syncthreads();
    return sh.flag != 0;
}

// ---- weight streaming -------------------------------------------------------------------------------
enum { PH_QKV = 0, PH_O = 1, PH_GU = 2, PH_DOWN = 3, PH_HEAD = 4 };

struct Phase {
    const uint16_t* W;    // matrix of this layer
    int kind, Kd;
    int planes;           // planes of its activations: 2 = split (fp16 high + 8-bit low), 1 = single fp16
};

__device__ inline int count_mine(int n, int first, int stride) { return first < n ? (n - 1 - first) / stride + 1 : 0; }

// A *unit* is one 16-row weight tile streamed over this wave's share of the reduction dimension.
// Units of a wave slot in a phase (all waves of a workgroup share them, splitting k, except in the
// output head where every wave owns whole tiles):
//   QKV : per owned index i (of d/16): the two tiles of one rotary pair of q or k, then (after all
//         pairs) one tile of v  -> 3 units per index, so every workgroup streams the same bytes
//   O, DOWN : one tile per owned index
//   GU  : pair items (gate tile + up tile of the same 16 features), two streams per step
//   HEAD: vocabulary tiles, indexed by global wave id
__device__ inline int n_units(const FusedArgs& a, int kind) {
    const int nwg = gridDim.x, w = blockIdx.x;
    if (kind == PH_QKV) return 3 * count_mine(a.d / 16, w, nwg);
    if (kind == PH_GU) return count_mine(a.F / 16, w, nwg);
    if (kind == PH_HEAD) return count_mine(a.V / 16, w * FWAVES + (int)(threadIdx.x >> 6), nwg * FWAVES);
    return count_mine(a.d / 16, w, nwg);
}

// first weight row of stream `st` of unit `u`
__device__ inline int unit_row(const FusedArgs& a, int kind, int u, int st) {
    const int nwg = gridDim.x, w = blockIdx.x;
    if (kind == PH_QKV) {
        const int c = count_mine(a.d / 16, w, nwg);
        if (u < 2 * c) {
            const int item = w + (u >> 1) * nwg;      // rotary pair: index over q pairs, then k pairs
            const int per = a.d / 32;                 // pairs per projection
            const int grp = item / per, idx = item % per;
            const int pph = a.dh / 32;                // pairs per head: features (i, i + dh/2)
            const int h = idx / pph, j = idx % pph;
            return grp * a.d + h * a.dh + j * 16 + (u & 1) * (a.dh / 2);
        }
        return 2 * a.d + (w + (u - 2 * c) * nwg) * 16;
    }
    if (kind == PH_GU) return st * a.F + (w + u * nwg) * 16;
    if (kind == PH_HEAD) return (w * FWAVES + (int)(threadIdx.x >> 6) + u * nwg * FWAVES) * 16;
    return (w + u * nwg) * 16;
}

// One step of one weight tile: 16 rows x 128 reduction elements. Fragment c of lane (r = lane & 15, g = lane >> 4)
// holds elements 32 c + 8 g .. + 7 of row r, so the four lanes of a row read 64 contiguous bytes per instruction
// and an instruction touches 16 half lines (a lane reading its own 64 contiguous bytes would spread every
// instruction over 32 lines, each requested four times per step).
__device__ inline void load_w(Frag8 (&f)[4], const uint16_t* p) {
#pragma unroll
    for (int c = 0; c < 4; ++c) f[c].u = *reinterpret_cast<const uint4*>(p + c * 32);
}

// The reduction dimension is processed in chunks whose activations fit the LDS staging area
// (xs_steps steps of 128 elements for the launch's row count); chunk c of a Kd-long reduction:
__device__ inline int n_chunks(const FusedArgs& a, const Phase& ph) {
    const int xs = ph.planes == 2 ? a.xs_steps2 : a.xs_steps;
    return (ph.Kd / 128 + xs - 1) / xs;
}
__device__ inline void chunk_range(const FusedArgs& a, const Phase& ph, int c, int& cs0, int& cs1) {
    const int steps = ph.Kd / 128, nch = n_chunks(a, ph);
    cs0 = steps * c / nch;
    cs1 = steps * (c + 1) / nch;
}

struct WaveWork {         // wave-uniform description of this wave's share of one chunk of a phase
    int cs0, ncs;         // the chunk: first step, steps
    int ks0, nks;         // this wave's steps inside it
    int n_my, T;          // units, total steps
};
__device__ inline WaveWork wave_work(const FusedArgs& a, const Phase& ph, int chunk) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    WaveWork w;
    int cs1;
    chunk_range(a, ph, chunk, w.cs0, cs1);
    w.ncs = cs1 - w.cs0;
    if (ph.kind == PH_HEAD) { w.ks0 = w.cs0; w.nks = w.ncs; }
    else {
        w.ks0 = w.cs0 + w.ncs * wave / FWAVES;
        w.nks = w.cs0 + w.ncs * (wave + 1) / FWAVES - w.ks0;
    }
    w.n_my = __builtin_amdgcn_readfirstlane(n_units(a, ph.kind));
    w.T = w.n_my * w.nks;
    return w;
}

__device__ inline const uint16_t* w_ptr(const FusedArgs& a, const Phase& ph, int u, int st, int ks, int lane) {
    return ph.W + (size_t)(unit_row(a, ph.kind, u, st) + (lane & 15)) * ph.Kd + ks * 128 + (lane >> 4) * 8;
}

// Weight streaming through a register ring. A step (128 reduction elements) of a phase with NA
// streams occupies NA weight fragments (4 x 16 B per lane each); the ring holds DS steps, so DS-1
// steps of weights are in flight while one is consumed. The activation operand is NOT loaded per step from
// global memory: measured on this chip, per-step activation loads (L2 hits) cut the weight streaming rate by
// 30-45 % because they share the vector-memory path; the phase's activations are staged into LDS once per
// workgroup and read from there. The streaming loop is kept free of branches around vector-memory instructions
// (past the wave's last step it re-requests one cached line and skips the arithmetic), because the wait
// counters are exact only in straight-line code; finished units leave their partial sums in LDS
// inside the loop and every epilogue runs after it.

// What survives a phase boundary: the weights issued ahead for the next phase (see prime_steps).
constexpr int RING_SLOTS = 6;
struct Ring {
    Frag8 f[RING_SLOTS][4];   // slot (step % DS) * NA + stream
};
// Per phase: DS = steps the ring holds, PF = steps requested while the grid barrier in front of the phase resolves
// (the other DS - 1 - PF follow the staging requests). Chosen by sweeps inside ONE run of the nine-row 7B launch (the
// machines differ by more than the settings do), milliseconds per step relative to the setting kept:
//   single-tile phases (QKV, O, head): DS 2 / PF 1, i.e. ONE step (4 KiB per wave) in flight; DS 3 / PF 2 +0.4 % (O),
//     +0.7 % (QKV), DS 4 / PF 2 +2.2 % (all three together), PF 0 +1.5 % (QKV), +1.9 % (O); the head is indifferent;
//   down: DS 3 / PF 2 (DS 2 / PF 1 +0.5 %, DS 4 / PF 2 or 3 +0.8 %, DS 5 / PF 4 equal);
//   gate/up (NA = 2): DS 3 / PF 2, the whole ring inside the barrier (PF 1 +1.1 %, PF 0 +2.3 %, DS 2 / PF 1 +0.9 %;
//     a fourth step needs 8 ring slots and costs 3-4 % in spills).
// Deeper rings do not stream faster: a compute unit's memory queues hold less than 8 waves x 16 KiB, and whatever is
// queued in front of the staged activations or the epilogue's stores delays them.
constexpr int DS_QKV = 2, PF_QKV = 1, DS_O = 2, PF_O = 1, DS_GU = 3, PF_GU = 2, DS_DOWN = 3, PF_DOWN = 2, DS_HEAD = 2, PF_HEAD = 1;
static_assert(DS_QKV <= RING_SLOTS && DS_O <= RING_SLOTS && DS_DOWN <= RING_SLOTS && DS_HEAD <= RING_SLOTS && 2 * DS_GU <= RING_SLOTS,
              "the ring holds DS steps of NA fragments");

// Issue the weights of this wave's steps T0 .. T1-1 (of the first DS-1) of chunk `chunk` of phase `ph` into
// their ring slots. Weights never depend on activations, so the first PF steps are issued while the grid
// barrier in front of the phase resolves and the others (if any) right behind the requests that stage the
// phase's activations. The loads are unconditional (steps past the wave's last one re-request one cached line),
// so that the number of vector-memory instructions issued here is a compile-time constant: stage_wait counts
// on it.
template <int NA, int T0, int T1>
__device__ inline void prime_steps(const FusedArgs& a, const Phase& ph, int chunk, Ring& R) {
    const int lane = threadIdx.x & 63;
    const WaveWork w = wave_work(a, ph, chunk);
    const int nks = max(w.nks, 1);
    const uint16_t* park = reinterpret_cast<const uint16_t*>(a.gf);
#pragma unroll
    for (int t = T0; t < T1; ++t) {
        const bool on = t < w.T;
        const int tc = on ? t : 0;
#pragma unroll
        for (int s = 0; s < NA; ++s)
            load_w(R.f[t * NA + s], on ? w_ptr(a, ph, tc / nks, s, w.ks0 + tc % nks, lane) : park);
    }
}
// vector-memory instructions prime_steps<NA, T0, T1> issues
template <int NA, int T0, int T1> struct PrimeCount { static constexpr int value = (T1 - T0) * NA * 4; };

// Copy rows 0..M-1, steps cs0 .. cs0+ncs-1 of the fp16 activations X[16][Kd] into LDS and, for split
// activations, of their 8-bit low plane Xlo[16][Kd] right behind them in the same LDS row: a row is
// ncs*256 bytes (+ ncs*128 bytes) + 16 bytes of padding, so that the 16-byte operand reads of 16 rows
// fall into distinct banks. The copy uses loads that write LDS directly (16 bytes per lane, lane l of an
// instruction lands at the instruction's LDS base + 16 l): a block of 64 consecutive pieces of one row and
// plane per instruction, the blocks dealt round-robin to the waves. No registers hold the data, so all of a
// wave's blocks are in flight at once and the addressing is a handful of scalar operations per block. The
// caller waits for them with stage_wait.
__device__ inline void stage_x(const FusedArgs& a, uint4* xs, const uint16_t* X, const uint8_t* Xlo, int Kd, int cs0, int ncs) {
    typedef void __attribute__((address_space(3))) * lptr_t;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int hi_p = ncs * 16, lo_p = Xlo ? ncs * 8 : 0;              // 16-byte pieces of a row, per plane
    const int bh = (hi_p + 63) >> 6, bpr = bh + ((lo_p + 63) >> 6);    // 64-piece blocks per row: high plane, both
    const int stride = hi_p + lo_p + 1, total = a.M * bpr;
    const char* xh = reinterpret_cast<const char*>(X) + (size_t)cs0 * 256;
    const char* xl = reinterpret_cast<const char*>(Xlo ? (const void*)Xlo : (const void*)X) + (size_t)cs0 * 128;
    int row = 0, blk = wave;
    while (blk >= bpr) { blk -= bpr; ++row; }
    for (int j = wave; j < total; j += FWAVES) {
        const bool low = blk >= bh;
        const int b0 = (low ? blk - bh : blk) * 64;                    // first piece of the block inside its plane
        const int n = (low ? lo_p : hi_p) - b0;                        // pieces the plane has from there on (>= 1)
        const char* src = low ? xl + (size_t)row * Kd : xh + (size_t)row * Kd * 2;
        uint4* dst = xs + row * stride + (low ? hi_p : 0) + b0;
        // Written as assembly so that the compiler does not track the request: it would wait for it (and for every
        // weight load behind it) at the first unrelated reuse of the address registers. The caller's stage_wait is the
        // wait that counts. m0 = the block's LDS byte address; one wait state between writing m0 and its use. The
        // compiler warns that m0 is a reserved register which it does not preserve around the statement: nothing
        // else in this kernel uses m0 (no other LDS-direct load, no indirect register indexing, no message).
        const uint32_t lds_at = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lptr_t)dst);
        const char* g = src + (size_t)(b0 + lane) * 16;
        if (lane < n)
            asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_at) : "memory", "m0");
        blk += FWAVES;
        while (blk >= bpr) { blk -= bpr; ++row; }
    }
}
// The same copy restricted to what THIS wave reads in the streaming loop: every row's pieces of the wave's own steps
// ks0 .. ks0+nks-1 of the chunk (all waves of a workgroup walk the same units and split the reduction dimension, so no
// wave reads another wave's columns). The wave's own wait (stage_wait) is then all the synchronisation the staged
// data needs: no workgroup barrier between staging and streaming.
__device__ inline void stage_x_own(const FusedArgs& a, uint4* xs, const uint16_t* X, const uint8_t* Xlo, int Kd, const WaveWork& w) {
    typedef void __attribute__((address_space(3))) * lptr_t;
    const int lane = threadIdx.x & 63;
    const int hi_p = w.ncs * 16, lo_p = Xlo ? w.ncs * 8 : 0;
    const int stride = hi_p + lo_p + 1;
    const int k0 = w.ks0 - w.cs0;                                      // first own step inside the chunk
    const int nh = w.nks * 16, nl = Xlo ? w.nks * 8 : 0;              // own pieces per row: high plane, low plane
    const char* xh = reinterpret_cast<const char*>(X) + (size_t)w.ks0 * 256;
    const char* xl = reinterpret_cast<const char*>(Xlo ? (const void*)Xlo : (const void*)X) + (size_t)w.ks0 * 128;
    for (int row = 0; row < a.M; ++row) {
        for (int b0 = 0; b0 < nh; b0 += 64) {
            uint4* dst = xs + row * stride + k0 * 16 + b0;
            const uint32_t lds_at = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lptr_t)dst);
            const char* g = xh + (size_t)row * Kd * 2 + (size_t)(b0 + lane) * 16;
            if (lane < nh - b0)
                asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_at) : "memory", "m0");
        }
        for (int b0 = 0; b0 < nl; b0 += 64) {
            uint4* dst = xs + row * stride + hi_p + k0 * 8 + b0;
            const uint32_t lds_at = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lptr_t)dst);
            const char* g = xl + (size_t)row * Kd + (size_t)(b0 + lane) * 16;
            if (lane < nl - b0)
                asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_at) : "memory", "m0");
        }
    }
}
// Waits for this wave's staging requests, leaving the N vector-memory instructions issued after them (the
// weight steps of prime_steps) in flight: the counter retires in issue order.
template <int N>
__device__ inline void stage_wait() {
    static_assert(N >= 0 && N < 64, "the wait counter has six bits");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Streams one chunk: this wave's units x steps, partial sums of finished units to sh.red
// (stored on the first chunk, accumulated on later ones; slot = unit * NA + stream).
template <int NA, int DS, bool SPLIT>
__device__ inline void stream_chunk(const FusedArgs& a, Shared& sh, const uint4* xs, const Phase& ph,
                                    const WaveWork& w, bool first, Ring& R) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int r = lane & 15, g = lane >> 4;
    if (w.T > 0) {
        Frag8 (&A)[RING_SLOTS][4] = R.f;             // the ring: steps 0 .. DS-2 are on their way (prime_steps)
        const uint16_t* wp[NA];             // this lane's pointers to the next step to request
        int jn = 0, kn = 0;                 // (unit, step) of that step
        // Past the last step the pointers park on one lane-uniform, always-valid address, so the
        // surplus requests of the padded loop cost a single cached line each.
        const uint16_t* park = reinterpret_cast<const uint16_t*>(a.gf);
        auto set_unit = [&](int j) {
#pragma unroll
            for (int s = 0; s < NA; ++s) wp[s] = w_ptr(a, ph, j, s, w.ks0, lane);
        };
        auto advance = [&]() {              // scalar control only
            if (kn + 1 < w.nks) {
                ++kn;
#pragma unroll
                for (int s = 0; s < NA; ++s) wp[s] += 128;
            } else if (jn + 1 < w.n_my) {
                kn = 0; ++jn; set_unit(jn);
            } else {
#pragma unroll
                for (int s = 0; s < NA; ++s) wp[s] = park;
            }
        };
        auto request = [&](int slot) {      // weights of the next step, then advance
#pragma unroll
            for (int s = 0; s < NA; ++s) load_w(A[slot * NA + s], wp[s]);
            advance();
        };
        set_unit(0);
        // steps 0 .. DS-2 have been requested by prime_steps: move the request pointers behind them
#pragma unroll
        for (int t = 0; t < DS - 1; ++t) advance();
        // this lane's activation operand: row r (padding rows read row 0; their results are dropped)
        const uint4* xrow = xs + (r < a.M ? r : 0) * (w.ncs * (SPLIT ? 24 : 16) + 1);
        const uint4* xl = xrow + (w.ks0 - w.cs0) * 16 + g;                     // fragment c of step k: xl[16 k + 4 c]
        const uint2* xlo = reinterpret_cast<const uint2*>(xrow + w.ncs * 16) + (w.ks0 - w.cs0) * 16 + g;   // 8-bit low plane behind the high plane: xlo[16 k + 4 c]
        float4_t acc[NA], acl[NA];
#pragma unroll
        for (int s = 0; s < NA; ++s) { acc[s] = float4_t{0.f, 0.f, 0.f, 0.f}; acl[s] = float4_t{0.f, 0.f, 0.f, 0.f}; }
        int k = 0, junit = 0;
        for (int t0 = 0; t0 < w.T; t0 += DS) {
#pragma unroll
            for (int j = 0; j < DS; ++j) {
                request((j + DS - 1) % DS);                   // unconditional: step t0 + j + DS - 1, clamped
                if (t0 + j < w.T) {                           // no vector-memory instructions inside this branch
                    Frag8 Bf[4], Bl[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) Bf[c].u = xl[k * 16 + c * 4];
                    if constexpr (SPLIT) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            const uint2 lo8 = xlo[k * 16 + c * 4];
                            b8x8_to_f16x8(lo8.x, lo8.y, Bl[c]);
                        }
                    }
#pragma unroll
                    for (int s = 0; s < NA; ++s) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) bf16x8_to_f16x8(A[j * NA + s][c]);
#pragma unroll
                        for (int c = 0; c < 4; ++c) acc[s] = mfma_16x16x32(A[j * NA + s][c], Bf[c], acc[s]);
                        if constexpr (SPLIT) {
#pragma unroll
                            for (int c = 0; c < 4; ++c) acl[s] = mfma_16x16x32(A[j * NA + s][c], Bl[c], acl[s]);
                        }
                    }
                    if (++k == w.nks) {
#pragma unroll
                        for (int s = 0; s < NA; ++s)
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                float* slot = &sh.red[junit * NA + s][wave][i][lane];
                                const float t = SPLIT ? acc[s][i] + acl[s][i] * kLoInv : acc[s][i];
                                *slot = first ? t : *slot + t;
                            }
#pragma unroll
                        for (int s = 0; s < NA; ++s) { acc[s] = float4_t{0.f, 0.f, 0.f, 0.f}; acl[s] = float4_t{0.f, 0.f, 0.f, 0.f}; }
                        k = 0;
                        ++junit;
                    }
                }
            }
        }
    } else if (first) {
        for (int j = 0; j < w.n_my * NA; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) sh.red[j][wave][i][lane] = 0.f;
    }
}

// Streams a whole phase: for every chunk stage its activations, stream, and issue the next chunk's
// first weights before the staging barrier. On return sh.red holds every unit's partial sums and
// all waves have passed a workgroup barrier.
template <int NA, bool SPLIT, bool TR, int DS, int PF1, bool OWN = true>
__device__ inline void stream_phase(const FusedArgs& a, Shared& sh, uint4* xs, const Phase& ph,
                                    const uint16_t* __restrict__ X, const uint8_t* __restrict__ Xlo, Ring& R,
                                    int trace_layer = -1, int trace_slot = 0) {
    const int nch = n_chunks(a, ph);
    for (int c = 0; c < nch; ++c) {
        const WaveWork w = wave_work(a, ph, c);
        if (c > 0) __syncthreads();                     // every wave has finished reading the previous chunk
        if (c == 0) stamp_fine<TR>(a, trace_layer, trace_slot + 2);
        if constexpr (OWN) stage_x_own(a, xs, X, SPLIT ? Xlo : nullptr, ph.Kd, w);
        else stage_x(a, xs, X, SPLIT ? Xlo : nullptr, ph.Kd, w.cs0, w.ncs);
        // the ring's remaining steps travel behind the staging requests (chunk 0: steps 0 .. PF1-1 were issued
        // inside the barrier)
        // (the fences keep the compiler from moving weight loads in front of the staging requests: stage_wait
        // relies on the issue order)
        __builtin_amdgcn_sched_barrier(0);
        if (c == 0) {
            prime_steps<NA, PF1, DS - 1>(a, ph, c, R);
            __builtin_amdgcn_sched_barrier(0);
            stage_wait<PrimeCount<NA, PF1, DS - 1>::value>();
        } else {
            prime_steps<NA, 0, DS - 1>(a, ph, c, R);
            __builtin_amdgcn_sched_barrier(0);
            stage_wait<PrimeCount<NA, 0, DS - 1>::value>();
        }
        if constexpr (!OWN) __syncthreads();     // shared staging: every wave's pieces have landed
        if (c == 0) stamp_fine<TR>(a, trace_layer, trace_slot);
        stream_chunk<NA, DS, SPLIT>(a, sh, xs, ph, w, c == 0, R);
    }
    __syncthreads();
    stamp_fine<TR>(a, trace_layer, trace_slot + 1);
}

// Split-K reduction and epilogue of a GEMM phase, 128 threads: thread -> (row, two features).
// epi(unit, row, f0, v[NA][2]) receives the finished sums of features f0, f0+1 of the unit's tile(s).
template <int NA, class Epi>
__device__ inline void reduce_epilogue(const FusedArgs& a, Shared& sh, int n_my, Epi&& epi) {
    if (threadIdx.x < 128) {
        const int row = threadIdx.x >> 3, f0 = (threadIdx.x & 7) * 2;
        for (int j = 0; j < n_my; ++j) {
            float v[NA][2];
#pragma unroll
            for (int s = 0; s < NA; ++s)
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int f = f0 + q;
                    const int ln = (f >> 2) * 16 + row, i = f & 3;
                    float t = 0.f;
#pragma unroll
                    for (int wv = 0; wv < FWAVES; ++wv) t += sh.red[j * NA + s][wv][i][ln];
                    v[s][q] = t;
                }
            if (row < a.M) epi(j, row, f0, v);      // padding rows publish nothing (nobody reads rows >= M of an exchange buffer)
        }
    }
    __syncthreads();        // sh.red is free again (it shares LDS with the attention buffers)
}

// rs[row] = rsqrt(mean square + eps) from the per-workgroup partial sums of one norm point.
// ss_issue starts the loads (8 per thread) so that they travel with the phase's weights;
// ss_finish reduces them in a fixed order after the streaming loop.
__device__ inline void ss_issue(const float* ss /*[nwg][16]*/, float (&v)[8]) {
    const int nwg = gridDim.x, row = threadIdx.x & 15, part = threadIdx.x >> 4;      // 32 parts
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        // unconditional load (see stage_x); the value is first looked at in ss_finish, after the streaming
        v[i] = ss[(size_t)min(part + 32 * i, nwg - 1) * 16 + row];
    }
}
__device__ inline void ss_finish(const FusedArgs& a, Shared& sh, const float (&v)[8]) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) t += ((int)(threadIdx.x >> 4) + 32 * i < (int)gridDim.x) ? v[i] : 0.f;
    sh.ss_acc[threadIdx.x & 15][threadIdx.x >> 4] = t;
    __syncthreads();
    if (threadIdx.x < 16) {
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < 32; ++j) s += sh.ss_acc[threadIdx.x][j];
        sh.rs[threadIdx.x] = rsqrtf(s / (float)a.d + a.eps);
    }
    __syncthreads();
}

// publish this workgroup's partial sum of squares (threads < 128 hold one row each, 8 threads per row)
__device__ inline void publish_ss(Shared& sh, float* ss_out /*[16] of this workgroup*/, float mine) {
    if (threadIdx.x < 128) sh.ss_acc[threadIdx.x >> 3][threadIdx.x & 7] = mine;
    __syncthreads();
    if (threadIdx.x < 16) {
        float t = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) t += sh.ss_acc[threadIdx.x][j];
        st_f32(ss_out + threadIdx.x, t);
    }
    __syncthreads();
}

// ---- attention ---------------------------------------------------------------------------------------
// Block-table entries of this wave's pages of attention item `item` (clamped to a valid item and valid pages, so the
// loads are unconditional). They do not depend on the layer's activations: the first item's are requested while the
// grid barrier in front of the attention phase resolves, a later item's at the end of the item before it, which
// takes one memory round trip out of every item.
__device__ inline void attn_pages(const FusedArgs& a, const Shared& sh, int item, int (&pg)[PPW]) {
    const int n_items = a.B * a.H * a.nsplit, wave = threadIdx.x >> 6;
    item = min(item, n_items - 1);
    const int split = item % a.nsplit, b = item / a.nsplit / a.H;
    const int n_pages = (sh.seq_len[b] + a.R + kPageSize - 1) / kPageSize;
    const int32_t* bt = a.block_table + (size_t)sh.seq_slot[b] * a.mpps;
    const int pbase = (split * AW + wave) * PPW;
#pragma unroll
    for (int pp = 0; pp < PPW; ++pp) pg[pp] = bt[min(pbase + pp, n_pages - 1)];
}

template <int DH, bool TR, bool TREE>
__device__ inline void attention_phase(const FusedArgs& a, Shared& sh, int layer, int (&pg_next)[PPW]) {
    constexpr int NC32 = DH / 32, NC16 = DH / 16;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 15, g = lane >> 4;
    const int S = a.nsplit, n_items = a.B * a.H * S;
    const float scale = rsqrtf((float)DH);
    const size_t lo = (size_t)layer * 16 * a.d;
    const uint16_t* qb = a.qbuf + lo;
    const uint16_t* qlb = a.qlbuf + lo;
    const uint16_t* kn = a.knew + lo;
    const uint8_t* knl = a.knewl + lo;
    const uint16_t* vn = a.vnew + lo * kPageSize;
    uint16_t* ob = a.attn + lo;
    uint8_t* obl = a.attnl + lo;
    const int PSZ = 32 + 16 * DH;

    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int split = item % S, bh = item / S, h = bh % a.H, b = bh / a.H;
        const int slot = sh.seq_slot[b];
        const int len = sh.seq_len[b];
        // Pages are taken at their cache positions, PPW consecutive pages per wave and a fixed AW*PPW pages per split,
        // and a page that holds new rows is composed from the cache (slots < len) and the exchange
        // buffers (slots len .. len+R-1). The arithmetic a row sees therefore depends only on its own
        // position, never on how many rows are verified with it or on the host's length bound: a token
        // verified as a draft gets bit-identical logits to the same token decoded one at a time.
        const int n_pages = (len + a.R + kPageSize - 1) / kPageSize;

        float m_run = -INFINITY, l_run = 0.f;
        float4_t acc[NC16];
#pragma unroll
        for (int c = 0; c < NC16; ++c) acc[c] = float4_t{0.f, 0.f, 0.f, 0.f};
        if (wave < AW) {
            const int pbase = (split * AW + wave) * PPW;
            if (pbase < n_pages) {
                // One round trip: the query fragments and every key / value fragment (the block-table entries of this
                // wave's pages were requested ahead). All addresses of (2) are formed before its first load is issued, and
                // the scheduling fences keep anything else (in particular reloads of spilled pointers, which
                // would wait for all earlier loads) out of the load block.
                int pg[PPW];
#pragma unroll
                for (int pp = 0; pp < PPW; ++pp) pg[pp] = pg_next[pp];       // requested ahead (attn_pages)
                Frag8 bq[NC32], bql[NC32];
                // token tree (Sec. 3.3): which new rows query row r sees (bit j: row j of the sequence), itself and its
                // ancestors; loaded with the fragments
                const unsigned long long* ancp = a.row_anc_g + b * a.R + min(r, a.R - 1);     // TREE only
                const size_t qo = (size_t)(b * a.R + min(r, a.R - 1)) * a.d + (size_t)h * DH + g * 8;
                const uint16_t *qp = qb + qo, *qlp = qlb + qo;
                Frag8 ak[PPW][NC32];
                uint2 akl[PPW][NC32];               // 8-bit low plane of the keys, widened right before use
                Frag4 bv[PPW][NC16], nv[PPW][NC16];
                const int npp = a.R == 1 ? 1 : 2, pg0 = len / kPageSize;
                // A key slot at or past len is a NEW row: its lane reads the exchange buffer instead of the cache
                // page (pointer select, same registers). New values come from the page-shaped exchange buffer
                // and are merged token by token below.
                const uint16_t *kp[PPW], *vp[PPW], *nvp[PPW];
                const uint8_t* klp[PPW];
                size_t pbase_off[PPW];
                bool p_new[PPW];
#pragma unroll
                for (int pp = 0; pp < PPW; ++pp) {
                    const int p = min(pbase + pp, n_pages - 1);
                    p_new[pp] = p >= pg0;
                    const size_t base = (((size_t)layer * a.n_pages + pg[pp]) * a.H + h) * kPageSize * DH;
                    pbase_off[pp] = base;
                    const int ks = p * kPageSize + r;                   // this lane's key slot
                    const size_t ko = (size_t)(b * a.R + min(max(ks - len, 0), a.R - 1)) * a.d + (size_t)h * DH + g * 8;
                    kp[pp] = ks >= len ? kn + ko : a.kpages + base + (size_t)r * DH + g * 8;
                    klp[pp] = ks >= len ? knl + ko : a.klpages + base + (size_t)r * DH + g * 8;
                    vp[pp] = a.vpages + base + (size_t)r * kPageSize + 4 * g;
                    // pages without new rows read one shared line instead (the loads stay unconditional)
                    const int pi = min(max(p - pg0, 0), npp - 1);
                    nvp[pp] = p >= pg0 ? vn + ((size_t)(b * npp + pi) * a.H + h) * kPageSize * DH + (size_t)r * kPageSize + 4 * g : vn;
                }
                __builtin_amdgcn_sched_barrier(0);
                unsigned anc = 0;
                if constexpr (TREE) anc = (unsigned)*ancp;
#pragma unroll
                for (int c = 0; c < NC32; ++c) bq[c].u = *reinterpret_cast<const uint4*>(qp + c * 32);
#pragma unroll
                for (int c = 0; c < NC32; ++c) bql[c].u = *reinterpret_cast<const uint4*>(qlp + c * 32);
#pragma unroll
                for (int pp = 0; pp < PPW; ++pp) {
#pragma unroll
                    for (int c = 0; c < NC32; ++c) ak[pp][c].u = *reinterpret_cast<const uint4*>(kp[pp] + c * 32);
#pragma unroll
                    for (int c = 0; c < NC32; ++c) akl[pp][c] = *reinterpret_cast<const uint2*>(klp[pp] + c * 32);
#pragma unroll
                    for (int c = 0; c < NC16; ++c) bv[pp][c].u = *reinterpret_cast<const uint2*>(vp[pp] + (size_t)c * 16 * kPageSize);
#pragma unroll
                    for (int c = 0; c < NC16; ++c) nv[pp][c].u = *reinterpret_cast<const uint2*>(nvp[pp] + (p_new[pp] ? (size_t)c * 16 * kPageSize : 0));
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int pp = 0; pp < PPW; ++pp) {
                    const int p = pbase + pp, s0 = p * kPageSize;       // s0: first slot of the page
                    if (p >= n_pages) continue;
                    // new rows' values replace the cache's (unconditional selects: nothing here may be sunk into a branch)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int c = 0; c < NC16; ++c) bv[pp][c].h[j] = (s0 + 4 * g + j >= len) ? nv[pp][c].h[j] : bv[pp][c].h[j];
                    if (s0 + kPageSize > len) {                         // the page holds new rows
                        const size_t base = pbase_off[pp];
                        const int ks = s0 + r;
                        // this wave owns the page: store its new rows into the cache for later steps
                        if (ks >= len && ks < len + a.R) {
                            uint16_t* kd = a.kpages + base + (size_t)r * DH + g * 8;
                            uint8_t* kld = a.klpages + base + (size_t)r * DH + g * 8;
#pragma unroll
                            for (int c = 0; c < NC32; ++c) *reinterpret_cast<uint4*>(kd + c * 32) = ak[pp][c].u;
#pragma unroll
                            for (int c = 0; c < NC32; ++c) *reinterpret_cast<uint2*>(kld + c * 32) = akl[pp][c];
                        }
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int vs = s0 + 4 * g + j;
                            if (vs >= len && vs < len + a.R) {
#pragma unroll
                                for (int c = 0; c < NC16; ++c)
                                    a.vpages[base + (size_t)(c * 16 + r) * kPageSize + 4 * g + j] = bv[pp][c].h[j];
                            }
                        }
                    }
                    // both operands split: hi.hi + 2^-12 (hi.lo + lo.hi), in the order the general path uses
                    float4_t s = float4_t{0.f, 0.f, 0.f, 0.f}, sl = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int c = 0; c < NC32; ++c) s = mfma_16x16x32(ak[pp][c], bq[c], s);
#pragma unroll
                    for (int c = 0; c < NC32; ++c) sl = mfma_16x16x32(ak[pp][c], bql[c], sl);
#pragma unroll
                    for (int c = 0; c < NC32; ++c) {
                        Frag8 kl;
                        b8x8_to_f16x8(akl[pp][c].x, akl[pp][c].y, kl);
                        sl = mfma_16x16x32(kl, bq[c], sl);
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) s[i] += sl[i] * kLoInv;
                    float sv[4], mx = -INFINITY;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int ts = s0 + 4 * g + i;                 // slot of this score's key
                        // chain: query row r sits at slot len + r and sees everything up to itself; tree: committed slots
                        // are visible to every query row, new rows by the mask (bit ts - len)
                        const bool vis = TREE ? (r < a.R) && (ts < len || (ts < len + a.R && ((anc >> ((ts - len) & 31)) & 1u)))
                                              : (r < a.R) && (ts <= len + r);
                        sv[i] = vis ? s[i] * scale : -INFINITY;
                        mx = fmaxf(mx, sv[i]);
                    }
                    mx = fmaxf(mx, __shfl_xor(mx, 16));
                    mx = fmaxf(mx, __shfl_xor(mx, 32));
                    const float m_new = fmaxf(m_run, mx);
                    const float alpha = (m_new == -INFINITY) ? 1.f : __expf(m_run - m_new);
                    Frag4 pa;
                    float rsum = 0.f;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float pv = (sv[i] == -INFINITY) ? 0.f : __expf(sv[i] - m_new);
                        rsum += pv;
                        pa.h[i] = f32_to_f16(pv);
                    }
                    rsum += __shfl_xor(rsum, 16);
                    rsum += __shfl_xor(rsum, 32);
                    l_run = l_run * alpha + rsum;
                    m_run = m_new;
                    float al[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) al[i] = __shfl(alpha, 4 * g + i);
#pragma unroll
                    for (int c = 0; c < NC16; ++c) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) acc[c][i] *= al[i];
                        acc[c] = mfma_16x16x16(pa, bv[pp][c], acc[c]);
                    }
                }
            }
            stamp_fine<TR>(a, layer, 12);
            if (g == 0) { sh.att_m[wave][r] = m_run; sh.att_l[wave][r] = l_run; }
#pragma unroll
            for (int c = 0; c < NC16; ++c)
#pragma unroll
                for (int i = 0; i < 4; ++i) sh.att_o[wave][4 * g + i][c * 16 + r] = acc[c][i];
        }
        __syncthreads();
        float* part = a.apart + (((size_t)layer * a.B * a.H + bh) * S + split) * PSZ;
        // merge the waves: thread t -> (q, channel pair)
        for (int idx = threadIdx.x; idx < 16 * DH / 2; idx += FT) {
            const int q = idx / (DH / 2), c = (idx % (DH / 2)) * 2;
            float M = -INFINITY;
#pragma unroll
            for (int w = 0; w < AW; ++w) M = fmaxf(M, sh.att_m[w][q]);
            float Lq = 0.f, O0 = 0.f, O1 = 0.f;
            if (M != -INFINITY) {
#pragma unroll
                for (int w = 0; w < AW; ++w) {
                    const float f = __expf(sh.att_m[w][q] - M);
                    Lq += sh.att_l[w][q] * f;
                    O0 += sh.att_o[w][q][c] * f;
                    O1 += sh.att_o[w][q][c + 1] * f;
                }
            }
            if (S == 1) {
                if (q < a.R) {
                    uint32_t hi;
                    uint16_t lw;
                    split_pack_h2_b8(Lq > 0.f ? O0 / Lq : 0.f, Lq > 0.f ? O1 / Lq : 0.f, hi, lw);
                    const size_t o = (size_t)(b * a.R + q) * a.d + (size_t)h * DH + c;
                    st_u32(ob + o, hi);
                    st_u16(obl + o, lw);
                }
            } else {
                if (c == 0) { st_f32(part + q, M); st_f32(part + 16 + q, Lq); }
                st_f32x2(part + 32 + q * DH + c, O0, O1);
            }
        }
        if (S > 1) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's partial stores have completed
            __syncthreads();
            stamp_fine<TR>(a, layer, 13);
            if (threadIdx.x == 0) {
                int* cnt = a.acount + (size_t)layer * a.B * a.H + bh;
                const int old = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                sh.flag = (old == S - 1) ? 1 : 0;
                if (old == S - 1) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            __syncthreads();
            stamp_fine<TR>(a, layer, 14);
            if (sh.flag) {                   // last to arrive: combine the S partials of (b, h)
                const float* pbase = a.apart + (((size_t)layer * a.B * a.H + bh) * S) * PSZ;
                for (int idx = threadIdx.x; idx < 16 * DH / 2; idx += FT) {
                    const int q = idx / (DH / 2), c = (idx % (DH / 2)) * 2;
                    // the partials of up to 8 splits travel together (unconditional, clamped loads): a loop
                    // with one dependent round trip per split would cost more than the attention itself
                    float M = -INFINITY, Lq = 0.f, O0 = 0.f, O1 = 0.f;
                    for (int s0 = 0; s0 < S; s0 += 8) {
                        float pm[8], pl[8];
                        float2 po[8];
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            const float* ps = pbase + (size_t)min(s0 + j, S - 1) * PSZ;
                            pm[j] = ps[q]; pl[j] = ps[16 + q];
                            po[j] = *reinterpret_cast<const float2*>(ps + 32 + q * DH + c);
                        }
                        float Mn = M;
#pragma unroll
                        for (int j = 0; j < 8; ++j) if (s0 + j < S) Mn = fmaxf(Mn, pm[j]);
                        if (Mn != -INFINITY) {
                            const float f0 = __expf(M - Mn);           // M = -inf on the first group: exp gives 0
                            Lq *= f0; O0 *= f0; O1 *= f0;
#pragma unroll
                            for (int j = 0; j < 8; ++j)
                                if (s0 + j < S) {
                                    const float f = __expf(pm[j] - Mn);
                                    Lq += pl[j] * f; O0 += po[j].x * f; O1 += po[j].y * f;
                                }
                        }
                        M = Mn;
                    }
                    if (q < a.R) {
                        uint32_t hi;
                        uint16_t lw;
                        split_pack_h2_b8(Lq > 0.f ? O0 / Lq : 0.f, Lq > 0.f ? O1 / Lq : 0.f, hi, lw);
                        const size_t o = (size_t)(b * a.R + q) * a.d + (size_t)h * DH + c;
                        st_u32(ob + o, hi);
                        st_u16(obl + o, lw);
                    }
                }
            }
        }
        attn_pages(a, sh, item + gridDim.x, pg_next);
        __syncthreads();
    }
}

// ---- output head: per-wave vocabulary tiles, running statistics in registers ----------------------
__device__ inline bool hbefore(float v, int i, float w, int j) { return v > w || (v == w && i < j); }

// KD: entries of the list (the call's k <= KD <= KTOP): a two-entry list is all the paper's default k = 2 needs, and
// the merges below cost in proportion to KD squared.
template <int KD>
struct HStat {
    float mx, sum, lx;
    int arg;
    float tv[KD];
    int ti[KD];
    __device__ void init() {
        mx = -INFINITY; sum = 0.f; lx = -INFINITY; arg = 0x7FFFFFFF;
#pragma unroll
        for (int j = 0; j < KD; ++j) { tv[j] = -INFINITY; ti[j] = 0x7FFFFFFF; }
    }
    __device__ void push_top(float v, int n) {
        if (!hbefore(v, n, tv[KD - 1], ti[KD - 1])) return;
        tv[KD - 1] = v; ti[KD - 1] = n;
#pragma unroll
        for (int j = KD - 1; j > 0; --j)
            if (hbefore(tv[j], ti[j], tv[j - 1], ti[j - 1])) {
                const float fv = tv[j]; tv[j] = tv[j - 1]; tv[j - 1] = fv;
                const int fi = ti[j]; ti[j] = ti[j - 1]; ti[j - 1] = fi;
            }
    }
    __device__ void add(float v, int n) {
        if (v > mx) { sum = sum * __expf(mx - v) + 1.f; mx = v; arg = n; }
        else sum += __expf(v - mx);
        push_top(v, n);
    }
    __device__ void merge_xor(int off) {
        const float omx = __shfl_xor(mx, off), osum = __shfl_xor(sum, off), olx = __shfl_xor(lx, off);
        const int oarg = __shfl_xor(arg, off);
        float otv[KD]; int oti[KD];
#pragma unroll
        for (int j = 0; j < KD; ++j) { otv[j] = __shfl_xor(tv[j], off); oti[j] = __shfl_xor(ti[j], off); }
        merge(omx, osum, olx, oarg, otv, oti);
    }
    __device__ void merge(float omx, float osum, float olx, int oarg, const float (&otv)[KD], const int (&oti)[KD]) {
        const float M = fmaxf(mx, omx);
        if (M != -INFINITY) sum = sum * __expf(mx - M) + osum * __expf(omx - M);
        if (hbefore(omx, oarg, mx, arg)) arg = oarg;
        mx = M;
        lx = fmaxf(lx, olx);
#pragma unroll
        for (int j = 0; j < KD; ++j) push_top(otv[j], oti[j]);
    }
};

// Consumes the logits tiles a wave has accumulated in sh.red (unit u of global wave gw is vocabulary
// tile gw + u * waves of the launch): per-row running statistics, merged per workgroup.
template <int KD, bool TREE>
__device__ inline void head_epilogue(const FusedArgs& a, Shared& sh, uint4* xs, int chunks) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 15, g = lane >> 4;
    const int gw = blockIdx.x * FWAVES + wave, ngw = gridDim.x * FWAVES;     // global wave id, waves of the launch
    const int row = r;
    int x = -1;
    if (row < a.M) {
        const int b = row / a.R, rr = row % a.R;
        x = (rr < a.K && rr < a.draft_len[b]) ? a.drafts[(size_t)b * a.K + rr] : -1;
        if (x >= a.V || TREE) x = -1;               // token trees: the nodes' logits are picked below
    }
    HStat<KD> st;
    st.init();
    const float rs = sh.rs[r];
    const int n_my = n_units(a, PH_HEAD);
    for (int u = 0; u < n_my; ++u) {
        const int t = gw + u * ngw;
        const int n = t * 16 + 4 * g;
        float lv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            lv[i] = sh.red[u][wave][i][lane] * rs;
            st.add(lv[i], n + i);
            if (n + i == x) st.lx = lv[i];
        }
        if (a.logits_dbg && row < a.M)
            *reinterpret_cast<float4*>(a.logits_dbg + (size_t)row * a.V + n) = make_float4(lv[0], lv[1], lv[2], lv[3]);
    }
    if constexpr (TREE) {
        // Token tree: node i of sequence b is judged by the row of its PARENT (row 0, the pending token, for a child of
        // the root), and a row may have several children. A node whose token lies in one of this wave's vocabulary
        // tiles takes its logit from the tile's sums: element (row, token % 16) of unit token / 16 / waves.
        for (int j = lane; j < a.B * a.K; j += 64) {
            const int b = j / a.K, i = j % a.K;
            int nn = a.draft_len[b];
            nn = nn < 0 ? 0 : (nn > a.K ? a.K : nn);
            const int tok = i < nn ? a.drafts[j] : -1;
            if (tok >= 0 && tok < a.V && (tok >> 4) % ngw == gw) {
                const int u = (tok >> 4) / ngw, prow = b * a.R + tree_parent_of(a.parent, b, a.K, i, nn) + 1;
                st_f32(a.hp_lx + b * a.R + i, sh.red[u][wave][tok & 3][((tok >> 2) & 3) * 16 + prow] * sh.rs[prow]);
            }
        }
    }
    st.merge_xor(16);
    st.merge_xor(32);
    // merge the 8 waves of the workgroup (fixed order) so that the acceptance phase reads one record per
    // workgroup and row; the staging area is free by now
    float* ws_f = reinterpret_cast<float*>(xs);                   // [FWAVES][16][3 + KD]
    int* ws_i = reinterpret_cast<int*>(ws_f + FWAVES * 16 * (3 + KD));   // [FWAVES][16][1 + KD]
    if (g == 0) {
        float* f = ws_f + (wave * 16 + r) * (3 + KD);
        int* i = ws_i + (wave * 16 + r) * (1 + KD);
        f[0] = st.mx; f[1] = st.sum; f[2] = st.lx; i[0] = st.arg;
#pragma unroll
        for (int j = 0; j < KD; ++j) { f[3 + j] = st.tv[j]; i[1 + j] = st.ti[j]; }
    }
    __syncthreads();
    if (threadIdx.x < 16 && (int)threadIdx.x < a.M) {
        const int rr = threadIdx.x;
        HStat<KD> m;
        m.init();
        for (int w = 0; w < FWAVES; ++w) {
            const float* f = ws_f + (w * 16 + rr) * (3 + KD);
            const int* i = ws_i + (w * 16 + rr) * (1 + KD);
            float otv[KD]; int oti[KD];
#pragma unroll
            for (int j = 0; j < KD; ++j) { otv[j] = f[3 + j]; oti[j] = i[1 + j]; }
            m.merge(f[0], f[1], f[2], i[0], otv, oti);
        }
        const size_t o = (size_t)rr * chunks + blockIdx.x;
        st_f32(a.hp_max + o, m.mx); st_f32(a.hp_sum + o, m.sum); st_i32(a.hp_arg + o, m.arg);
#pragma unroll
        for (int j = 0; j < KTOP; ++j) {          // the record keeps KTOP entries: the unused ones never rank ahead of anything
            st_f32(a.hp_topv + o * KTOP + j, j < KD ? m.tv[j < KD ? j : 0] : -INFINITY);
            st_i32(a.hp_topi + o * KTOP + j, j < KD ? m.ti[j < KD ? j : 0] : 0x7FFFFFFF);
        }
        if (m.lx != -INFINITY) st_f32(a.hp_lx + rr, m.lx);
    }
}

// Statistics of row `row` over the per-workgroup records (`chunks` = workgroups of the launch; lanes stride over them,
// four records in flight per lane) and the verdict of Eq. 8 on candidate token x with logit lx at that row (x < 0: none).
// Every lane returns the row's arg-max; lane 0's `ok` is the verdict.
__device__ __forceinline__ void accept_eval(const FusedArgs& a, int chunks, int row, int x, float lx, bool& ok, int& arg_out) {
    const int lane = threadIdx.x & 63;
    float mx = -INFINITY, sum = 0.f;
    int arg = 0x7FFFFFFF, ahead = 0;
    for (int c0 = lane; c0 < chunks; c0 += 64 * 4) {
        float cm[4], cs[4], tv[4][KTOP];
        int ca[4], ti[4][KTOP];
#pragma unroll
        for (int q = 0; q < 4; ++q) {          // unconditional loads (clamped), all in flight together
            const size_t o = (size_t)row * chunks + min(c0 + 64 * q, chunks - 1);
            cm[q] = a.hp_max[o]; cs[q] = a.hp_sum[o]; ca[q] = a.hp_arg[o];
#pragma unroll
            for (int j = 0; j < KTOP; ++j) { tv[q][j] = a.hp_topv[o * KTOP + j]; ti[q][j] = a.hp_topi[o * KTOP + j]; }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (c0 + 64 * q >= chunks) continue;
            const float M = fmaxf(mx, cm[q]);
            if (M != -INFINITY) sum = sum * __expf(mx - M) + cs[q] * __expf(cm[q] - M);
            if (hbefore(cm[q], ca[q], mx, arg)) arg = ca[q];
            mx = M;
            if (x >= 0)
#pragma unroll
                for (int j = 0; j < KTOP; ++j) ahead += (ti[q][j] != x && hbefore(tv[q][j], ti[q][j], lx, x)) ? 1 : 0;
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        const float omx = __shfl_xor(mx, off), osum = __shfl_xor(sum, off);
        const int oarg = __shfl_xor(arg, off);
        ahead += __shfl_xor(ahead, off);
        const float M = fmaxf(mx, omx);
        if (M != -INFINITY) sum = sum * __expf(mx - M) + osum * __expf(omx - M);
        if (hbefore(omx, oarg, mx, arg)) arg = oarg;
        mx = M;
    }
    ok = false;
    if (x >= 0) {
        const float q = __expf(lx - mx) / sum;
        const bool in_k = ahead < a.topk, above = q > a.p, top1 = ahead == 0;
        ok = a.mode == LASER_MODE_RV ? (in_k && above)
           : a.mode == LASER_MODE_RV_OR_TOP1 ? (top1 || (in_k && above))
           : a.mode == LASER_MODE_TOPK_ONLY ? in_k : (top1 || above);
    }
    arg_out = arg;
}

// One workgroup per sequence, one wave per row (rows wave, wave + 8, ..).
__device__ inline void accept_phase(const FusedArgs& a, Shared& sh, int chunks) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int b = blockIdx.x; b < a.B; b += gridDim.x) {
        for (int r = wave; r < a.R; r += FWAVES) {
            const int row = b * a.R + r;
            int x = (r < a.K && r < a.draft_len[b]) ? a.drafts[(size_t)b * a.K + r] : -1;
            if (x >= a.V) x = -1;
            const float lx = x >= 0 ? a.hp_lx[row] : -INFINITY;
            bool ok;
            int arg;
            accept_eval(a, chunks, row, x, lx, ok, arg);
            if (lane == 0) {
                sh.row_ok[r] = ok ? 1 : 0;
                sh.row_arg[r] = arg;
            }
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            int dl = a.draft_len[b];
            dl = dl < 0 ? 0 : (dl > a.K ? a.K : dl);
            int n = 0;
            while (n < dl && sh.row_ok[n]) ++n;
            a.accept_len[b] = n;
            int32_t* out = a.out_tokens + (size_t)b * a.R;
            for (int j = 0; j < a.R; ++j) out[j] = j < n ? a.drafts[(size_t)b * a.K + j] : (j == n ? sh.row_arg[n] : -1);
        }
        __syncthreads();
    }
}

// The same for a token tree (Sec. 3.3, Sec. 3.4): one job per row (its arg-max, for the token that follows the accepted
// branch) and one per node (Eq. 8 on the node's token against its parent's row), dealt to the waves; then thread 0
// walks the nodes in pseudo-sequence order: a node is verified iff its parent is and its token passed, the deepest
// verified node -- the first among equally deep -- ends the accepted branch.
__device__ inline void accept_phase_tree(const FusedArgs& a, Shared& sh, int chunks) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int b = blockIdx.x; b < a.B; b += gridDim.x) {
        int nn = a.draft_len[b];
        nn = nn < 0 ? 0 : (nn > a.K ? a.K : nn);
        for (int job = wave; job < a.R + nn; job += FWAVES) {
            bool ok;
            int arg;
            if (job < a.R) {
                accept_eval(a, chunks, b * a.R + job, -1, -INFINITY, ok, arg);
                if (lane == 0) sh.row_arg[job] = arg;
            } else {
                const int i = job - a.R;
                int x = a.drafts[(size_t)b * a.K + i];
                if (x >= a.V) x = -1;
                const float lx = x >= 0 ? a.hp_lx[b * a.R + i] : -INFINITY;
                accept_eval(a, chunks, b * a.R + tree_parent_of(a.parent, b, a.K, i, nn) + 1, x, lx, ok, arg);
                if (lane == 0) sh.row_ok[i] = ok ? 1 : 0;
            }
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            unsigned ver = 0;                        // bit i: node i is verified
            int depth[LASER_MAX_DRAFT + 1];
            int best = -1, best_depth = 0;
            for (int i = 0; i < nn; ++i) {
                const int par = tree_parent_of(a.parent, b, a.K, i, nn);
                depth[i] = 0;
                if (sh.row_ok[i] && (par < 0 || ((ver >> par) & 1u))) {
                    ver |= 1u << i;
                    depth[i] = par < 0 ? 1 : depth[par] + 1;
                    if (depth[i] > best_depth) { best = i; best_depth = depth[i]; }
                }
            }
            a.accept_len[b] = best_depth;
            int32_t* out = a.out_tokens + (size_t)b * a.R;
            for (int j = best_depth + 1; j < a.R; ++j) out[j] = -1;
            out[best_depth] = sh.row_arg[best + 1];
            for (int i = best, j = best_depth - 1; j >= 0; --j) {
                out[j] = a.drafts[(size_t)b * a.K + i];
                if (a.accept_path) a.accept_path[(size_t)b * a.K + j] = i;
                i = tree_parent_of(a.parent, b, a.K, i, nn);
            }
            if (a.accept_path)
                for (int j = best_depth; j < a.K; ++j) a.accept_path[(size_t)b * a.K + j] = -1;
        }
        __syncthreads();
    }
}

// ---- the kernel --------------------------------------------------------------------------------------
template <int DH, bool TR, bool TREE>
__global__ __launch_bounds__(FT) void verify_fused_kernel(FusedArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    Shared& sh = *reinterpret_cast<Shared*>(smem_raw);
    const int nwg = gridDim.x;
    unsigned long long epoch = 0;
    const size_t XS = (size_t)16 * a.d;                 // one x / xg buffer

    if (threadIdx.x < 16) {
        const int row = threadIdx.x;
        int pos = 0, b = 0;
        if (row < a.M) { b = row / a.R; pos = TREE ? a.row_pos_g[row] : a.lens[a.seq_ids[b]] + row % a.R; }
        sh.row_pos[row] = pos;
        sh.row_b[row] = b;
        const int sl = row < a.B ? a.seq_ids[row] : 0;
        sh.seq_slot[row] = sl;
        sh.seq_len[row] = row < a.B ? a.lens[sl] : 0;
    }
    __syncthreads();

    Ring ring;
    uint4* xs = reinterpret_cast<uint4*>(smem_raw + XS_OFFSET);
    const Phase p_head{a.wlm, PH_HEAD, a.d, 1};

    // ---- phase 0: embedding, x0, x0*g1[0], sum of squares ----
    {
        float ss = 0.f;
        const int row = threadIdx.x >> 3, f0 = (threadIdx.x & 7) * 2;
        const float* gain0 = a.L > 0 ? a.g1 : a.gf;
        for (int tile = blockIdx.x; tile < a.d / 16; tile += nwg) {
            if (threadIdx.x < 128) {
                float v0 = 0.f, v1 = 0.f;
                if (row < a.M) {
                    const int b = row / a.R, rr = row % a.R;
                    int tok = rr == 0 ? a.pending[b] : ((rr - 1) < a.draft_len[b] ? a.drafts[(size_t)b * a.K + rr - 1] : 0);
                    if (tok < 0 || tok >= a.V) tok = 0;
                    const uint32_t e = *reinterpret_cast<const uint32_t*>(a.emb + (size_t)tok * a.d + tile * 16 + f0);
                    v0 = __uint_as_float(e << 16);
                    v1 = __uint_as_float(e & 0xFFFF0000u);
                }
                const size_t o = (size_t)row * a.d + tile * 16 + f0;
                st_f32x2(a.xbuf + o, v0, v1);
                uint32_t hi;
                uint16_t lw;
                split_pack_h2_b8(v0 * gain0[tile * 16 + f0], v1 * gain0[tile * 16 + f0 + 1], hi, lw);
                st_u32(a.xgbuf + o, hi);
                st_u16(a.xglbuf + o, lw);
                ss += v0 * v0 + v1 * v1;
            }
        }
        publish_ss(sh, a.ssbuf + (size_t)blockIdx.x * 16, ss);
    }
    int ns = 0;
    auto no_prefetch = [] {};

    for (int l = 0; l < a.L; ++l) {
        // The barrier that ends the previous layer (or the embedding) opens the loop body, so that the
        // weights issued ahead during it are never carried around the loop's back edge.
        {
            const Phase p_q{a.wqkv + (size_t)l * 3 * a.d * a.d, PH_QKV, a.d, 2};
            stamp<TR>(a, ns);
            if (!grid_sync(a, sh, epoch, [&] { prime_steps<1, 0, PF_QKV>(a, p_q, 0, ring); })) return;
            stamp<TR>(a, ns);
        }
        const float* x_in = a.xbuf + (size_t)(2 * l) * XS;           // after the previous layer
        float* x_mid = a.xbuf + (size_t)(2 * l + 1) * XS;             // after attention
        float* x_out = a.xbuf + (size_t)(2 * l + 2) * XS;             // after the FFN
        const uint16_t* xg_in = a.xgbuf + (size_t)(2 * l) * XS;
        uint16_t* xg_mid = a.xgbuf + (size_t)(2 * l + 1) * XS;
        uint16_t* xg_out = a.xgbuf + (size_t)(2 * l + 2) * XS;
        const uint8_t* xgl_in = a.xglbuf + (size_t)(2 * l) * XS;
        uint8_t* xgl_mid = a.xglbuf + (size_t)(2 * l + 1) * XS;
        uint8_t* xgl_out = a.xglbuf + (size_t)(2 * l + 2) * XS;
        const float* ss_in = a.ssbuf + (size_t)(2 * l) * nwg * 16;
        float* ss_mid = a.ssbuf + (size_t)(2 * l + 1) * nwg * 16;
        float* ss_out = a.ssbuf + (size_t)(2 * l + 2) * nwg * 16;
        const size_t lo = (size_t)l * XS;

        const Phase p_qkv{a.wqkv + (size_t)l * 3 * a.d * a.d, PH_QKV, a.d, 2};
        const Phase p_o{a.wo + (size_t)l * a.d * a.d, PH_O, a.d, 2};
        const Phase p_gu{a.wgu + (size_t)l * 2 * a.F * a.d, PH_GU, a.d, 2};
        const Phase p_dn{a.wdown + (size_t)l * a.d * a.F, PH_DOWN, a.F, 1};
        const int w = blockIdx.x;

        // ---- QKV + RoPE ----
        {
            float ssv[8];
            ss_issue(ss_in, ssv);
            stream_phase<1, true, TR, DS_QKV, PF_QKV>(a, sh, xs, p_qkv, xg_in, xgl_in, ring, l, 0);
            ss_finish(a, sh, ssv);
            const int per = a.d / 32, pph = DH / 32, half = DH / 2;
            const int cnt = count_mine(a.d / 16, w, nwg);
            float keep[2] = {0.f, 0.f};
            reduce_epilogue<1>(a, sh, 3 * cnt, [&](int u, int row, int f0, float (&v)[1][2]) {
                const float rs = sh.rs[row];
                if (u < 2 * cnt) {
                    if ((u & 1) == 0) { keep[0] = v[0][0]; keep[1] = v[0][1]; return; }   // first half of a rotary pair
                    const int item = w + (u >> 1) * nwg;
                    const int grp = item / per, idx = item % per;
                    const int h = idx / pph, j = idx % pph;
                    const int c0 = h * DH + j * 16 + f0;                  // channel of keep[*]; partner at c0 + half
                    const int pos = sh.row_pos[row];
                    float o0[2], o1[2];
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        const float2 cs = a.rope[(size_t)pos * half + (j * 16 + f0 + q)];
                        const float x0 = keep[q] * rs, x1 = v[0][q] * rs;
                        o0[q] = x0 * cs.x - x1 * cs.y;
                        o1[q] = x0 * cs.y + x1 * cs.x;
                    }
                    // queries and keys are published split: queries with an fp16 low plane, keys with the
                    // 8-bit low plane the cache keeps
                    const size_t ro = lo + (size_t)row * a.d;
                    uint32_t hi, lw;
                    uint16_t l8;
                    if (grp == 0) {
                        split_pack_h2(o0[0], o0[1], hi, lw);
                        st_u32(a.qbuf + ro + c0, hi); st_u32(a.qlbuf + ro + c0, lw);
                        split_pack_h2(o1[0], o1[1], hi, lw);
                        st_u32(a.qbuf + ro + c0 + half, hi); st_u32(a.qlbuf + ro + c0 + half, lw);
                    } else {
                        split_pack_h2_b8(o0[0], o0[1], hi, l8);
                        st_u32(a.knew + ro + c0, hi); st_u16(a.knewl + ro + c0, l8);
                        split_pack_h2_b8(o1[0], o1[1], hi, l8);
                        st_u32(a.knew + ro + c0 + half, hi); st_u16(a.knewl + ro + c0 + half, l8);
                    }
                } else {
                    const int idx = w + (u - 2 * cnt) * nwg;
                    // values go into the page-shaped exchange buffer at the row's slot of its page
                    const int bb = sh.row_b[row], npp = a.R == 1 ? 1 : 2;
                    const int pos = TREE ? sh.seq_len[bb] + row - bb * a.R : sh.row_pos[row];        // cache slot (row order), not the rotary position
                    const int pi = row < a.M ? pos / kPageSize - sh.seq_len[bb] / kPageSize : 0;
                    const int ch = idx * 16 + f0;                          // channel (head * dh + c) of v[0][0]
                    uint16_t* dst = a.vnew + lo * kPageSize + ((size_t)(bb * npp + pi) * a.d + ch) * kPageSize + pos % kPageSize;
                    if (row < a.M) {                                       // padding rows have no slot
                        st_u16(dst, f32_to_f16(v[0][0] * rs));
                        st_u16(dst + kPageSize, f32_to_f16(v[0][1] * rs));
                    }
                }
            });
        }
        stamp<TR>(a, ns);
        // (nothing of the O projection is requested here: it would queue in front of the attention phase's key / value
        // loads; its first steps go into the barrier behind the attention phase)
        int pg_first[PPW];
        if (!grid_sync(a, sh, epoch, [&] { attn_pages(a, sh, blockIdx.x, pg_first); })) return;
        stamp<TR>(a, ns);

        // ---- attention ----
        attention_phase<DH, TR, TREE>(a, sh, l, pg_first);
        stamp<TR>(a, ns);
        if (!grid_sync(a, sh, epoch, [&] { prime_steps<1, 0, PF_O>(a, p_o, 0, ring); })) return;
        stamp<TR>(a, ns);

        // ---- O projection + residual; publish x, x*g2, sum of squares ----
        {
            float ss = 0.f;
            const float* g2 = a.g2 + (size_t)l * a.d;
            stream_phase<1, true, TR, DS_O, PF_O>(a, sh, xs, p_o, a.attn + lo, a.attnl + lo, ring, l, 3);
            reduce_epilogue<1>(a, sh, n_units(a, PH_O), [&](int u, int row, int f0, float (&v)[1][2]) {
                const int item = w + u * nwg;
                const size_t o = (size_t)row * a.d + item * 16 + f0;
                const float n0 = x_in[o] + v[0][0], n1 = x_in[o + 1] + v[0][1];
                st_f32x2(x_mid + o, n0, n1);
                uint32_t hi;
                uint16_t lw;
                split_pack_h2_b8(n0 * g2[item * 16 + f0], n1 * g2[item * 16 + f0 + 1], hi, lw);
                st_u32(xg_mid + o, hi);
                st_u16(xgl_mid + o, lw);
                ss += n0 * n0 + n1 * n1;
            });
            publish_ss(sh, ss_mid + (size_t)blockIdx.x * 16, ss);
        }
        stamp<TR>(a, ns);
        if (!grid_sync(a, sh, epoch, [&] { prime_steps<2, 0, PF_GU>(a, p_gu, 0, ring); })) return;
        stamp<TR>(a, ns);

        // ---- gate/up + SwiGLU ----
        {
            float ssv[8];
            ss_issue(ss_mid, ssv);
            stream_phase<2, true, TR, DS_GU, PF_GU>(a, sh, xs, p_gu, xg_mid, xgl_mid, ring, l, 6);
            ss_finish(a, sh, ssv);
            uint16_t* act = a.act + (size_t)l * 16 * a.F;
            reduce_epilogue<2>(a, sh, n_units(a, PH_GU), [&](int u, int row, int f0, float (&v)[2][2]) {
                const int item = w + u * nwg;
                const float rs = sh.rs[row];
                float o[2];
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const float gt = v[0][q] * rs, up = v[1][q] * rs;
                    o[q] = gt / (1.f + __expf(-gt)) * up;
                }
                st_u32(act + (size_t)row * a.F + item * 16 + f0, pack_h2(o[0], o[1]));
            });
        }
        stamp<TR>(a, ns);
        if (!grid_sync(a, sh, epoch, [&] { prime_steps<1, 0, PF_DOWN>(a, p_dn, 0, ring); })) return;
        stamp<TR>(a, ns);

        // ---- down projection + residual; publish x, x*gain(next norm), sum of squares ----
        {
            float ss = 0.f;
            const bool last = l + 1 == a.L;
            const float* gn = last ? a.gf : a.g1 + (size_t)(l + 1) * a.d;
            stream_phase<1, false, TR, DS_DOWN, PF_DOWN>(a, sh, xs, p_dn, a.act + (size_t)l * 16 * a.F, nullptr, ring, l, 9);
            reduce_epilogue<1>(a, sh, n_units(a, PH_DOWN), [&](int u, int row, int f0, float (&v)[1][2]) {
                const int item = w + u * nwg;
                const size_t o = (size_t)row * a.d + item * 16 + f0;
                const float n0 = x_mid[o] + v[0][0], n1 = x_mid[o + 1] + v[0][1];
                st_f32x2(x_out + o, n0, n1);
                uint32_t hi;
                uint16_t lw;
                split_pack_h2_b8(n0 * gn[item * 16 + f0], n1 * gn[item * 16 + f0 + 1], hi, lw);
                st_u32(xg_out + o, hi);
                st_u16(xgl_out + o, lw);
                ss += n0 * n0 + n1 * n1;
            });
            publish_ss(sh, ss_out + (size_t)blockIdx.x * 16, ss);
        }
    }
    stamp<TR>(a, ns);
    if (!grid_sync(a, sh, epoch, [&] { prime_steps<1, 0, PF_HEAD>(a, p_head, 0, ring); })) return;
    stamp<TR>(a, ns);

    // ---- output head + acceptance ----
    const int chunks = nwg;            // one record per workgroup and row goes from the head to the acceptance phase
    {
        float ssv[8];
        ss_issue(a.ssbuf + (size_t)(2 * a.L) * nwg * 16, ssv);
        stream_phase<1, false, TR, DS_HEAD, PF_HEAD, false>(a, sh, xs, p_head, a.xgbuf + (size_t)(2 * a.L) * XS, nullptr, ring);
        ss_finish(a, sh, ssv);
        if (a.topk <= 2) head_epilogue<2, TREE>(a, sh, xs, chunks);
        else head_epilogue<KTOP, TREE>(a, sh, xs, chunks);
    }
    stamp<TR>(a, ns);
    if (!grid_sync(a, sh, epoch, no_prefetch)) return;
    stamp<TR>(a, ns);
    if constexpr (TREE) accept_phase_tree(a, sh, chunks);
    else accept_phase(a, sh, chunks);
    stamp<TR>(a, ns);
}

// ---- host side ---------------------------------------------------------------------------------------
static int g_num_cu = 0;
static int g_lds_max = 0;            // largest dynamic LDS one workgroup may ask for

static bool query_device() {
    if (g_num_cu) return true;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return false;
    g_lds_max = (int)std::min<size_t>(prop.sharedMemPerBlock, 160 * 1024);
    g_num_cu = prop.multiProcessorCount;
    return true;
}

struct FusedWS {
    void* blob = nullptr;
    size_t bytes = 0;
    unsigned long long* bar = nullptr;     // [0] count, abort at [64], BAR_FLAGS flag copies from [128] on, 32 words apart
    int L = 0, d = 0, F = 0, nwg = 0, bh_cap = 0, dh = 0;
    float* xbuf; uint16_t* xgbuf; uint8_t* xglbuf; float* ssbuf; uint16_t *qbuf, *knew, *vnew, *attn, *act;
    uint16_t* qlbuf; uint8_t *knewl, *attnl; float* apart; int* acount;
    float *hp_max, *hp_sum; int32_t* hp_arg; float* hp_topv; int32_t* hp_topi; float* hp_lx;
    unsigned long long epoch = 0;
    long long* trace = nullptr;
    int trace_cap = 0;
};

// context splits of a launch: a fixed AW * PPW pages (256 tokens) each, enough to cover the longest sequence
static int fused_splits(int max_len_ub, int R) {
    const int pages_ub = (max_len_ub + R + kPageSize - 1) / kPageSize;
    return std::max(1, (pages_ub + AW * PPW - 1) / (AW * PPW));
}

// max_len_ub: the host's bound of the longest committed context of the batch. A batch whose (sequence, head, context
// split) triples exceed what the partial buffer holds takes the general path instead.
bool fused_supported(const Model* m, int B, int K, int max_len_ub) {
    const laser_model_desc& d = m->d;
    if (!query_device()) return false;
    const int nwg = g_num_cu, M = B * (K + 1);
    if ((long)B * d.n_heads * fused_splits(max_len_ub, K + 1) > 16L * nwg) return false;
    auto per = [](int n, int lanes) { return (n + lanes - 1) / lanes; };
    // every wave slot accumulates at most MAX_UNITS tiles per phase; the norm reduction reads <= 256 partials
    return d.n_layers > 0 && M >= 1 && M <= 16 && d.d_model % 128 == 0 && d.ffn % 128 == 0 && d.vocab % 16 == 0 &&
           (m->dh == 64 || m->dh == 128) && nwg <= 256 &&
           3 * per(d.d_model / 16, nwg) <= MAX_UNITS && 2 * per(d.ffn / 16, nwg) <= MAX_UNITS &&
           per(d.vocab / 16, nwg * FWAVES) <= MAX_UNITS &&
           g_lds_max >= (int)sizeof(Shared) && (size_t)g_lds_max >= XS_OFFSET + 16384 && ((size_t)g_lds_max - XS_OFFSET) / M >= 400;
}

void fused_free(Model* m) {
    FusedWS* ws = reinterpret_cast<FusedWS*>(m->fused_ws);
    if (!ws) return;
    if (ws->blob) (void)hipFree(ws->blob);
    if (ws->bar) (void)hipFree(ws->bar);
    if (ws->trace) (void)hipFree(ws->trace);
    delete ws;
    m->fused_ws = nullptr;
}

static int fused_prepare(Model* m, int B, hipStream_t stream, FusedWS** out) {
    LASER_REQUIRE(query_device(), LASER_E_HIP, "cannot query the device");
    const laser_model_desc& d = m->d;
    FusedWS* ws = reinterpret_cast<FusedWS*>(m->fused_ws);
    const int nwg = g_num_cu;
    const int bh_cap = 16 * nwg;                      // (sequence, head, split) triples the partial buffer can hold
    if (!ws) {
        ws = new FusedWS();
        m->fused_ws = ws;
        const size_t L = d.n_layers, XS = (size_t)16 * d.d_model, PSZ = 32 + 16 * m->dh, CH = (size_t)nwg * FWAVES;
        size_t off = 0;
        auto take = [&](size_t bytes) { size_t o = off; off += (bytes + 255) & ~(size_t)255; return o; };
        const size_t o_x = take((2 * L + 1) * XS * 4), o_xg = take((2 * L + 1) * XS * 2), o_ss = take((2 * L + 1) * nwg * 16 * 4);
        const size_t o_q = take(L * XS * 2), o_k = take(L * XS * 2), o_v = take(L * XS * kPageSize * 2), o_a = take(L * XS * 2);
        const size_t o_xgl = take((2 * L + 1) * XS), o_ql = take(L * XS * 2), o_kl = take(L * XS), o_al = take(L * XS);
        const size_t o_act = take(L * 16 * (size_t)d.ffn * 2), o_ap = take(L * bh_cap * PSZ * 4), o_ac = take(L * bh_cap * 4);
        const size_t o_hm = take(16 * CH * 4), o_hs = take(16 * CH * 4), o_ha = take(16 * CH * 4);
        const size_t o_tv = take(16 * CH * KTOP * 4), o_ti = take(16 * CH * KTOP * 4), o_lx = take(16 * 4);
        LASER_HIP_CHECK(hipMalloc(&ws->blob, off));
        ws->bytes = off;
        LASER_HIP_CHECK(hipMemsetAsync(ws->blob, 0, off, stream));
        LASER_HIP_CHECK(hipMalloc((void**)&ws->bar, 1024 + BAR_FLAGS * 256));
        LASER_HIP_CHECK(hipMemsetAsync(ws->bar, 0, 1024 + BAR_FLAGS * 256, stream));
        char* b = reinterpret_cast<char*>(ws->blob);
        ws->xbuf = (float*)(b + o_x); ws->xgbuf = (uint16_t*)(b + o_xg); ws->ssbuf = (float*)(b + o_ss);
        ws->qbuf = (uint16_t*)(b + o_q); ws->knew = (uint16_t*)(b + o_k); ws->vnew = (uint16_t*)(b + o_v);
        ws->attn = (uint16_t*)(b + o_a); ws->act = (uint16_t*)(b + o_act); ws->apart = (float*)(b + o_ap);
        ws->acount = (int*)(b + o_ac);
        ws->xglbuf = (uint8_t*)(b + o_xgl); ws->qlbuf = (uint16_t*)(b + o_ql); ws->knewl = (uint8_t*)(b + o_kl);
        ws->attnl = (uint8_t*)(b + o_al);
        ws->hp_max = (float*)(b + o_hm); ws->hp_sum = (float*)(b + o_hs); ws->hp_arg = (int32_t*)(b + o_ha);
        ws->hp_topv = (float*)(b + o_tv); ws->hp_topi = (int32_t*)(b + o_ti); ws->hp_lx = (float*)(b + o_lx);
        ws->nwg = nwg; ws->bh_cap = bh_cap;
        const size_t lds = (size_t)g_lds_max;
        const void* fns[6] = {(const void*)verify_fused_kernel<128, false, false>, (const void*)verify_fused_kernel<128, true, false>,
                              (const void*)verify_fused_kernel<64, false, false>, (const void*)verify_fused_kernel<64, true, false>,
                              (const void*)verify_fused_kernel<128, false, true>, (const void*)verify_fused_kernel<64, false, true>};
        for (const void* f : fns) LASER_HIP_CHECK(hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    }
    if (m->fused_trace && !ws->trace) {
        ws->trace_cap = 2 * (5 * d.n_layers + 2) + 4 + 16 * d.n_layers;
        LASER_HIP_CHECK(hipMalloc((void**)&ws->trace, (size_t)ws->nwg * ws->trace_cap * sizeof(long long)));
        LASER_HIP_CHECK(hipMemsetAsync(ws->trace, 0, (size_t)ws->nwg * ws->trace_cap * sizeof(long long), stream));
    }
    *out = ws;
    (void)B;
    return LASER_OK;
}

// parent != NULL: a token tree (drafts / draft_len = its nodes and their count); the caller has filled m->row_pos and
// m->row_anc for this step (rows_kernel) on the same stream.
int run_fused(Model* m, KV* kv, const int32_t* ids_dev, const int32_t* pending, const int32_t* drafts, const int32_t* parent,
              const int32_t* draft_len, int B, int K, int topk, float p, int mode, int32_t* accept_len,
              int32_t* out_tokens, int32_t* accept_path, float* logits_dbg, int max_len_ub, hipStream_t stream) {
    FusedWS* ws = nullptr;
    int rc = fused_prepare(m, B, stream, &ws);
    if (rc) return rc;
    const laser_model_desc& d = m->d;
    const int R = K + 1;
    const int S = fused_splits(max_len_ub, R);
    LASER_REQUIRE(B * d.n_heads * S <= ws->bh_cap, LASER_E_LIMIT,
                  "context of %d tokens needs %d attention splits; the persistent kernel holds %d",
                  max_len_ub + R, B * d.n_heads * S, ws->bh_cap);      // fused_supported() has already ruled this out
    FusedArgs a{};
    a.wqkv = d.wqkv; a.wo = d.wo; a.wgu = d.wgu; a.wdown = d.wdown; a.emb = d.emb; a.wlm = d.wlm;
    a.g1 = d.g1; a.g2 = d.g2; a.gf = d.gf;
    a.L = d.n_layers; a.d = d.d_model; a.H = d.n_heads; a.dh = m->dh; a.F = d.ffn; a.V = d.vocab; a.eps = d.eps;
    a.rope = m->rope;
    a.kpages = kv->kpages; a.klpages = kv->klpages; a.vpages = kv->vpages; a.block_table = kv->block_table; a.lens = kv->len;
    a.mpps = kv->d.max_pages_per_seq; a.n_pages = kv->d.n_pages;
    a.seq_ids = ids_dev; a.pending = pending; a.drafts = drafts; a.draft_len = draft_len;
    a.parent = parent; a.row_pos_g = m->row_pos; a.row_anc_g = m->row_anc; a.accept_path = accept_path;
    a.B = B; a.K = K; a.R = R; a.M = B * R;
    a.xbuf = ws->xbuf; a.xgbuf = ws->xgbuf; a.ssbuf = ws->ssbuf; a.qbuf = ws->qbuf; a.knew = ws->knew; a.vnew = ws->vnew;
    a.attn = ws->attn; a.act = ws->act; a.apart = ws->apart; a.acount = ws->acount; a.nsplit = S;
    a.xglbuf = ws->xglbuf; a.qlbuf = ws->qlbuf; a.knewl = ws->knewl; a.attnl = ws->attnl;
    a.xs_steps = (int)((((size_t)g_lds_max - XS_OFFSET) / a.M - 16) / 256);
    a.xs_steps2 = (int)((((size_t)g_lds_max - XS_OFFSET) / a.M - 16) / 384);
    a.hp_max = ws->hp_max; a.hp_sum = ws->hp_sum; a.hp_arg = ws->hp_arg; a.hp_topv = ws->hp_topv; a.hp_topi = ws->hp_topi;
    a.hp_lx = ws->hp_lx;
    a.topk = topk; a.mode = mode; a.p = p; a.accept_len = accept_len; a.out_tokens = out_tokens; a.logits_dbg = logits_dbg;
    a.bar_count = ws->bar; a.bar_flag = ws->bar + 128; a.abort_flag = reinterpret_cast<int*>(ws->bar + 64);
    a.epoch0 = ws->epoch;
    a.trace = m->fused_trace && !parent ? ws->trace : nullptr;
    a.trace_cap = ws->trace_cap;
    void* args[] = {&a};
    const bool tr = a.trace != nullptr;
    // (a token tree is never traced: its launches take the untraced instantiation)
    const void* fn = parent ? (m->dh == 128 ? (const void*)verify_fused_kernel<128, false, true> : (const void*)verify_fused_kernel<64, false, true>)
                   : m->dh == 128 ? (tr ? (const void*)verify_fused_kernel<128, true, false> : (const void*)verify_fused_kernel<128, false, false>)
                                  : (tr ? (const void*)verify_fused_kernel<64, true, false> : (const void*)verify_fused_kernel<64, false, false>);
    const bool prof = m->prof_on && m->prof_n < m->prof_cap;
    if (prof) LASER_HIP_CHECK(hipEventRecord(m->prof_ev[2 * m->prof_n], stream));
    LASER_HIP_CHECK(hipLaunchCooperativeKernel(fn, dim3(ws->nwg), dim3(FT), args, (size_t)g_lds_max, stream));
    ws->epoch += 5ull * d.n_layers + 2ull;       // barriers this launch passes; advanced only once it is enqueued
    if (prof) { LASER_HIP_CHECK(hipEventRecord(m->prof_ev[2 * m->prof_n + 1], stream)); ++m->prof_n; }
    return LASER_OK;
}

// Copies the stamps of the last traced launch: out[nwg][cap]; returns nwg and cap.
int fused_read_trace(Model* m, hipStream_t stream, long long* out, int max_elems, int* nwg, int* cap) {
    FusedWS* ws = reinterpret_cast<FusedWS*>(m->fused_ws);
    LASER_REQUIRE(ws && ws->trace, LASER_E_INVALID_ARG, "no trace recorded (set option fused_trace first)");
    *nwg = ws->nwg; *cap = ws->trace_cap;
    LASER_REQUIRE((long)ws->nwg * ws->trace_cap <= max_elems, LASER_E_LIMIT, "trace needs %ld elements", (long)ws->nwg * ws->trace_cap);
    LASER_HIP_CHECK(hipMemcpyAsync(out, ws->trace, (size_t)ws->nwg * ws->trace_cap * sizeof(long long), hipMemcpyDeviceToHost, stream));
    LASER_HIP_CHECK(hipStreamSynchronize(stream));
    return LASER_OK;
}

int fused_status(Model* m, hipStream_t stream, int* aborted) {
    *aborted = 0;
    FusedWS* ws = reinterpret_cast<FusedWS*>(m->fused_ws);
    if (!ws) return LASER_OK;
    LASER_HIP_CHECK(hipMemcpyAsync(aborted, ws->bar + 64, sizeof(int), hipMemcpyDeviceToHost, stream));
    LASER_HIP_CHECK(hipStreamSynchronize(stream));
    return LASER_OK;
}

}  // namespace laser
