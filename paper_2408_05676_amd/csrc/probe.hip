// Measured peaks of the device, reported beside the datasheet figures: a streaming read, a streaming copy and a
// register-resident matrix-core loop. They share nothing with the decoding path; the benchmark runs them in the
// same process so that a roofline fraction can also be quoted against what this chip delivered that day.
#include "common.h"
#include "mfma.h"

namespace laser {

typedef unsigned u32x4_p __attribute__((ext_vector_type(4)));

// Grid-stride over 16-byte pieces, four loads in flight per thread; the XOR of everything read is stored only if
// it matches an impossible pattern, so the loads cannot be dropped.
__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4_p* __restrict__ src, size_t n16, unsigned* sink) {
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    u32x4_p x = {0u, 0u, 0u, 0u};
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4_p a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        x ^= a ^ b ^ c ^ d;
    }
    for (; i < n16; i += stride) x ^= src[i];
    if ((x[0] ^ x[1]) == 0x9E3779B9u && (x[2] ^ x[3]) == 0x7F4A7C15u) sink[0] = x[0];
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const u32x4_p* __restrict__ src, u32x4_p* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4_p a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
    }
    for (; i < n16; i += stride) dst[i] = src[i];
}

typedef float f32x16_p __attribute__((ext_vector_type(16)));

// Four independent 32x32x16 fp16 accumulation chains per wave, operands fixed in registers: nothing but the
// matrix pipe is exercised. 4 * iters instructions of 32768 flops per wave.
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float* sink) {
    Frag8 a, b;
#pragma unroll
    for (int i = 0; i < 4; ++i) { a.v4[i] = 0x3C003C00u + threadIdx.x; b.v4[i] = 0x38003800u + (threadIdx.x >> 3); }
    f32x16_p c0, c1, c2, c3;
#pragma unroll
    for (int e = 0; e < 16; ++e) { c0[e] = 0.f; c1[e] = 1.f; c2[e] = 2.f; c3[e] = 3.f; }
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a.v, b.v, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a.v, b.v, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a.v, b.v, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a.v, b.v, c3, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) s += c0[e] + c1[e] + c2[e] + c3[e];
    if (s == 12345.678f) sink[0] = s;
}

// Nothing at all: what a launch of `blocks` wavefronts costs when no wavefront does any work.
__global__ __launch_bounds__(64) void probe_empty_kernel(int* sink) {
    if (sink == nullptr && threadIdx.x == 12345u) *sink = 0;
}

// One exchange between ALL workgroups of a cooperative launch, as the persistent few-row kernel does it between two
// phases: every thread stores a value into a region nobody has read yet (write-through store), waits for the store to
// complete, the workgroups meet at a grid barrier (one counter, the last arriver sets a flag on its own line), then
// every thread reads four values other workgroups wrote (plain cached loads) and checks them. `iters` exchanges in
// a row, each in a fresh region. Every wait is bounded; an expired wait or a stale value is counted in errs.
__global__ __launch_bounds__(512) void probe_exchange_kernel(unsigned* count, unsigned* flag, int iters, float* buf, int* errs) {
    __shared__ int ok_s;
    const unsigned nwg = gridDim.x;
    const size_t region = (size_t)512 * nwg;
    int bad = 0;
    for (int it = 0; it < iters; ++it) {
        float* rb = buf + (size_t)it * region;
        __hip_atomic_store(&rb[(size_t)threadIdx.x * nwg + blockIdx.x], (float)(it * 1000 + (int)blockIdx.x + 1), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (threadIdx.x == 0) {
            const unsigned epoch = (unsigned)it + 1u;
            bool ok = true;
            const unsigned old = __hip_atomic_fetch_add(count, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (old == epoch * nwg - 1u) {
                __hip_atomic_store(flag, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                int spins = 0;
                while (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < epoch) {
                    __builtin_amdgcn_s_sleep(1);
                    if (++spins > 4000000) { ok = false; break; }
                }
            }
            ok_s = ok ? 1 : 0;
        }
        __syncthreads();
        if (!ok_s) { if (threadIdx.x == 0) atomicAdd(errs, 1000000); return; }
        for (int j = 0; j < 4; ++j) {
            const unsigned o = (blockIdx.x + (unsigned)j * 67u + (unsigned)it) % nwg;
            if (rb[(size_t)threadIdx.x * nwg + o] != (float)(it * 1000 + (int)o + 1)) ++bad;
        }
    }
    if (bad) atomicAdd(errs, bad);
}

// A pair of timing events that is destroyed on every way out of a probe.
struct EventPair {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t create() {
        hipError_t e = hipEventCreate(&e0);
        return e != hipSuccess ? e : hipEventCreate(&e1);
    }
    ~EventPair() {
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    }
};

}  // namespace laser

using namespace laser;

extern "C" int laser_probe_hbm(void* buf, size_t bytes, int reps, void* stream_v, float* read_gbs, float* copy_gbs) {
    LASER_REQUIRE(buf != nullptr && read_gbs != nullptr && copy_gbs != nullptr, LASER_E_INVALID_ARG, "NULL argument");
    LASER_REQUIRE(bytes >= (1u << 20) && bytes % 32 == 0 && reps >= 1 && reps <= 1000, LASER_E_INVALID_ARG,
                  "bytes must be a multiple of 32 and at least 1 MiB, reps 1..1000");
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_v);
    int ncu = 0;
    LASER_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, 0));
    EventPair ev;
    LASER_HIP_CHECK(ev.create());
    hipEvent_t e0 = ev.e0, e1 = ev.e1;
    const unsigned grid = (unsigned)ncu * 16u;
    u32x4_p* lo = reinterpret_cast<u32x4_p*>(buf);
    u32x4_p* hi = lo + bytes / 32;
    unsigned* sink = reinterpret_cast<unsigned*>(buf);     // never written: the pattern cannot match
    float ms = 0.f;
    // read: the whole buffer
    hipLaunchKernelGGL(probe_read_kernel, dim3(grid), dim3(256), 0, stream, (const u32x4_p*)lo, bytes / 16, sink);
    LASER_HIP_CHECK(hipEventRecord(e0, stream));
    for (int i = 0; i < reps; ++i)
        hipLaunchKernelGGL(probe_read_kernel, dim3(grid), dim3(256), 0, stream, (const u32x4_p*)lo, bytes / 16, sink);
    LASER_HIP_CHECK(hipEventRecord(e1, stream));
    LASER_HIP_CHECK(hipEventSynchronize(e1));
    LASER_HIP_CHECK(hipEventElapsedTime(&ms, e0, e1));
    *read_gbs = (float)((double)bytes * reps / (ms * 1e-3) / 1e9);
    // copy: first half to second half; bytes moved = read + written
    hipLaunchKernelGGL(probe_copy_kernel, dim3(grid), dim3(256), 0, stream, (const u32x4_p*)lo, hi, bytes / 32);
    LASER_HIP_CHECK(hipEventRecord(e0, stream));
    for (int i = 0; i < reps; ++i)
        hipLaunchKernelGGL(probe_copy_kernel, dim3(grid), dim3(256), 0, stream, (const u32x4_p*)lo, hi, bytes / 32);
    LASER_HIP_CHECK(hipEventRecord(e1, stream));
    LASER_HIP_CHECK(hipEventSynchronize(e1));
    LASER_HIP_CHECK(hipEventElapsedTime(&ms, e0, e1));
    *copy_gbs = (float)((double)bytes * reps / (ms * 1e-3) / 1e9);
    LASER_HIP_CHECK(hipGetLastError());
    return LASER_OK;
}

extern "C" int laser_probe_mfma_f16(void* scratch, int reps, void* stream_v, float* tflops) {
    LASER_REQUIRE(scratch != nullptr && tflops != nullptr && reps >= 1 && reps <= 1000, LASER_E_INVALID_ARG,
                  "NULL argument or reps outside 1..1000");
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_v);
    int ncu = 0;
    LASER_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, 0));
    EventPair ev;
    LASER_HIP_CHECK(ev.create());
    hipEvent_t e0 = ev.e0, e1 = ev.e1;
    const int iters = 4096;
    const unsigned grid = (unsigned)ncu * 4u;               // 16 waves per compute unit, 4 per SIMD
    float* sink = reinterpret_cast<float*>(scratch);       // never written: the sum cannot match
    float ms = 0.f;
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(grid), dim3(256), 0, stream, iters, sink);
    LASER_HIP_CHECK(hipEventRecord(e0, stream));
    for (int i = 0; i < reps; ++i) hipLaunchKernelGGL(probe_mfma_kernel, dim3(grid), dim3(256), 0, stream, iters, sink);
    LASER_HIP_CHECK(hipEventRecord(e1, stream));
    LASER_HIP_CHECK(hipEventSynchronize(e1));
    LASER_HIP_CHECK(hipEventElapsedTime(&ms, e0, e1));
    const double flops = (double)grid * 4.0 * 4.0 * iters * 32768.0 * reps;   // workgroups x waves x chains x iters x flops
    *tflops = (float)(flops / (ms * 1e-3) / 1e12);
    LASER_HIP_CHECK(hipGetLastError());
    return LASER_OK;
}

extern "C" int laser_probe_launch(int blocks, int reps, void* stream_v, float* us_per_launch) {
    LASER_REQUIRE(us_per_launch != nullptr && blocks >= 1 && reps >= 1 && reps <= 100000, LASER_E_INVALID_ARG,
                  "NULL argument, blocks < 1 or reps outside 1..100000");
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_v);
    EventPair ev;
    LASER_HIP_CHECK(ev.create());
    float ms = 0.f;
    int* none = nullptr;
    hipLaunchKernelGGL(probe_empty_kernel, dim3((unsigned)blocks), dim3(64), 0, stream, none);
    LASER_HIP_CHECK(hipEventRecord(ev.e0, stream));
    for (int i = 0; i < reps; ++i) hipLaunchKernelGGL(probe_empty_kernel, dim3((unsigned)blocks), dim3(64), 0, stream, none);
    LASER_HIP_CHECK(hipEventRecord(ev.e1, stream));
    LASER_HIP_CHECK(hipEventSynchronize(ev.e1));
    LASER_HIP_CHECK(hipEventElapsedTime(&ms, ev.e0, ev.e1));
    *us_per_launch = ms * 1e3f / (float)reps;
    LASER_HIP_CHECK(hipGetLastError());
    return LASER_OK;
}

extern "C" int laser_probe_exchange(void* scratch, size_t bytes, int iters, void* stream_v, float* us_per_exchange, int* errors) {
    LASER_REQUIRE(scratch != nullptr && us_per_exchange != nullptr && errors != nullptr, LASER_E_INVALID_ARG, "NULL argument");
    LASER_REQUIRE(iters >= 1 && iters <= 10000, LASER_E_INVALID_ARG, "iters outside 1..10000");
    hipStream_t stream = reinterpret_cast<hipStream_t>(stream_v);
    int ncu = 0, dev = 0, coop = 0;
    LASER_HIP_CHECK(hipGetDevice(&dev));
    LASER_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    LASER_HIP_CHECK(hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev));
    LASER_REQUIRE(coop != 0, LASER_E_SHAPE, "the device does not support cooperative launches");
    // layout of the caller's scratch: [0, 4096) counter / flag / error words on separate lines, then the exchange regions
    const size_t region_bytes = (size_t)512 * ncu * sizeof(float);
    LASER_REQUIRE(bytes >= 4096 + region_bytes * (size_t)iters, LASER_E_LIMIT, "scratch of %zu bytes is too small for %d exchanges (%zu needed)",
                  bytes, iters, 4096 + region_bytes * (size_t)iters);
    unsigned* count = reinterpret_cast<unsigned*>(scratch);
    unsigned* flag = count + 64;
    int* errs = reinterpret_cast<int*>(count + 128);
    float* buf = reinterpret_cast<float*>(reinterpret_cast<char*>(scratch) + 4096);
    EventPair ev;
    LASER_HIP_CHECK(ev.create());
    void* args[] = {&count, &flag, &iters, &buf, &errs};
    // the first pass over fresh memory is several times slower than the steady state: one untimed launch, then the timed one
    int total_errs = 0;
    for (int pass = 0; pass < 2; ++pass) {
        LASER_HIP_CHECK(hipMemsetAsync(scratch, 0, 4096 + region_bytes * (size_t)iters, stream));
        LASER_HIP_CHECK(hipEventRecord(ev.e0, stream));
        LASER_HIP_CHECK(hipLaunchCooperativeKernel(reinterpret_cast<const void*>(probe_exchange_kernel), dim3((unsigned)ncu), dim3(512), args, 0, stream));
        LASER_HIP_CHECK(hipEventRecord(ev.e1, stream));
        int e = 0;
        LASER_HIP_CHECK(hipMemcpyAsync(&e, errs, sizeof(int), hipMemcpyDeviceToHost, stream));
        LASER_HIP_CHECK(hipStreamSynchronize(stream));
        total_errs += e;
    }
    float ms = 0.f;
    LASER_HIP_CHECK(hipEventElapsedTime(&ms, ev.e0, ev.e1));
    *errors = total_errs;
    *us_per_exchange = ms * 1e3f / (float)iters;
    return LASER_OK;
}
