// Internal helpers shared by the translation units of liblaser (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstdarg>
#include <cstdio>

#include "../../include/laser.h"

namespace laser {

void set_error(const char* fmt, ...);

#define LASER_HIP_CHECK(expr)                                                                   \
    do {                                                                                        \
        hipError_t e__ = (expr);                                                                \
        if (e__ != hipSuccess) {                                                                \
            ::laser::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__), __FILE__, \
                               __LINE__);                                                       \
            return LASER_E_HIP;                                                                 \
        }                                                                                       \
    } while (0)

#define LASER_REQUIRE(cond, code, ...)       \
    do {                                     \
        if (!(cond)) {                       \
            ::laser::set_error(__VA_ARGS__); \
            return (code);                   \
        }                                    \
    } while (0)

// ---- suffix-index hashing, used identically by the host builder and the lookup kernel ----------
__host__ __device__ inline uint64_t mix64(uint64_t x) {
    x ^= x >> 30;
    x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27;
    x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}

// Hash of (key, n, the n tokens in text order).
__host__ __device__ inline uint64_t ngram_hash(int64_t key, int n, const int32_t* toks) {
    uint64_t h = mix64((uint64_t)key + 0x9E3779B97F4A7C15ull * (uint64_t)(n + 1));
    for (int i = 0; i < n; ++i) h = mix64(h ^ ((uint64_t)(uint32_t)toks[i] + 0x632BE59BD9B4E019ull));
    return h;
}

// One slot of the open-addressing n-gram table. count == 0 marks an empty slot.
struct IndexEntry {
    int64_t key;
    uint32_t start;      // first index into the sorted occurrence array
    uint32_t count_n;    // occurrences (low 28 bits) | n (high 4 bits)
};
static_assert(sizeof(IndexEntry) == 16, "entry layout");

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

}  // namespace laser
