// Internal helpers shared by the library's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>
#include "banditspec.h"

namespace bs {

void set_error(const char* fmt, ...);

#define BS_FAIL(code, ...)            \
    do {                              \
        ::bs::set_error(__VA_ARGS__); \
        return (code);                \
    } while (0)

#define BS_REQUIRE(cond, code, ...) \
    do {                            \
        if (!(cond)) BS_FAIL(code, __VA_ARGS__); \
    } while (0)

#define BS_HIP(expr)                                                                        \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess) BS_FAIL(BS_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

#define BS_LAUNCH_CHECK()                                                                   \
    do {                                                                                    \
        hipError_t e_ = hipGetLastError();                                                  \
        if (e_ != hipSuccess) BS_FAIL(BS_EHIP, "kernel launch failed: %s", hipGetErrorString(e_)); \
    } while (0)

// ---- Philox4x32-10 (Salmon et al., SC'11), host and device -------------------------------------
enum : uint32_t { PURPOSE_DRAFT = 0, PURPOSE_ACCEPT = 1, PURPOSE_FINAL = 2, PURPOSE_BANDIT = 3, PURPOSE_NOISE = 4 };

__host__ __device__ inline uint32_t mulhi32(uint32_t a, uint32_t b) {
    return (uint32_t)(((uint64_t)a * (uint64_t)b) >> 32);
}

struct Philox4 { uint32_t w[4]; };

// all four output words for counter (c0, c1, c2, c3)
__host__ __device__ inline Philox4 philox4(uint64_t seed, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3) {
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = mulhi32(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = mulhi32(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    Philox4 o;
    o.w[0] = c0; o.w[1] = c1; o.w[2] = c2; o.w[3] = c3;
    return o;
}

__host__ __device__ inline uint32_t philox_word(uint64_t seed, uint32_t b, uint32_t t, uint32_t slot,
                                                uint32_t purpose) {
    uint32_t c0 = b, c1 = t, c2 = slot, c3 = purpose;
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = mulhi32(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = mulhi32(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return c0;
}

__host__ __device__ inline float u_open_closed(uint32_t w) { return (float)((w >> 8) + 1u) * 5.9604644775390625e-8f; }
__host__ __device__ inline float u_closed_open(uint32_t w) { return (float)(w >> 8) * 5.9604644775390625e-8f; }

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace bs
