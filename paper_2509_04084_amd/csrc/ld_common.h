// Shared host/device helpers of the gfx950 LowDiff kernels (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lowdiff.h"

#define LD_WAVE 64

#define LD_CHECK_HIP(expr)                         \
    do {                                           \
        hipError_t e_ = (expr);                    \
        if (e_ != hipSuccess) return LD_ERR_HIP;   \
    } while (0)

// A launch that failed to enqueue leaves a sticky-free error we must consume.
static inline ld_status ld_launch_status() {
    return hipGetLastError() == hipSuccess ? LD_OK : LD_ERR_HIP;
}

static inline bool ld_aligned(const void* p, size_t a) {
    return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0;
}

static inline size_t ld_round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

#ifdef __HIPCC__

typedef float ld_f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t ld_u32x4 __attribute__((ext_vector_type(4)));

// Streaming (non-temporal) 16-byte accesses; p must be 16-byte aligned.
__device__ __forceinline__ ld_f32x4 ld_nt_load(const ld_f32x4* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ ld_u32x4 ld_nt_load(const ld_u32x4* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void ld_nt_store(ld_f32x4 x, ld_f32x4* p) { __builtin_nontemporal_store(x, p); }
__device__ __forceinline__ void ld_nt_store(ld_u32x4 x, ld_u32x4* p) { __builtin_nontemporal_store(x, p); }

__device__ __forceinline__ int ld_lane() { return __lane_id(); }

// |x| as an integer that orders like the magnitude (sign bit cleared).
__device__ __forceinline__ uint32_t ld_key(float x) { return __float_as_uint(x) & 0x7FFFFFFFu; }

// Inclusive scan over the 64 lanes of a wave.
__device__ __forceinline__ uint32_t ld_wave_iscan(uint32_t x) {
#pragma unroll
    for (int d = 1; d < LD_WAVE; d <<= 1) {
        uint32_t y = __shfl_up(x, d, LD_WAVE);
        if (ld_lane() >= d) x += y;
    }
    return x;
}

__device__ __forceinline__ uint32_t ld_wave_sum(uint32_t x) {
#pragma unroll
    for (int d = LD_WAVE / 2; d > 0; d >>= 1) x += __shfl_xor(x, d, LD_WAVE);
    return x;
}

// Exclusive scan over a 256-thread block. `sh` holds 4 words; returns the
// exclusive prefix of x and the block total. Ends with a barrier so `sh` may be
// reused right away.
__device__ __forceinline__ uint32_t ld_block_escan256(uint32_t x, uint32_t* sh, uint32_t& total) {
    const uint32_t inc = ld_wave_iscan(x);
    const int w = threadIdx.x >> 6;
    if (ld_lane() == LD_WAVE - 1) sh[w] = inc;
    __syncthreads();
    const uint32_t t0 = sh[0], t1 = sh[1], t2 = sh[2], t3 = sh[3];
    total = t0 + t1 + t2 + t3;
    uint32_t base = 0;
    if (w > 0) base += t0;
    if (w > 1) base += t1;
    if (w > 2) base += t2;
    __syncthreads();
    return base + inc - x;
}

// Device-scope load that is not served from a stale per-CU cache line.
__device__ __forceinline__ uint32_t ld_load_coherent(const uint32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

#endif  // __HIPCC__
