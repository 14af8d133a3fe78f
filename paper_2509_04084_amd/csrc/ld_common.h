// Shared host/device helpers of the gfx950 LowDiff kernels (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "lowdiff.h"

#define LD_WAVE 64

// An entry point calls this once, after its argument checks and before its first launch: an
// error that the caller's own earlier HIP calls left behind in this thread is dropped here, so
// that it is not taken for a failure of this call's launches.
static inline void ld_begin_call() { (void)hipGetLastError(); }

// Status of the launch just enqueued (reading it also clears the error). Checked after every
// launch: when it is not LD_OK the entry point returns at once, with earlier kernels of the
// call already enqueued - the outputs are then unspecified.
static inline ld_status ld_launch_status() {
    return hipGetLastError() == hipSuccess ? LD_OK : LD_ERR_HIP;
}

static inline bool ld_aligned(const void* p, size_t a) {
    return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0;
}

static inline size_t ld_round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Per-step scalars of an Adam replay window, prepared on the host in double.
#define LD_MAX_ADAM_STEPS 64
struct LdAdamSteps {
    float lr_over_bc1[LD_MAX_ADAM_STEPS];  // lr / (1 - beta1^s)
    float inv_bc2[LD_MAX_ADAM_STEPS];      // 1 / (1 - beta2^s)
    float beta1, one_m_beta1, beta2, one_m_beta2, eps;
};

// Scalars of steps step0+1 .. step0+W (W <= LD_MAX_ADAM_STEPS).
static inline void ld_fill_adam_steps(LdAdamSteps& a, int32_t W, int64_t step0, float lr, float beta1,
                                      float beta2, float eps) {
    for (int32_t t = 0; t < LD_MAX_ADAM_STEPS; ++t) {
        a.lr_over_bc1[t] = 0.0f;
        a.inv_bc2[t] = 0.0f;
    }
    for (int32_t t = 0; t < W; ++t) {
        const double s = static_cast<double>(step0 + 1 + t);
        const double bc1 = 1.0 - pow(static_cast<double>(beta1), s);
        const double bc2 = 1.0 - pow(static_cast<double>(beta2), s);
        a.lr_over_bc1[t] = static_cast<float>(static_cast<double>(lr) / bc1);
        a.inv_bc2[t] = static_cast<float>(1.0 / bc2);
    }
    a.beta1 = beta1;
    a.one_m_beta1 = 1.0f - beta1;
    a.beta2 = beta2;
    a.one_m_beta2 = 1.0f - beta2;
    a.eps = eps;
}

// Whether a replay with this eps needs the square root that handles denormal arguments.
static inline bool ld_adam_careful(float eps) { return !(eps >= 1e-12f); }

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

__device__ __forceinline__ float ld_bf16_widen(uint32_t h) { return __uint_as_float(h << 16); }

// One Adam step on one element (Eq. (4); bias-corrected, eps added to the root of the
// corrected second moment). The only place the arithmetic is written: every replay
// kernel, fused window or single step, dense or sparse gradient, runs these operations.
//   lr_bc1 = lr / (1 - beta1^s), ibc2 = 1 / (1 - beta2^s), both prepared on the host in double
// The hardware square root takes a denormal argument for zero. Next to an eps of ordinary size
// that is far below the tolerance (the root of a denormal is below 1.1e-19); with eps = 0, or an eps
// that small, it would decide the result (a zero denominator). TINY_EPS (chosen per call from eps,
// see ld_adam_careful) scales such arguments into the normal range first: sqrt(x) =
// sqrt(x * 2^64) * 2^-32, exact scalings.
template <bool TINY_EPS>
__device__ __forceinline__ void ld_adam_step(float& w, float& m, float& v, float g, float b1,
                                             float omb1, float b2, float omb2, float eps,
                                             float lr_bc1, float ibc2) {
    m = __fmaf_rn(b1, m, __fmul_rn(omb1, g));
    v = __fmaf_rn(b2, v, __fmul_rn(__fmul_rn(omb2, g), g));
    float x = __fmul_rn(v, ibc2), root;
    if (TINY_EPS) {
        const bool tiny = x < 0x1p-96f;
        x = tiny ? __fmul_rn(x, 0x1p+64f) : x;
        root = __builtin_amdgcn_sqrtf(x);
        root = tiny ? __fmul_rn(root, 0x1p-32f) : root;
    } else {
        root = __builtin_amdgcn_sqrtf(x);
    }
    const float denom = __fadd_rn(root, eps);
    const float upd = __fmul_rn(__fmul_rn(lr_bc1, m), __builtin_amdgcn_rcpf(denom));
    w = __fsub_rn(w, upd);
}

// Device-scope load that is not served from a stale per-CU cache line.
__device__ __forceinline__ uint32_t ld_load_coherent(const uint32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

#endif  // __HIPCC__
