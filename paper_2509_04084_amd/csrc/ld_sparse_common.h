// Pieces shared by the kernels that replay sparse diffs (not part of the ABI): the table of a
// window's diffs as it travels in kernel arguments, and the chunk table that tells where in
// every diff the records of a 49152-element chunk of the parameter array begin.
#pragma once

#include <limits.h>

#include "ld_common.h"

namespace {

constexpr int64_t kChunk = 49152;          // elements per chunk of the range table
constexpr int kGroupMax = 64;              // diffs per launch (pointer table travels as a kernel argument)

struct DiffTable {
    const int32_t* idx[kGroupMax];
    const float* val[kGroupMax];
    int32_t K[kGroupMax];
};

__device__ __forceinline__ int32_t lower_bound_idx(const int32_t* __restrict__ idx, int32_t lo, int32_t hi,
                                                   int64_t target) {
    while (lo < hi) {
        const int32_t mid = lo + ((hi - lo) >> 1);
        if (static_cast<int64_t>(idx[mid]) < target) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// ctab[t*(nchunk+1) + b] = number of records of diff t with idx < min(n, b*kChunk).
// A workgroup covers 256 consecutive boundaries of one diff: two threads bracket
// the whole run with full searches, then every thread bisects inside the bracket.
__global__ __launch_bounds__(256) void k_chunks(DiffTable tb, int64_t n, int32_t nchunk,
                                                int32_t* __restrict__ ctab) {
    __shared__ int32_t bracket[2];
    const int32_t b0 = blockIdx.x * 256;
    const int32_t b = b0 + threadIdx.x;
    const int t = blockIdx.y;
    const int32_t* __restrict__ idx = tb.idx[t];
    const int32_t K = tb.K[t];
    if (threadIdx.x < 2) {
        int32_t bb = threadIdx.x == 0 ? b0 : b0 + 255;
        if (bb > nchunk) bb = nchunk;
        int64_t target = static_cast<int64_t>(bb) * kChunk;
        if (target > n) target = n;
        bracket[threadIdx.x] = lower_bound_idx(idx, 0, K, target);
    }
    __syncthreads();
    if (b > nchunk) return;
    int64_t target = static_cast<int64_t>(b) * kChunk;
    if (target > n) target = n;
    ctab[static_cast<int64_t>(t) * (nchunk + 1) + b] = lower_bound_idx(idx, bracket[0], bracket[1], target);
}

int32_t chunks(int64_t n) { return static_cast<int32_t>((n + kChunk - 1) / kChunk); }

// Argument checks common to the sparse replays.
ld_status check_diff_args(const void* w, int64_t n, const int32_t* const* idx, const float* const* val,
                          const int64_t* K, int32_t W) {
    if (n < 0 || n > INT32_MAX || W < 0 || W > LD_MAX_WINDOW) return LD_ERR_RANGE;
    if (W == 0) return LD_OK;
    if (!idx || !val || !K) return LD_ERR_NULL;
    if (n > 0 && !w) return LD_ERR_NULL;
    if (!ld_aligned(w, 16)) return LD_ERR_ALIGN;
    for (int32_t t = 0; t < W; ++t) {
        if (K[t] < 0 || K[t] > n) return LD_ERR_RANGE;
        if (K[t] > 0 && (!idx[t] || !val[t])) return LD_ERR_NULL;
        if (!ld_aligned(idx[t], 4) || !ld_aligned(val[t], 4)) return LD_ERR_ALIGN;
    }
    return LD_OK;
}

}  // namespace
