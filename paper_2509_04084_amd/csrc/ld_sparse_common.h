// Pieces shared by the kernels that replay sparse diffs (not part of the ABI): the table of a
// window's diffs as it travels in kernel arguments, and the chunk table that tells where in
// every diff the records of a 49152-element chunk of the parameter array begin.
#pragma once

#include <limits.h>

#include "ld_common.h"

namespace {

constexpr int64_t kChunk = 49152;          // elements per chunk of the range table
constexpr int kGroupMax = 64;              // diffs per launch of the Adam replay and of the combine
constexpr int kTableMax = 128;             // diffs a table holds (it travels as a kernel argument: 2.5 KB)

struct DiffTable {
    const int32_t* idx[kTableMax];
    const float* val[kTableMax];
    int32_t K[kTableMax];
};

__device__ __forceinline__ int32_t lower_bound_idx(const int32_t* __restrict__ idx, int32_t lo, int32_t hi,
                                                   int64_t target) {
    while (lo < hi) {
        const int32_t mid = lo + ((hi - lo) >> 1);
        if (static_cast<int64_t>(idx[mid]) < target) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// First position p in [lo, hi) with idx[p] >= target (hi if there is none), found by the
// whole wave: 64 probes per round trip to memory, so four rounds cover 2^24 records.
__device__ __forceinline__ int32_t wave_lower_bound(const int32_t* __restrict__ idx, int32_t lo, int32_t hi,
                                                    int64_t target) {
    const int lane = ld_lane();
    while (hi - lo > LD_WAVE) {
        const int32_t step = (hi - lo + LD_WAVE - 1) / LD_WAVE;
        const int64_t p = static_cast<int64_t>(lo) + static_cast<int64_t>(lane + 1) * step - 1;
        const bool reached = p >= hi || static_cast<int64_t>(idx[p]) >= target;
        const uint64_t mask = __ballot(reached);
        if (mask == 0) return hi;  // the last probe was record hi - 1
        const int f = __builtin_ctzll(mask);
        const int64_t top = static_cast<int64_t>(lo) + static_cast<int64_t>(f + 1) * step - 1;
        lo += f * step;
        if (top < hi) hi = static_cast<int32_t>(top);
    }
    const bool reached = lo + lane < hi && static_cast<int64_t>(idx[lo + lane]) >= target;
    const uint64_t mask = __ballot(reached);
    return mask ? lo + __builtin_ctzll(mask) : hi;
}

// Number of keys below `tgt` among records [L, L + 32) of an ascending index list of K records;
// records before the list count as below, records past its end as not below. idx + L must be
// 16-byte aligned.
__device__ __forceinline__ int32_t keys_below(const int32_t* __restrict__ idx, int32_t K, int64_t L, int32_t tgt) {
    int32_t below = 0;
    if (L >= 0 && L <= K - 32) {
        const ld_u32x4* v = reinterpret_cast<const ld_u32x4*>(idx + L);
        ld_u32x4 x[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) x[q] = v[q];
#pragma unroll
        for (int q = 0; q < 8; ++q)
            below += (static_cast<int32_t>(x[q].x) < tgt) + (static_cast<int32_t>(x[q].y) < tgt) +
                     (static_cast<int32_t>(x[q].z) < tgt) + (static_cast<int32_t>(x[q].w) < tgt);
    } else {
#pragma unroll 1
        for (int m = 0; m < 32; ++m) {
            const int64_t p = L + m;
            below += p < 0 || (p < K && idx[p] < tgt);
        }
    }
    return below;
}

constexpr int kLineTries = 3;
constexpr int kChunkThreads = 256;
constexpr int kChunkPer = 2;                                // boundaries per thread
constexpr int kChunkSpan = kChunkThreads * kChunkPer;       // boundaries per workgroup

// ctab[t*(nchunk+1) + b] = number of records of diff t with idx < min(n, b*kChunk).
// A workgroup covers kChunkSpan consecutive boundaries of one diff. The time of this kernel is
// the length of its chain of dependent loads (a few microseconds each), so the chain is kept
// short: two waves bracket the workgroup's run of boundaries with 64-way searches, one load
// per thread then cuts the bracket into kChunkSpan pieces whose end keys go to LDS, every
// boundary finds its piece there, and bisects inside it (about one chunk's records). All
// boundaries are resident at once (two per thread, their searches interleaved).
__global__ __launch_bounds__(kChunkThreads) void k_chunks(DiffTable tb, int64_t n, int32_t nchunk,
                                                          int32_t* __restrict__ ctab) {
    __shared__ int32_t bracket[2];
    __shared__ int32_t piv[kChunkSpan];
    const int32_t b0 = blockIdx.x * kChunkSpan;
    const int t = blockIdx.y;
    const int32_t* __restrict__ idx = tb.idx[t];
    const int32_t K = tb.K[t];
    const int w = threadIdx.x >> 6;
    if (w < 2) {
        int32_t bb = w == 0 ? b0 : b0 + kChunkSpan - 1;
        if (bb > nchunk) bb = nchunk;
        int64_t target = static_cast<int64_t>(bb) * kChunk;
        if (target > n) target = n;
        const int32_t p = wave_lower_bound(idx, 0, K, target);
        if (ld_lane() == 0) bracket[w] = p;
    }
    __syncthreads();
    const int32_t B0 = bracket[0], B1 = bracket[1];
    const int32_t step = (B1 - B0 + kChunkSpan - 1) / kChunkSpan;  // records per piece (0: empty bracket)
#pragma unroll
    for (int j = 0; j < kChunkPer; ++j) {
        const int q = j * kChunkThreads + threadIdx.x;
        const int64_t p = static_cast<int64_t>(B0) + static_cast<int64_t>(q + 1) * step - 1;
        piv[q] = (step > 0 && p < B1) ? idx[p] : INT_MAX;
    }
    __syncthreads();
    int32_t lo[kChunkPer], hi[kChunkPer];
    int64_t target[kChunkPer], guess[kChunkPer];
    int64_t t_first = static_cast<int64_t>(b0) * kChunk, t_last = static_cast<int64_t>(b0 + kChunkSpan - 1) * kChunk;
    if (t_first > n) t_first = n;
    if (t_last > n) t_last = n;
#pragma unroll
    for (int j = 0; j < kChunkPer; ++j) {
        const int32_t b = b0 + j * kChunkThreads + threadIdx.x;
        target[j] = static_cast<int64_t>(b) * kChunk;
        if (target[j] > n) target[j] = n;
        // first piece whose end key reaches the target (kChunkSpan: none, the answer is B1)
        int a = 0, z = kChunkSpan;
        while (a < z) {
            const int mid = (a + z) >> 1;
            if (static_cast<int64_t>(piv[mid]) < target[j]) a = mid + 1; else z = mid;
        }
        const int64_t first = static_cast<int64_t>(B0) + static_cast<int64_t>(a) * step;
        const int64_t last = first + step - 1;  // the piece's end record: it reaches the target
        lo[j] = static_cast<int32_t>(first < B1 ? first : B1);
        hi[j] = static_cast<int32_t>(last < B1 ? last : B1);
        if (step == 0 || b > nchunk) lo[j] = hi[j] = B1;
        // Where the keys between the piece's ends would put the target if they were evenly
        // spaced (the key just before the piece and the one at its end are known, or bounded by
        // the workgroup's first and last targets). Only a guess: the probes below are checked.
        const int64_t key_lo = a > 0 ? static_cast<int64_t>(piv[a - 1]) : t_first - 1;
        const int64_t key_hi = (a < kChunkSpan && piv[a] != INT_MAX) ? static_cast<int64_t>(piv[a]) : t_last;
        const int64_t den = key_hi > key_lo ? key_hi - key_lo : 1;
        guess[j] = (first - 1) + ((target[j] - key_lo) * (hi[j] - (first - 1)) + den - 1) / den;
    }
    // Probe whole 128-byte lines (32 keys), starting with the line of the guess and moving to a
    // neighbour when the target lies outside: the time of this kernel is the number of distinct
    // lines it pulls from memory (nothing stays cached with every search of the table in
    // flight), and a single key per probe would pull a line per bisection step.
    const int32_t mis = static_cast<int32_t>((reinterpret_cast<uintptr_t>(idx) >> 2) & 31u);
#pragma unroll 1
    for (int j = 0; j < kChunkPer; ++j) {
        if (lo[j] >= hi[j]) continue;
        int64_t g = guess[j];
        if (g > hi[j] - 1) g = hi[j] - 1;
        if (g < lo[j]) g = lo[j];
        int64_t L = ((g + mis) & ~static_cast<int64_t>(31)) - mis;  // idx + L: 128-byte aligned
        const int32_t tgt = static_cast<int32_t>(target[j]);  // targets are at most n <= INT_MAX
#pragma unroll 1
        for (int tries = 0; tries < kLineTries && lo[j] < hi[j]; ++tries) {
            const int32_t below = keys_below(idx, K, L, tgt);
            if (below == 32) {
                const int64_t nl = L + 32;
                lo[j] = nl > hi[j] ? hi[j] : (nl > lo[j] ? static_cast<int32_t>(nl) : lo[j]);
                L += 32;
            } else if (below == 0) {
                hi[j] = L < lo[j] ? lo[j] : (L < hi[j] ? static_cast<int32_t>(L) : hi[j]);
                L -= 32;
            } else {
                lo[j] = hi[j] = static_cast<int32_t>(L + below);
            }
        }
    }
    bool more = true;
    while (more) {  // the searches of a thread advance together: their loads are in flight at once
        int32_t mid[kChunkPer], key[kChunkPer];
#pragma unroll
        for (int j = 0; j < kChunkPer; ++j) {
            mid[j] = lo[j] + ((hi[j] - lo[j]) >> 1);
            key[j] = lo[j] < hi[j] ? idx[mid[j]] : 0;
        }
        more = false;
#pragma unroll
        for (int j = 0; j < kChunkPer; ++j) {
            if (lo[j] < hi[j]) {
                if (static_cast<int64_t>(key[j]) < target[j]) lo[j] = mid[j] + 1; else hi[j] = mid[j];
            }
            more |= lo[j] < hi[j];
        }
    }
#pragma unroll
    for (int j = 0; j < kChunkPer; ++j) {
        const int32_t b = b0 + j * kChunkThreads + threadIdx.x;
        if (b <= nchunk) ctab[static_cast<int64_t>(t) * (nchunk + 1) + b] = lo[j];
    }
}

int32_t chunks(int64_t n) { return static_cast<int32_t>((n + kChunk - 1) / kChunk); }

// Enqueues the chunk table of the first `ndiff` diffs of `tb`.
void launch_chunks(const DiffTable& tb, int32_t ndiff, int64_t n, int32_t nchunk, int32_t* ctab, hipStream_t s) {
    k_chunks<<<dim3((nchunk + 1 + kChunkSpan - 1) / kChunkSpan, ndiff), dim3(kChunkThreads), 0, s>>>(tb, n, nchunk, ctab);
}

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
