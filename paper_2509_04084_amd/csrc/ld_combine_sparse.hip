// ld_combine_sparse: N per-worker record lists combined into one.
//
// Sync of Algorithm 1 (Sec. IV-B; Eq. (3)) for compressed gradients: what an
// all-gather leaves on every rank is N ascending (idx, val) lists; the synchronized
// diff that is checkpointed holds every index recorded by at least one worker, with
// the workers' values added in worker order (one fp32 add each, starting from +0)
// and multiplied by `scale` (1 for a sum, 1/N for a mean).
//
// The index space is cut into 8192-element sub-tiles, one wave each, in two passes:
//   k_combine_count  marks the sub-tile's recorded positions in an LDS bitmap, counts
//                    them and leaves the bitmap in the workspace (1 KB per sub-tile);
//   k_combine_groups / k_combine_scan   scan the counts (inside groups of 1024
//                    sub-tiles, then the at most 1024 group sums);
//   k_combine_emit   fetches the bitmap (marking the positions a second time cost more
//                    than the n / 8 bytes written and read), ranks every position among the
//                    recorded ones and adds the values at their rank in a small LDS array, list
//                    after list (LDS operations of one wave complete in order, and
//                    inside one list the indices are distinct), then writes the array
//                    out as one contiguous run at the sub-tile's offset. A dense tile
//                    of the sub-tile would cost 32 KB of LDS per wave and leave one
//                    wave per SIMD; the ranked array takes 7.5 KB.
// The records of a sub-tile are found as in ld_merge_sparse: chunk table +
// interpolated 128-record windows, verified. HBM traffic: the indices twice, the values
// once, the bitmaps out and in, the output once.
#include "ld_sparse_common.h"

namespace {

constexpr int kSub = 8192;                 // elements per wave sub-tile
constexpr int kChunkSubs = static_cast<int>(kChunk / kSub);  // sub-tiles per chunk of the range table
static_assert(static_cast<int64_t>(kSub) * kChunkSubs == kChunk, "sub-tiles must tile a chunk");
constexpr int kWin = 2;                    // 64-record windows per list loaded ahead (three: 6 % slower, the third is mostly unused)
constexpr int kPre = 8;                    // lists whose windows are loaded before any is used
constexpr int kMargin = 24;                // records the window starts before the interpolated position
constexpr int kWords = kSub / 32;          // bitmap words per sub-tile: 256
constexpr int kSubsPerGroup = 1024;        // n <= 2^31-1 gives at most 1024 groups
constexpr int kCap = 1024;                 // distinct indices of a sub-tile accumulated per round of the emission

// Calls f(t, i, v) for every record (i, v) of list t with lo <= i < hi, list after list
// (t ascending); all lanes of the wave take part, one record per lane and call.
template <bool VAL, class F>
__device__ __forceinline__ void sweep_records(const DiffTable& tb, int32_t W, const int32_t* __restrict__ ctab,
                                              int32_t nchunk, int64_t sub, int32_t lo, int32_t hi, int lane,
                                              F&& f) {
    const int32_t chunk = static_cast<int32_t>(sub / kChunkSubs), part = static_cast<int32_t>(sub % kChunkSubs);
    int32_t c0 = 0, c1 = 0;  // lane t: where list t's records of this chunk lie
    if (lane < W) {
        const int32_t* row = ctab + static_cast<int64_t>(lane) * (nchunk + 1) + chunk;
        c0 = row[0];
        c1 = row[1];
    }
    int32_t start = c0 + ((c1 - c0) * part) / kChunkSubs - kMargin;  // the guess for this sub-tile
    if (start < c0) start = c0;
    auto from = [&](int t, int32_t p, int32_t end) {  // records [p, end) up to the first at or beyond hi
        for (; p < end; p += LD_WAVE) {
            const bool have = p + lane < end;
            const int32_t i = have ? tb.idx[t][p + lane] : INT_MAX;
            const float v = (VAL && have) ? tb.val[t][p + lane] : 0.0f;
            if (i >= lo && i < hi) f(t, i, v);
            if (__ballot(i >= hi)) break;
        }
    };
#pragma unroll 1
    for (int32_t t0 = 0; t0 < W; t0 += kPre) {
        int32_t s_[kPre], e_[kPre], b_[kPre], ri[kPre][kWin];
        float rv[kPre][kWin];
#pragma unroll
        for (int g = 0; g < kPre; ++g) {
            const int t = (t0 + g < W) ? t0 + g : 0;
            s_[g] = __builtin_amdgcn_readlane(start, t);
            b_[g] = __builtin_amdgcn_readlane(c0, t);
            e_[g] = (t0 + g < W) ? __builtin_amdgcn_readlane(c1, t) : s_[g];  // past W: an empty window
#pragma unroll
            for (int u = 0; u < kWin; ++u) {
                const int32_t p = s_[g] + u * LD_WAVE + lane;
                const bool h = p < e_[g];
                ri[g][u] = h ? tb.idx[t][p] : INT_MAX;
                rv[g][u] = (VAL && h) ? tb.val[t][p] : 0.0f;
            }
        }
#pragma unroll
        for (int g = 0; g < kPre; ++g) {
            if (s_[g] < e_[g]) {
                const int t = t0 + g;
                const int32_t first = __builtin_amdgcn_readfirstlane(ri[g][0]);
                if (s_[g] == b_[g] || first <= lo) {  // the window begins before the sub-tile's records do
                    bool more = true;
#pragma unroll
                    for (int u = 0; u < kWin; ++u) {
                        if (more) {
                            if (ri[g][u] >= lo && ri[g][u] < hi) f(t, ri[g][u], rv[g][u]);
                            more = !__ballot(ri[g][u] >= hi);
                        }
                    }
                    if (more) from(t, s_[g] + kWin * LD_WAVE, e_[g]);
                } else {  // guess too late: find the first record of the sub-tile inside the chunk
                    from(t, lower_bound_idx(tb.idx[t], b_[g], s_[g], lo), e_[g]);
                }
            }
            __builtin_amdgcn_wave_barrier();  // keep list g's LDS traffic ahead of list g+1's
        }
    }
}

struct SubTile {
    int64_t sub;
    int32_t lo, hi;
    bool live;
};

__device__ __forceinline__ SubTile sub_tile(int64_t n) {
    // consecutive workgroups go to different XCDs: each XCD walks one contiguous eighth of the index space
    SubTile s;
    const int64_t per = (static_cast<int64_t>(gridDim.x) + 7) / 8;
    s.sub = static_cast<int64_t>(blockIdx.x % 8) * per + blockIdx.x / 8;
    s.live = s.sub * kSub < n;
    const int64_t lo64 = s.sub * kSub;
    s.lo = static_cast<int32_t>(s.live ? lo64 : 0);
    s.hi = static_cast<int32_t>(s.live ? ((n - lo64) < kSub ? n : lo64 + kSub) : 0);  // n <= INT_MAX
    return s;
}

__global__ __launch_bounds__(LD_WAVE) void k_combine_count(int64_t n, int32_t nchunk, DiffTable tb, int32_t W,
                                                           const int32_t* __restrict__ ctab,
                                                           uint32_t* __restrict__ counts,
                                                           uint32_t* __restrict__ bitmaps) {
    __shared__ uint32_t bm[kWords];
    const int lane = threadIdx.x;
    const SubTile s = sub_tile(n);
    if (!s.live) return;
#pragma unroll
    for (int j = 0; j < kWords / LD_WAVE; ++j) bm[j * LD_WAVE + lane] = 0;
    __syncthreads();  // one wave: orders the fill before the marks
    sweep_records<false>(tb, W, ctab, nchunk, s.sub, s.lo, s.hi, lane, [&](int, int32_t i, float) {
        const uint32_t q = static_cast<uint32_t>(i - s.lo);
        atomicOr(&bm[q >> 5], 1u << (q & 31));
    });
    __syncthreads();
    uint32_t c = 0;
#pragma unroll
    for (int j = 0; j < kWords / LD_WAVE; ++j) {
        const uint32_t word = bm[j * LD_WAVE + lane];
        c += __popc(word);
        bitmaps[s.sub * kWords + j * LD_WAVE + lane] = word;  // k_combine_emit takes it from here
    }
    c = ld_wave_sum(c);
    if (lane == 0) counts[s.sub] = c;
}

// One workgroup per group of kSubsPerGroup sub-tiles: counts -> exclusive prefix inside the group
// (in place), group total -> gsum.
__global__ __launch_bounds__(256) void k_combine_groups(uint32_t* __restrict__ counts, int32_t nsub,
                                                        uint32_t* __restrict__ gsum) {
    __shared__ uint32_t sh[4];
    constexpr int per = kSubsPerGroup / 256;
    const int32_t first = blockIdx.x * kSubsPerGroup + threadIdx.x * per;
    uint32_t x[per], sum = 0;
#pragma unroll
    for (int i = 0; i < per; ++i) {
        x[i] = first + i < nsub ? counts[first + i] : 0u;
        sum += x[i];
    }
    uint32_t total;
    uint32_t before = ld_block_escan256(sum, sh, total);
#pragma unroll
    for (int i = 0; i < per; ++i) {
        if (first + i < nsub) counts[first + i] = before;
        before += x[i];
    }
    if (threadIdx.x == 0) gsum[blockIdx.x] = total;
}

// Exclusive scan of the group sums (at most 1024 groups: n <= 2^31-1); total -> *out_count.
__global__ __launch_bounds__(1024) void k_combine_scan(const uint32_t* __restrict__ gsum, uint32_t* __restrict__ goff,
                                                       int32_t ngrp, int64_t* __restrict__ out_count) {
    __shared__ uint32_t sh[1024 / LD_WAVE];
    const uint32_t x = static_cast<int32_t>(threadIdx.x) < ngrp ? gsum[threadIdx.x] : 0u;
    const uint32_t inc = ld_wave_iscan(x);
    const int w = threadIdx.x >> 6;
    if (ld_lane() == LD_WAVE - 1) sh[w] = inc;
    __syncthreads();
    uint32_t base = 0, total = 0;
#pragma unroll
    for (int i = 0; i < 1024 / LD_WAVE; ++i) {
        const uint32_t t = sh[i];
        if (i < w) base += t;
        total += t;
    }
    if (static_cast<int32_t>(threadIdx.x) < ngrp) goff[threadIdx.x] = base + inc - x;
    if (threadIdx.x == 0) *out_count = static_cast<int64_t>(total);
}

__global__ __launch_bounds__(LD_WAVE) void k_combine_emit(int64_t n, int32_t nchunk, DiffTable tb, int32_t W,
                                                          const int32_t* __restrict__ ctab,
                                                          const uint32_t* __restrict__ prefix, int32_t nsub,
                                                          const uint32_t* __restrict__ gsum,
                                                          const uint32_t* __restrict__ goff,
                                                          const uint32_t* __restrict__ bitmaps, float scale,
                                                          int32_t* __restrict__ out_idx,
                                                          float* __restrict__ out_val, int64_t out_cap) {
    __shared__ uint32_t bm[kWords];      // recorded positions of the sub-tile
    __shared__ uint16_t wpre[kWords];    // recorded positions before each bitmap word
    __shared__ float acc[kCap];          // sums, at the rank of their position among the recorded ones
    __shared__ uint16_t accq[kCap];      // ... and the positions themselves
    const int lane = threadIdx.x;
    const SubTile s = sub_tile(n);
    if (!s.live) return;
    // records written before this sub-tile: its group's offset + its prefix inside the group; its own
    // count is the distance to the next prefix (or to the group's total)
    const int32_t grp = static_cast<int32_t>(s.sub / kSubsPerGroup);
    const uint32_t before = prefix[s.sub];
    const bool last_of_group = (s.sub + 1) % kSubsPerGroup == 0 || s.sub + 1 >= nsub;
    const uint32_t mine = (last_of_group ? gsum[grp] : prefix[s.sub + 1]) - before;
    if (mine == 0) return;  // nothing recorded in this sub-tile
    const int64_t off = static_cast<int64_t>(goff[grp]) + before;
#pragma unroll
    for (int j = 0; j < kWords / LD_WAVE; ++j) bm[j * LD_WAVE + lane] = bitmaps[s.sub * kWords + j * LD_WAVE + lane];
    __syncthreads();  // one wave: orders the fill before what reads it
    {  // lane l owns bitmap words 4l .. 4l+3
        uint32_t c[kWords / LD_WAVE], sum = 0;
#pragma unroll
        for (int j = 0; j < kWords / LD_WAVE; ++j) {
            c[j] = __popc(bm[lane * (kWords / LD_WAVE) + j]);
            sum += c[j];
        }
        uint32_t run = ld_wave_iscan(sum) - sum;
#pragma unroll
        for (int j = 0; j < kWords / LD_WAVE; ++j) {
            wpre[lane * (kWords / LD_WAVE) + j] = static_cast<uint16_t>(run);
            run += c[j];
        }
    }
    // Rounds of kCap distinct indices (one round unless the sub-tile is crowded): the values are added,
    // list after list, at the rank of their position; then the round is written out as one run.
#pragma unroll 1
    for (uint32_t r0 = 0; r0 < mine; r0 += kCap) {
#pragma unroll
        for (int j = 0; j < kCap / LD_WAVE; ++j) acc[j * LD_WAVE + lane] = 0.0f;
        __syncthreads();
        sweep_records<true>(tb, W, ctab, nchunk, s.sub, s.lo, s.hi, lane, [&](int, int32_t i, float v) {
            const uint32_t q = static_cast<uint32_t>(i - s.lo);
            const uint32_t rank = wpre[q >> 5] + __popc(bm[q >> 5] & ((1u << (q & 31)) - 1u));
            if (rank - r0 < static_cast<uint32_t>(kCap)) {
                acc[rank - r0] = __fadd_rn(acc[rank - r0], v);
                accq[rank - r0] = static_cast<uint16_t>(q);
            }
        });
        __syncthreads();
        const uint32_t cnt = mine - r0 < static_cast<uint32_t>(kCap) ? mine - r0 : static_cast<uint32_t>(kCap);
        for (uint32_t i = lane; i < cnt; i += LD_WAVE) {
            const int64_t pos = off + r0 + i;
            if (pos < out_cap) {
                out_idx[pos] = s.lo + static_cast<int32_t>(accq[i]);
                out_val[pos] = __fmul_rn(scale, acc[i]);
            }
        }
        __syncthreads();
    }
}

}  // namespace

namespace {
struct CombineLayout { size_t ctab, counts, gsum, goff, bitmaps, total; };
CombineLayout combine_layout(int64_t n, int32_t N) {
    CombineLayout L;
    size_t o = 0;
    auto take = [&](size_t bytes) { const size_t at = o; o += ld_round_up(bytes, 256); return at; };
    const size_t nsub = static_cast<size_t>((n + kSub - 1) / kSub);
    const size_t ngrp = (nsub + kSubsPerGroup - 1) / kSubsPerGroup;
    L.ctab = take(static_cast<size_t>(N) * (static_cast<size_t>(chunks(n)) + 1) * 4);
    L.counts = take(nsub * 4);
    L.gsum = take(ngrp * 4);
    L.goff = take(ngrp * 4);
    L.bitmaps = take(nsub * kWords * 4);  // recorded positions of every sub-tile: n / 8 bytes
    L.total = o;
    return L;
}
}  // namespace

extern "C" size_t ld_combine_sparse_workspace(int64_t n, int32_t N) {
    if (n <= 0 || N <= 0 || N > LD_MAX_WORKERS) return 256;
    return combine_layout(n, N).total;
}

extern "C" ld_status ld_combine_sparse(const int32_t* const* idx, const float* const* val, const int64_t* K,
                                       int32_t N, int64_t n, float scale, int32_t* out_idx, float* out_val,
                                       int64_t out_cap, int64_t* out_count, void* workspace,
                                       size_t workspace_bytes, ld_stream stream) {
    if (n < 0 || n > INT32_MAX || N < 0 || N > LD_MAX_WORKERS || out_cap < 0) return LD_ERR_RANGE;
    if (!out_count) return LD_ERR_NULL;
    if (!ld_aligned(out_count, 8)) return LD_ERR_ALIGN;
    if (N > 0 && (!idx || !val || !K)) return LD_ERR_NULL;
    int64_t total = 0;
    for (int32_t t = 0; t < N; ++t) {
        if (K[t] < 0 || K[t] > n) return LD_ERR_RANGE;
        if (K[t] > 0 && (!idx[t] || !val[t])) return LD_ERR_NULL;
        if (!ld_aligned(idx[t], 4) || !ld_aligned(val[t], 4)) return LD_ERR_ALIGN;
        total += K[t];
    }
    if (out_cap > 0 && (!out_idx || !out_val)) return LD_ERR_NULL;
    if (!ld_aligned(out_idx, 4) || !ld_aligned(out_val, 4)) return LD_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    ld_begin_call();
    const int32_t nsub = static_cast<int32_t>((n + kSub - 1) / kSub);
    const int32_t ngrp = (nsub + kSubsPerGroup - 1) / kSubsPerGroup;
    if (n == 0 || N == 0 || total == 0) {  // an empty result: only the count is written
        static_assert(sizeof(uint32_t) == 4, "");
        k_combine_scan<<<dim3(1), dim3(1024), 0, s>>>(nullptr, nullptr, 0, out_count);
        return ld_launch_status();
    }
    const CombineLayout L = combine_layout(n, N);
    if (!workspace || !ld_aligned(workspace, 256) || workspace_bytes < L.total) return LD_ERR_WORKSPACE;
    char* ws = static_cast<char*>(workspace);
    int32_t* ctab = reinterpret_cast<int32_t*>(ws + L.ctab);
    uint32_t* counts = reinterpret_cast<uint32_t*>(ws + L.counts);
    uint32_t* gsum = reinterpret_cast<uint32_t*>(ws + L.gsum);
    uint32_t* goff = reinterpret_cast<uint32_t*>(ws + L.goff);
    uint32_t* bitmaps = reinterpret_cast<uint32_t*>(ws + L.bitmaps);
    static_assert(LD_MAX_WORKERS <= kGroupMax, "one launch must hold every list");
    DiffTable tb = {};
    for (int32_t t = 0; t < kGroupMax; ++t) {
        const bool live = t < N;
        tb.idx[t] = live ? idx[t] : nullptr;
        tb.val[t] = live ? val[t] : nullptr;
        tb.K[t] = live ? static_cast<int32_t>(K[t]) : 0;
    }
    const int32_t nchunk = chunks(n);
    const dim3 grid(static_cast<uint32_t>((nsub + 7) / 8 * 8)), wave(LD_WAVE);
    launch_chunks(tb, N, n, nchunk, ctab, s);
    if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    k_combine_count<<<grid, wave, 0, s>>>(n, nchunk, tb, N, ctab, counts, bitmaps);
    if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    k_combine_groups<<<dim3(ngrp), dim3(256), 0, s>>>(counts, nsub, gsum);
    if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    k_combine_scan<<<dim3(1), dim3(1024), 0, s>>>(gsum, goff, ngrp, out_count);
    if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    k_combine_emit<<<grid, wave, 0, s>>>(n, nchunk, tb, N, ctab, counts, nsub, gsum, goff, bitmaps, scale, out_idx,
                                         out_val,
                                         out_cap);
    return ld_launch_status();
}
