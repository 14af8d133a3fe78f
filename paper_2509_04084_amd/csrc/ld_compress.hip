// ld_compress_topk: per-segment exact top-k sparsification with error feedback.
//
// Comp of Algorithm 1 (Sec. IV-B) at ratio rho (Sec. II-C, Sec. VII-A): the
// compressed gradient that is reused as the differential checkpoint.  The
// selection rule (|r+g| descending on the bit pattern, ties to the lower index,
// records ascending, selected residuals zeroed) is stated in lowdiff.h.
//
// Design: ONE streaming pass over gradient and residual, then three small passes
// over a candidate set of about 1.7 * k elements.
//
//   k_prep    one workgroup per segment. The segment table travels in its kernel arguments,
//             packed as a dictionary of the distinct (length, k) pairs plus one byte per
//             segment (a model has few distinct tensor shapes); every workgroup rebuilds the
//             prefix sums it needs from it. Tables that do not pack (more than 160 distinct
//             pairs or 2048 segments) go through k_upload launches first. From a 16K-element sample of |r+g| it
//             estimates three keys: a candidate threshold tau (the sample key at a
//             rank high enough that, with overwhelming probability, at least k
//             elements of the segment lie at or above it), the likeliest threshold
//             T_est (the sample key at the rank that corresponds to k), and the top
//             of the fine bins that the later passes lay over the keys above tau.
//             When the whole segment fits in the sample the three are exact.
//   k_main    the only full pass, 12 bytes per element. One wave per 4096-element
//             tile, each XCD walking one contiguous eighth of the tiles in address
//             order. Elements with key >= tau
//             go, in index order, into the tile's candidate slot. The residual is
//             written as if T_est were the threshold: +0 where key >= T_est, r + g
//             elsewhere - so that the scattered repair writes of the last pass touch
//             only the elements between T_est and the true threshold (a few percent
//             of k) instead of all k selected positions.
//   k_hist    histogram of the candidates over 2048 fine bins; k_bin (one workgroup
//             per segment) finds the bin b holding the k-th largest key.
//   k_gather  per tile: #candidates in bins above b; the (few) keys inside bin b are
//             gathered per segment. k_select (one workgroup per segment) selects the
//             exact threshold T and tie count among them, fixes the per-tile counts
//             up, and scans them into output offsets.
//   k_emit    ordered emission of (idx, val); repairs the residual where the
//             T_est guess and the true selection differ.
//
// The estimates can never make the result wrong, only slower:
//   * a tile with more candidates than its slot holds is marked, its residual is
//     stored unzeroed, and the later passes re-read that tile from the residual;
//   * a segment with fewer than k candidates, or with more keys in bin b than the
//     gather list holds, gets its residual restored from the slots and is handed to
//     the k_full_* kernels: a plain three-level radix select over the whole segment -
//     unless the overfull bin holds one value only (massive ties: zeros of a frozen
//     layer, values on a grid): then that value is the threshold and its ties are
//     taken in index order without leaving the candidate path.
//   * a segment whose sample holds the candidate threshold's own key hundreds of times (a
//     frozen layer's zeros, a constant) is "tied": its candidates are the keys above that
//     key, nothing is pre-zeroed, and if they are fewer than k the repeated key is the
//     threshold; its ties are counted per tile and taken in index order from the residual.
// The slot size (256 .. 2048 candidates per tile) and the lanes per tile of the candidate
// passes (16, 32 or 64) are chosen per call from the densities seg_k / n_s, so that calls
// at 5 or 10 % keep the same structure (the paper varies rho from 0.001 to 0.1, Exp. 10).
// Per-segment steps run as kernels of their own (a kernel boundary is the only
// device-wide hand-over the normal path needs). The full-segment path is ONE launch (k_full)
// that returns at once when no segment was handed to it; otherwise its five phases hand over
// through a barrier across the grid, which is kept small enough to be resident as a whole.
#include <math.h>

#include <atomic>

#include "ld_common.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / LD_WAVE;
constexpr int kTile = 4096;                       // elements per k_main workgroup
#ifndef LD_SLOT_MIN
#define LD_SLOT_MIN 128
#endif
constexpr int kSlotMin = LD_SLOT_MIN;             // candidate slots per tile: 128 serve densities up to ~1 % (a denser
constexpr int kSlotMax = 2048;                    // layout of the slots made the candidate passes slower); denser calls get more (multiples of 64)
constexpr int kTilesPerGroup = 64;
constexpr int kGroup = kTile * kTilesPerGroup;    // 262144 elements per small-pass workgroup
constexpr int kBins = 2048;
constexpr int kTopBin = kBins - 1;
constexpr int kShift1 = 20, kShift2 = 9;          // radix digits: [30:20] [19:9] [8:0]
constexpr int kPrepThreads = 512;
constexpr int kSample = 16384;                        // sampled elements per segment
constexpr int kSampleItems = kSample / kPrepThreads;
static_assert(kSampleItems <= 32 && kSampleItems % 8 == 0, "valid mask is 32 bits; loads go in batches of 8");
constexpr int kSampleRuns = kSample / LD_WAVE;        // as 256 runs of 64 consecutive elements
constexpr float kSampleZ = 6.5f;                  // safety margin of the rank estimate, in sigmas
constexpr int kGatherBase = 4096;                 // gather list of a segment: kGatherBase + n_s / kGatherPer keys
constexpr int kGatherPer = 4096;
constexpr int kSegPerLaunch = 448;
constexpr int kFullGrid = 1024;                   // most workgroups of the (normally idle) k_full kernel
constexpr uint32_t kModeCand = 0, kModeFull = 1, kModeTies = 2;
constexpr uint32_t kTieSuspect = 512;             // sample keys equal to the candidate threshold (of 16384) that make a segment "tied"

constexpr uint32_t kOverflow = 0xFFFFFFFFu;       // tile count: slot too small, read the residual
constexpr int kSyncCount = 0, kSyncArrived = 1, kSyncGaveUp = 2, kSyncWords = 3;
constexpr int kDictMax = 160;                     // distinct (length, k) pairs of a packed segment table
constexpr int kDictSegs = 2048;                   // segments of a packed segment table

struct SegDesc {        // one per segment plus a sentinel
    int64_t off;        // first element
    int64_t out0;       // first output record
    int32_t k;          // records to keep
    int32_t group0;     // first group
};

struct GroupDesc {      // 64 bytes: all a workgroup needs to know about its group, in one fetch
    int64_t base;       // first element of the group's first tile (multiple of 4; may precede the segment)
    int64_t lo, hi;     // the segment's element range
    int64_t out0;       // the segment's first output record
    int32_t seg;
    int32_t k;          // records the segment keeps
    int32_t group0;     // the segment's first group
    int32_t ngroup;     // groups in the segment
    uint32_t tau;       // candidate threshold (see SegState)
    uint32_t sh;        // fine-bin shift
    uint32_t test;      // guessed threshold
    uint32_t tied;      // 1: the key tau - 1 is massively repeated (see SegState::tied)
};

struct SegState {       // 64 bytes
    uint32_t tau;       // candidate threshold (key); 0: every element, 0xFFFFFFFF: none
    uint32_t sh;        // fine bin of a candidate: min(kTopBin, (key - tau) >> sh)
    uint32_t test;      // guessed threshold T_est >= tau: k_main stores +0 where key >= T_est
    uint32_t prefix;    // k_bin: threshold bin; k_select: exact threshold T (k_full_*: radix prefix)
    uint32_t krem;      // rank left inside prefix; finally the number of ties to keep
    uint32_t mode;      // kModeCand | kModeFull | kModeTies
    uint32_t gcount;    // keys gathered from the threshold bin
    uint32_t fdone[4];  // tickets of the full-segment path: level 1, 2, 3, count
    uint32_t kmin, kmax;  // bounds of the threshold-bin keys that found no room in the gather list
    // A tied segment: the sample found one key repeated so often (a frozen layer's zeros, a constant)
    // that taking it as candidate threshold would make nearly every element a candidate. The
    // candidates are then the keys ABOVE it (tau = that key + 1) and nothing is pre-zeroed. If the
    // candidates turn out fewer than k, the threshold can only be that key or a smaller one:
    // k_gather counts the key per tile in the residual, k_select checks that with those ties k is
    // reached (else: the full path), and k_emit takes the ties in index order (kModeTies).
    uint32_t tied;
    uint32_t pad[2];
};

struct Ctx {
    SegDesc* desc;          // [n_seg + 1]
    GroupDesc* gdesc;       // [n_group]
    SegState* state;        // [n_seg]
    uint32_t* hist;         // [n_seg][kBins]
    uint32_t* cnt;          // [n_group * 64] candidates stored per tile, or kOverflow
    float* cval;            // [n_group * 64][slot]
    uint16_t* cidx;         // [n_group * 64][slot] element offset inside the tile
    uint32_t* tile_gt;      // [n_group * 64] keys above T
    uint32_t* tile_eq;      // [n_group * 64] keys equal to T
    uint32_t* group_gt;     // [n_group] sums over the group -> records emitted before the group
    uint32_t* group_eq;     // [n_group]                       -> ties before the group
    uint32_t* gkey;         // [n_seg][kGatherCap]
    int32_t* gtile;         // [n_seg][kGatherCap]
    int32_t* fail_groups;   // [n_group] groups of segments in kModeFull
    uint32_t* fail_count;   // [kSyncWords]: groups listed; arrivals at k_full's grid barrier; its give-up flag
    int32_t n_seg;
    int32_t n_group;
    int32_t slot;           // candidates a tile can store (kSlotMin .. kSlotMax, multiple of 64)
};

struct UploadBatch {
    int32_t off[kSegPerLaunch + 1];
    int32_t k[kSegPerLaunch];
    int64_t out0;     // records before the first segment of the batch
    int32_t group0;   // groups before it
    int32_t first;    // index of the batch's first segment
    int32_t count;
    int32_t n_seg;
};

// The segment table as k_prep takes it in its arguments when it packs: n_seg = 0 says that it
// did not and that k_upload has written the descriptors.
struct PackedTable {
    uint32_t len[kDictMax];
    uint32_t k[kDictMax];
    uint32_t off0[kDictSegs / LD_WAVE];    // per bucket of 64 segments: elements,
    uint32_t out0[kDictSegs / LD_WAVE];    //   records
    uint32_t group0[kDictSegs / LD_WAVE];  //   and groups before it
    uint8_t code[kDictSegs];
    int32_t n_seg;
};
static_assert(sizeof(PackedTable) + sizeof(Ctx) + 24 <= 4096, "k_prep's arguments must fit a kernel's 4 KB");

__host__ __device__ inline int64_t align_down4(int64_t x) { return x & ~static_cast<int64_t>(3); }

// Gather list of segment s = [lo, hi): first entry and capacity. Derived from the offsets alone,
// so that no table is needed: capacity >= kGatherBase + (hi - lo) / kGatherPer - 1.
__host__ __device__ inline int64_t gather_first(int32_t s, int64_t lo) {
    return static_cast<int64_t>(kGatherBase) * s + lo / kGatherPer;
}
__host__ __device__ inline uint32_t gather_cap(int64_t lo, int64_t hi) {
    return static_cast<uint32_t>(kGatherBase + hi / kGatherPer - lo / kGatherPer);
}

__host__ __device__ inline int32_t groups_of(int64_t off, int64_t end) {
    if (end <= off) return 0;
    return static_cast<int32_t>((end - align_down4(off) + kGroup - 1) / kGroup);
}

// ------------------------------------------------------------ block helpers

// Exclusive scan over NT threads (NT = 256 or 1024); `sh` holds NT/64 words.
template <int NT>
__device__ __forceinline__ uint32_t block_escan(uint32_t x, uint32_t* sh, uint32_t& total) {
    constexpr int NW = NT / LD_WAVE;
    const uint32_t inc = ld_wave_iscan(x);
    const int w = threadIdx.x >> 6;
    if (ld_lane() == LD_WAVE - 1) sh[w] = inc;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        const uint32_t t = sh[i];
        if (i < w) base += t;
        tot += t;
    }
    total = tot;
    __syncthreads();
    return base + inc - x;
}

// Ticket: true in exactly one workgroup per counter - the one that arrives last
// of `expected`. Everything the other workgroups wrote before taking their
// ticket is visible to it.
__device__ __forceinline__ bool last_block(uint32_t* counter, uint32_t expected) {
    __shared__ uint32_t ticket;
    __syncthreads();
    if (threadIdx.x == 0)
        ticket = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const bool last = (ticket == expected - 1);
    if (last) {
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        __syncthreads();
    }
    return last;
}

// In a histogram of kBins counters (global or LDS), scanned from the top bin
// down, finds the bin d with #(bins above d) < krem <= #(bins above d) + h[d].
// The finder writes res[0] = d, res[1] = krem - #(above d); every thread gets the
// histogram total. NT threads, `sh` >= NT/64 words. res is unchanged if krem is
// 0 or exceeds the total.
template <int NT, bool GLOBAL>
__device__ __forceinline__ uint32_t find_bin(const uint32_t* h, uint32_t krem, uint32_t* sh, uint32_t* res) {
    constexpr int per = kBins / NT;
    const int top = kBins - 1 - threadIdx.x * per;  // this thread's highest bin
    uint32_t v[per], sum = 0;
#pragma unroll
    for (int i = 0; i < per; ++i) {
        v[i] = GLOBAL ? ld_load_coherent(h + top - i) : h[top - i];
        sum += v[i];
    }
    uint32_t total;
    uint32_t above = block_escan<NT>(sum, sh, total);
#pragma unroll
    for (int i = 0; i < per; ++i) {
        if (above < krem && krem <= above + v[i]) {
            res[0] = static_cast<uint32_t>(top - i);
            res[1] = krem - above;
        }
        above += v[i];
    }
    __syncthreads();
    return total;
}

__device__ __forceinline__ void flush_hist(uint32_t* h, const uint32_t* lh) {
    for (int b = threadIdx.x; b < kBins; b += blockDim.x) {
        const uint32_t x = lh[b];
        if (x) atomicAdd(h + b, x);
    }
}

// The keys at R ranks (1 = largest), each rounded DOWN to a multiple of
// 2^kShift2: two radix levels resolve the top 22 bits, which is all an estimate
// needs. The ranks share one pass over the keys per level; ranks whose prefixes
// coincide share a histogram. `lh` holds R * kBins words, `res` 2 * R.
template <int NT, int ITEMS, int R>
__device__ void block_select_multi(const uint32_t (&key)[ITEMS], uint32_t valid_mask, const uint32_t (&rank)[R],
                                   uint32_t* lh, uint32_t* sh, uint32_t* res, uint32_t (&out)[R]) {
    uint32_t p[R], kr[R];
#pragma unroll
    for (int i = 0; i < R; ++i) { p[i] = 0; kr[i] = rank[i]; }
#pragma unroll 1
    for (int level = 0; level < 2; ++level) {
        const int match_shift = (level == 0) ? 31 : kShift1;
        const int digit_shift = (level == 0) ? kShift1 : kShift2;
        int own[R];  // the first rank with the same prefix: its histogram serves this one too
#pragma unroll
        for (int i = 0; i < R; ++i) {
            own[i] = i;
#pragma unroll
            for (int j = i - 1; j >= 0; --j)
                if (p[j] == p[i]) own[i] = j;
        }
        for (int b = threadIdx.x; b < R * kBins; b += NT) lh[b] = 0;
        __syncthreads();
#pragma unroll
        for (int q = 0; q < ITEMS; ++q) {
            if (!((valid_mask >> q) & 1u)) continue;
            const uint32_t d = (key[q] >> digit_shift) & 0x7FFu;
#pragma unroll
            for (int i = 0; i < R; ++i)
                if (own[i] == i && (key[q] >> match_shift) == (p[i] >> match_shift)) atomicAdd(&lh[i * kBins + d], 1u);
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < R; ++i) find_bin<NT, false>(lh + own[i] * kBins, kr[i], sh, res + 2 * i);
#pragma unroll
        for (int i = 0; i < R; ++i) {
            p[i] |= res[2 * i] << digit_shift;
            kr[i] = res[2 * i + 1];
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < R; ++i) out[i] = p[i];
}

__device__ __forceinline__ uint32_t mbcnt(uint64_t mask) {  // set bits of `mask` below this lane
    return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
}

__device__ __forceinline__ uint32_t umin(uint32_t a, uint32_t b) { return a < b ? a : b; }

__device__ __forceinline__ uint32_t fine_bin(uint32_t key, uint32_t tau, uint32_t sh) {
    return umin(static_cast<uint32_t>(kTopBin), (key - tau) >> sh);
}

// ------------------------------------------------------------------ geometry

typedef GroupDesc GroupRange;

__device__ __forceinline__ GroupRange group_range(const Ctx& c, int32_t g) {
    const ld_u32x4* p = reinterpret_cast<const ld_u32x4*>(c.gdesc + g);
    union { ld_u32x4 q[4]; GroupDesc d; } u;
#pragma unroll
    for (int i = 0; i < 4; ++i) u.q[i] = p[i];
    return u.d;
}

// Loads the 4 elements at e0..e0+3 that lie inside [lo, hi); returns the mask of
// valid components. e0 is a multiple of 4 and `p` is 16-byte aligned.
__device__ __forceinline__ uint32_t load4(const float* __restrict__ p, int64_t e0, int64_t lo, int64_t hi,
                                          float (&x)[4]) {
    if (e0 >= lo && e0 + 4 <= hi) {
        const ld_f32x4 q = *reinterpret_cast<const ld_f32x4*>(p + e0);
        x[0] = q.x; x[1] = q.y; x[2] = q.z; x[3] = q.w;
        return 0xF;
    }
    uint32_t mask = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        x[c] = 0.0f;
        if (e0 + c >= lo && e0 + c < hi) {
            x[c] = p[e0 + c];
            mask |= 1u << c;
        }
    }
    return mask;
}

__device__ __forceinline__ void store4(float* __restrict__ p, int64_t e0, uint32_t mask, const float (&x)[4]) {
    if (mask == 0xF) {
        *reinterpret_cast<ld_f32x4*>(p + e0) = ld_f32x4{x[0], x[1], x[2], x[3]};
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (mask & (1u << c)) p[e0 + c] = x[c];
    }
}

// -------------------------------------------------------------------- k_prep

__device__ __forceinline__ uint32_t hash32(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

// Segment tables of one batch: prefix sums over the batch entries before each one.
__global__ __launch_bounds__(512) void k_upload(UploadBatch ub, Ctx c) {
    __shared__ uint32_t sh[512 / LD_WAVE];
    const int j = threadIdx.x;
    const bool live = j < ub.count;
    const uint32_t my_groups = live ? static_cast<uint32_t>(groups_of(ub.off[j], ub.off[j + 1])) : 0u;
    const uint32_t my_k = live ? static_cast<uint32_t>(ub.k[j]) : 0u;  // the batch's sum is below 2^31
    uint32_t total;
    const uint32_t groups = block_escan<512>(my_groups, sh, total);
    const uint32_t ks = block_escan<512>(my_k, sh, total);
    if (!live) return;
    const int s = ub.first + j;
    c.desc[s] = SegDesc{ub.off[j], ub.out0 + ks, ub.k[j], ub.group0 + static_cast<int32_t>(groups)};
    if (s == ub.n_seg - 1)
        c.desc[s + 1] = SegDesc{ub.off[j + 1], ub.out0 + ks + my_k, 0,
                                ub.group0 + static_cast<int32_t>(groups + my_groups)};
    if (s == 0)
        for (int i = 0; i < kSyncWords; ++i) c.fail_count[i] = 0;
}

// Descriptor of segment `s` and the end of its range from the packed table. The host has summed
// the segments of every bucket of 64; what is left is a prefix over the segments of the own
// bucket before `s`: one lane per segment, three scans across the first wave.
__device__ __forceinline__ SegDesc desc_from_table(const PackedTable& pt, int32_t s, int64_t& end) {
    __shared__ uint32_t found[5];
    if (threadIdx.x < LD_WAVE) {
        const int bucket = s / LD_WAVE, lane = threadIdx.x;
        const int j = bucket * LD_WAVE + lane;
        const bool live = j < pt.n_seg;
        const uint32_t code = live ? pt.code[j] : 0u;
        const uint32_t len = live ? pt.len[code] : 0u, kk = live ? pt.k[code] : 0u;
        const uint32_t off = pt.off0[bucket] + ld_wave_iscan(len) - len;   // n <= 2^31 - 1: the sums fit 32 bits
        const uint32_t out0 = pt.out0[bucket] + ld_wave_iscan(kk) - kk;
        const uint32_t groups = static_cast<uint32_t>(groups_of(off, static_cast<int64_t>(off) + len));
        const uint32_t group0 = pt.group0[bucket] + ld_wave_iscan(groups) - groups;
        if (j == s) {
            found[0] = off; found[1] = len; found[2] = out0; found[3] = kk; found[4] = group0;
        }
    }
    __syncthreads();
    end = static_cast<int64_t>(found[0]) + found[1];
    return SegDesc{static_cast<int64_t>(found[0]), static_cast<int64_t>(found[2]), static_cast<int32_t>(found[3]),
                   static_cast<int32_t>(found[4])};
}

__global__ __launch_bounds__(kPrepThreads) void k_prep(const float* __restrict__ g,
                                                       const float* __restrict__ r, Ctx c,
                                                       int32_t no_estimate, PackedTable pt) {
    __shared__ uint32_t lh[3 * kBins];
    __shared__ uint32_t sh[kPrepThreads / LD_WAVE];
    __shared__ uint32_t res[6];
    const int s = blockIdx.x;
    SegDesc d;
    int64_t end;
    if (pt.n_seg > 0) {
        d = desc_from_table(pt, s, end);
        if (threadIdx.x == 0) {
            c.desc[s] = d;
            if (s == pt.n_seg - 1)
                c.desc[s + 1] = SegDesc{end, d.out0 + d.k, 0, d.group0 + groups_of(d.off, end)};
            if (s == 0)
                for (int i = 0; i < kSyncWords; ++i) c.fail_count[i] = 0;
        }
    } else {
        d = c.desc[s];
        end = c.desc[s + 1].off;
    }
    const int64_t off = d.off;
    const int32_t k = d.k;
    const int32_t ngroup = groups_of(off, end);
    if (threadIdx.x < sizeof(SegState) / 4) reinterpret_cast<uint32_t*>(&c.state[s])[threadIdx.x] = 0;
    for (int b = threadIdx.x; b < kBins; b += kPrepThreads) c.hist[static_cast<int64_t>(s) * kBins + b] = 0;

    // candidate threshold, guessed threshold and bin width from a sample of |r + g|
    const int64_t ns = end - off;
    uint32_t tau = 0xFFFFFFFFu, test = 0xFFFFFFFFu, binsh = 0, tied = 0;
    if (k > 0 && !no_estimate) {
        uint32_t key[kSampleItems];
        uint32_t valid = 0;
        const bool whole = ns <= kSample;
        const int lane = threadIdx.x & 63;
        const int64_t stride = ns / kSampleRuns;
        if (whole) {
#pragma unroll
            for (int i = 0; i < kSampleItems; ++i) {
                const int64_t e = off + i * kPrepThreads + threadIdx.x;
                key[i] = 0;
                if (e < end) {
                    key[i] = ld_key(__fadd_rn(r[e], g[e]));
                    valid |= 1u << i;
                }
            }
        } else {
            // every run lies inside the segment: no bounds checks, and the loads of kLoadBatch
            // items are issued together (one memory round trip per batch, not per item)
            constexpr int kLoadBatch = 8;
            valid = 0xFFFFFFFFu >> (32 - kSampleItems);
#pragma unroll
            for (int i0 = 0; i0 < kSampleItems; i0 += kLoadBatch) {
                float rv[kLoadBatch], gv[kLoadBatch];
#pragma unroll
                for (int i = 0; i < kLoadBatch; ++i) {
                    const int run = (i0 + i) * (kPrepThreads / LD_WAVE) + (threadIdx.x >> 6);
                    const int64_t jitter = __umulhi(hash32(static_cast<uint32_t>(run) * 2654435761u + static_cast<uint32_t>(s)),
                                                    static_cast<uint32_t>(stride - LD_WAVE + 1));
                    const int64_t e = off + run * stride + jitter + lane;
                    rv[i] = r[e];
                    gv[i] = g[e];
                }
#pragma unroll
                for (int i = 0; i < kLoadBatch; ++i) key[i0 + i] = ld_key(__fadd_rn(rv[i], gv[i]));
            }
        }
        // Sample ranks (1 = largest). The selected keys are rounded down to 2^kShift2, which only
        // adds a few candidates.
        uint32_t rank[3], sel[3];
        bool estimate = true;
        if (whole) {
            // the sample is the segment: the exact threshold lies in [tau, tau + 2^kShift2); every key
            // above that range is certainly selected; bins of width 1
            rank[0] = rank[1] = rank[2] = static_cast<uint32_t>(k);
        } else {
            // expected sample hits a = k * kSample / ns. Candidates: sample rank x with x = a + z*sqrt(x),
            // so that fewer than k elements at or above tau is a z-sigma event. Bins span [tau, hi]
            // where hi is the sample key at rank a - z*sqrt(a): the k-th largest key lies below it, in
            // a fine bin, except in a z-sigma event.
            const float a = static_cast<float>(k) * (static_cast<float>(kSample) / static_cast<float>(ns));
            const float sq = 0.5f * (kSampleZ + sqrtf(kSampleZ * kSampleZ + 4.0f * a));
            rank[0] = static_cast<uint32_t>(sq * sq) + 2u;
            const float lo_rank = a - kSampleZ * sqrtf(a);
            rank[2] = lo_rank > 1.0f ? static_cast<uint32_t>(lo_rank) : 1u;
            const uint32_t mid = static_cast<uint32_t>(a + 0.5f);
            rank[1] = mid < rank[2] ? rank[2] : (mid > rank[0] ? rank[0] : mid);
            estimate = rank[0] < static_cast<uint32_t>(kSample);
        }
        if (!estimate) {
            tau = 0;  // k too large for an estimate: everything is a candidate, nothing is pre-zeroed
            binsh = kShift1;
        } else {
            block_select_multi<kPrepThreads, kSampleItems, 3>(key, valid, rank, lh, sh, res, sel);
            tau = sel[0];
            if (whole) {
                test = tau + (1u << kShift2);
            } else {
                test = sel[1];
                // How often does the sample hold the candidate threshold's own key? (The selected keys
                // are rounded down to 2^kShift2: look at the sample keys of that bucket; if they are
                // many and all one value, that value is massively repeated in the segment.)
                uint32_t same = 0, kmin = 0xFFFFFFFFu, kmax = 0;
#pragma unroll
                for (int i = 0; i < kSampleItems; ++i) {
                    if ((key[i] >> kShift2) == (tau >> kShift2)) {
                        ++same;
                        kmin = umin(kmin, key[i]);
                        kmax = key[i] > kmax ? key[i] : kmax;
                    }
                }
                __syncthreads();
                if (threadIdx.x == 0) { res[0] = 0; res[1] = 0xFFFFFFFFu; res[2] = 0; }
                __syncthreads();
                same = ld_wave_sum(same);
                if ((threadIdx.x & 63) == 0 && same) atomicAdd(&res[0], same);
                if (kmin <= kmax) {
                    atomicMin(&res[1], kmin);
                    atomicMax(&res[2], kmax);
                }
                __syncthreads();
                if (res[0] >= kTieSuspect && res[1] == res[2] && res[1] != 0x7FFFFFFFu) {
                    tied = 1;  // candidates: the keys above it; no pre-zeroing (see SegState::tied)
                    tau = res[1] + 1u;
                    test = 0xFFFFFFFFu;
                }
                const uint32_t top = sel[2] | ((1u << kShift2) - 1u);
                const uint32_t range = top > tau ? top - tau : 0u;
                while ((range >> binsh) > static_cast<uint32_t>(kTopBin - 1)) ++binsh;
            }
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        c.state[s].tau = tau;
        c.state[s].sh = binsh;
        c.state[s].test = test;
        c.state[s].kmin = 0xFFFFFFFFu;
        c.state[s].tied = tied;
    }
    for (int32_t q = threadIdx.x; q < ngroup; q += kPrepThreads)
        c.gdesc[d.group0 + q] = GroupDesc{align_down4(off) + static_cast<int64_t>(q) * kGroup, off, end, d.out0,
                                          s, k, d.group0, ngroup, tau, binsh, test, tied};
}

// -------------------------------------------------------------------- k_main

constexpr int kMainWaves = 1;                                // waves per tile
constexpr int kMainRows = kTile / (kMainWaves * LD_WAVE * 4);  // float4 rows per lane
constexpr int kMainWaveTile = LD_WAVE * 4 * kMainRows;      // consecutive elements per wave

// SMALL: the slots have the minimum size (every call at the usual densities): a constant then.
template <bool SMALL>
__global__ __launch_bounds__(kMainWaves * LD_WAVE) void k_main(const float* __restrict__ g, float* __restrict__ r, Ctx c) {
    const int32_t slot_size = SMALL ? kSlotMin : c.slot;
    __shared__ uint32_t wtot[kMainWaves];
    // consecutive workgroups go to different XCDs: each XCD streams one contiguous eighth of the tiles
    const int32_t tile = static_cast<int32_t>((blockIdx.x % 8) * (gridDim.x / 8) + blockIdx.x / 8);
    const GroupDesc gd = group_range(c, tile / kTilesPerGroup);
    const int lane = ld_lane();
    const int w = threadIdx.x >> 6;
    const int64_t tbase = gd.base + static_cast<int64_t>(tile % kTilesPerGroup) * kTile;
    const int64_t t = tbase + w * kMainWaveTile;
    const int64_t seg_lo = gd.lo, seg_hi = gd.hi;
    if (tbase >= seg_hi) {  // tile slot past the end of the segment
        if (threadIdx.x == 0) c.cnt[tile] = 0;
        return;
    }
    const uint32_t tau = gd.tau, test = gd.test;
    const bool interior = t >= seg_lo && t + kMainWaveTile <= seg_hi;
    float a[kMainRows][4];
    uint32_t mask[kMainRows];
    if (interior) {  // unconditional 16-byte streaming accesses
        const ld_f32x4* g4 = reinterpret_cast<const ld_f32x4*>(g + t) + lane;
        const ld_f32x4* r4 = reinterpret_cast<const ld_f32x4*>(r + t) + lane;
        ld_f32x4 gq[kMainRows], rq[kMainRows];
#pragma unroll
        for (int j = 0; j < kMainRows; ++j) gq[j] = ld_nt_load(g4 + j * LD_WAVE);
#pragma unroll
        for (int j = 0; j < kMainRows; ++j) rq[j] = ld_nt_load(r4 + j * LD_WAVE);
#pragma unroll
        for (int j = 0; j < kMainRows; ++j) {
            a[j][0] = __fadd_rn(rq[j].x, gq[j].x);
            a[j][1] = __fadd_rn(rq[j].y, gq[j].y);
            a[j][2] = __fadd_rn(rq[j].z, gq[j].z);
            a[j][3] = __fadd_rn(rq[j].w, gq[j].w);
            mask[j] = 0xF;
        }
    } else {
#pragma unroll
        for (int j = 0; j < kMainRows; ++j) {
            const int64_t e0 = t + (j * LD_WAVE + lane) * 4;
            float gv[4], rv[4];
            mask[j] = load4(g, e0, seg_lo, seg_hi, gv);
            load4(r, e0, seg_lo, seg_hi, rv);
#pragma unroll
            for (int q = 0; q < 4; ++q) a[j][q] = __fadd_rn(rv[q], gv[q]);
        }
    }
    // candidates, in element order (wave, row, lane, component)
    uint32_t flag[kMainRows], zero[kMainRows], pos0[kMainRows], total = 0;
#pragma unroll
    for (int j = 0; j < kMainRows; ++j) {
        flag[j] = 0;
        zero[j] = 0;
        pos0[j] = total;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t key = ld_key(a[j][q]);
            const bool f = ((mask[j] >> q) & 1u) && key >= tau;
            flag[j] |= static_cast<uint32_t>(f) << q;
            zero[j] |= static_cast<uint32_t>(f && key >= test) << q;
            const uint64_t m = __ballot(f);
            pos0[j] += mbcnt(m);
            total += __popcll(m);
        }
    }
    uint32_t wbase = 0, btot = total;
    if (kMainWaves > 1) {
        if (lane == 0) wtot[w] = total;
        __syncthreads();
        btot = 0;
#pragma unroll
        for (int u = 0; u < kMainWaves; ++u) {
            const uint32_t x = wtot[u];
            if (u < w) wbase += x;
            btot += x;
        }
    }
    const bool fits = btot <= static_cast<uint32_t>(slot_size);  // else: the residual keeps r + g everywhere, the slot stays unused
    if (threadIdx.x == 0) c.cnt[tile] = fits ? btot : kOverflow;
    // residual: +0 where the guessed threshold selects, r + g elsewhere
#pragma unroll
    for (int j = 0; j < kMainRows; ++j) {
        float x[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) x[q] = (fits && ((zero[j] >> q) & 1u)) ? 0.0f : a[j][q];
        if (interior)
            ld_nt_store(ld_f32x4{x[0], x[1], x[2], x[3]}, reinterpret_cast<ld_f32x4*>(r + t) + j * LD_WAVE + lane);
        else
            store4(r, t + (j * LD_WAVE + lane) * 4, mask[j], x);
    }
    if (!fits || total == 0) return;
    float* sv = c.cval + static_cast<int64_t>(tile) * slot_size;
    uint16_t* si = c.cidx + static_cast<int64_t>(tile) * slot_size;
#pragma unroll
    for (int j = 0; j < kMainRows; ++j) {
        if (flag[j] == 0) continue;
        uint32_t pos = wbase + pos0[j];
        const uint32_t local = w * kMainWaveTile + (j * LD_WAVE + lane) * 4;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if ((flag[j] >> q) & 1u) {
                sv[pos] = a[j][q];
                si[pos] = static_cast<uint16_t>(local + q);
                ++pos;
            }
        }
    }
}

// ------------------------------------------------- passes over the candidates
//
// A wave of a small pass owns kTilesPerWave consecutive tiles of its group.
//
// Fast path, for tiles with at most ROW * 8 stored candidates (nearly all of them):
// 64 / ROW tiles at a time, one per row of ROW lanes (four tiles of up to 128 at the
// usual 1 % density). A lane holds 8 consecutive candidates of its row's tile (two
// 16-byte loads of values, one of in-tile offsets), so one trip through the loop body
// serves several tiles, and per-tile sums and prefixes are row operations. These
// passes are bound by instruction issue, not by memory: the body is kept small and
// rolled.
//
// Slow path (slow_tiles), for tiles with more stored candidates and for tiles whose
// slot overflowed (read back from the residual, which then holds r + g unzeroed,
// and filtered with the test k_main applied): begin(u); then item(have, val, local,
// stored) for batches of 64 candidates (one per lane, index order, called by all
// lanes together; `local` is the element's offset inside the tile, `stored` tells
// that the candidate comes from the slot); then end(u).
constexpr int kTilesPerWave = kTilesPerGroup / kWaves;
constexpr int kPerLane = 8;                   // candidates per lane

// Shape of the fast path: ROW lanes per tile (16, 32 or 64, chosen per call from the densities),
// so a trip serves 64 / ROW tiles of at most ROW * 8 candidates each.
template <int ROW>
struct Rows {
    static constexpr int kTiles = LD_WAVE / ROW;                 // tiles per trip
    static constexpr uint32_t kFast = ROW * kPerLane;            // candidates a tile may hold
    static constexpr int kTrips = kTilesPerWave / kTiles;
};

// Slot size as the candidate passes see it: calls that run them with 16 lanes per tile expect at
// most 128 candidates per tile and always get the minimum slot, a constant.
template <int ROW>
__device__ __forceinline__ int32_t slot_of(const Ctx& c) { return ROW == 16 ? kSlotMin : c.slot; }

__device__ __forceinline__ int wave_in_group() { return static_cast<int>(threadIdx.x >> 6) & (kWaves - 1); }

// Lane u < kTilesPerWave: the candidate count of the wave's tile u (k_main writes a
// count for every tile slot of every group, 0 past the end of a segment). Fetched
// first, so that it travels together with the group descriptor.
__device__ __forceinline__ uint32_t wave_counts(const Ctx& c, int32_t group) {
    const int lane = ld_lane();
    const int32_t tile0 = group * kTilesPerGroup + wave_in_group() * kTilesPerWave;
    return lane < kTilesPerWave ? c.cnt[tile0 + lane] : 0u;
}

template <int ROW>
__device__ __forceinline__ uint32_t row_iscan(uint32_t x) {  // inclusive scan over a row of ROW lanes
#pragma unroll
    for (int d = 1; d < ROW; d <<= 1) {
        const uint32_t y = __shfl_up(x, d, ROW);
        if ((ld_lane() & (ROW - 1)) >= d) x += y;
    }
    return x;
}

template <int ROW>
__device__ __forceinline__ uint32_t row_sum(uint32_t x) {
#pragma unroll
    for (int d = ROW / 2; d > 0; d >>= 1) x += __shfl_xor(x, d, ROW);
    return x;
}

struct Trip {
    float v[kPerLane];      // candidate values (entries at or past `have` are stale)
    uint32_t x[kPerLane];   // their offsets inside the tile (IDX only)
    uint32_t have;          // valid entries of this lane: 0..kPerLane
    uint32_t cn;            // stored count of the row's tile (kOverflow, or > ROW * 8: not served here)
    int u;                  // the row's tile, counted inside the wave
};

// The lane's part of trip q (tiles kTiles*q .. of the wave) as it comes from memory: only the
// entries the tile's count says are there (these passes are bound by the bytes they pull from the
// scattered slots: reading whole slots regardless of the counts made them a third slower). The
// trips of a batch are requested together.
struct TripRaw { ld_f32x4 a, b; ld_u32x4 xi; };
constexpr int kAhead = 4;   // trips requested together

template <bool IDX, int ROW>
__device__ __forceinline__ void trip_issue(const Ctx& c, int32_t tile0, uint32_t mycnt, int q, TripRaw& R) {
    typedef Rows<ROW> RW;
    const int lane = ld_lane();
    const int u = RW::kTiles * q + lane / ROW;
    const uint32_t cn = static_cast<uint32_t>(__shfl(static_cast<int>(mycnt), u, LD_WAVE));
    const uint32_t n = cn <= RW::kFast ? cn : 0u;
    const uint32_t first = static_cast<uint32_t>(lane & (ROW - 1)) * kPerLane;
    const int64_t at = static_cast<int64_t>(tile0 + u) * slot_of<ROW>(c) + first;
    R.a = ld_f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    R.b = R.a;
    R.xi = ld_u32x4{0u, 0u, 0u, 0u};
    if (first < n) R.a = *reinterpret_cast<const ld_f32x4*>(c.cval + at);
    if (first + 4 < n) R.b = *reinterpret_cast<const ld_f32x4*>(c.cval + at + 4);
    if (IDX && first < n) R.xi = *reinterpret_cast<const ld_u32x4*>(c.cidx + at);
}

template <bool IDX, int ROW>
__device__ __forceinline__ void trip_finish(const TripRaw& R, uint32_t mycnt, int q, Trip& Q) {
    typedef Rows<ROW> RW;
    const int lane = ld_lane();
    const int u = RW::kTiles * q + lane / ROW;
    const uint32_t cn = static_cast<uint32_t>(__shfl(static_cast<int>(mycnt), u, LD_WAVE));
    const uint32_t n = cn <= RW::kFast ? cn : 0u;
    const uint32_t first = static_cast<uint32_t>(lane & (ROW - 1)) * kPerLane;
    Q.v[0] = R.a.x; Q.v[1] = R.a.y; Q.v[2] = R.a.z; Q.v[3] = R.a.w;
    Q.v[4] = R.b.x; Q.v[5] = R.b.y; Q.v[6] = R.b.z; Q.v[7] = R.b.w;
    if (IDX) {
        const uint32_t xw[4] = {R.xi.x, R.xi.y, R.xi.z, R.xi.w};
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) Q.x[j] = (j & 1) ? (xw[j >> 1] >> 16) : (xw[j >> 1] & 0xFFFFu);
    }
    Q.have = first < n ? umin(n - first, static_cast<uint32_t>(kPerLane)) : 0u;
    Q.cn = cn;
    Q.u = u;
}

// Runs body(Q) for every trip of the wave, kAhead trips requested at a time. `first` holds the
// first batch, requested by the caller as early as it could.
template <bool IDX, int ROW, class Body>
__device__ __forceinline__ void for_trips(const Ctx& c, int32_t tile0, uint32_t mycnt, TripRaw (&first)[kAhead],
                                          Body&& body) {
    static_assert(Rows<ROW>::kTrips % kAhead == 0, "trips come in whole batches");
#pragma unroll 1
    for (int q0 = 0; q0 < Rows<ROW>::kTrips; q0 += kAhead) {
        if (q0 > 0) {
#pragma unroll
            for (int a = 0; a < kAhead; ++a) trip_issue<IDX, ROW>(c, tile0, mycnt, q0 + a, first[a]);
        }
#pragma unroll
        for (int a = 0; a < kAhead; ++a) {
            Trip Q;
            trip_finish<IDX, ROW>(first[a], mycnt, q0 + a, Q);
            body(Q, q0 + a);
        }
    }
}

template <bool IDX, int ROW>
__device__ __forceinline__ void first_trips(const Ctx& c, int32_t tile0, uint32_t mycnt, TripRaw (&first)[kAhead]) {
#pragma unroll
    for (int a = 0; a < kAhead; ++a) trip_issue<IDX, ROW>(c, tile0, mycnt, a, first[a]);
}

template <bool IDX, int ROW, class Begin, class Item, class End>
__device__ __forceinline__ void slow_tiles(const Ctx& c, const float* __restrict__ r, const GroupRange& gr,
                                           int32_t group, uint32_t mycnt, uint32_t tau, Begin&& begin, Item&& item,
                                           End&& end) {
    const int lane = ld_lane();
    const int tl0 = wave_in_group() * kTilesPerWave;
    const int32_t tile0 = group * kTilesPerGroup + tl0;
    const int64_t tbase0 = gr.base + static_cast<int64_t>(tl0) * kTile;
    // tiles of the wave that are not served by the fast path
    uint64_t todo = __ballot(lane < kTilesPerWave && mycnt > Rows<ROW>::kFast);
    while (todo) {
        const int u = __builtin_ctzll(todo);
        todo &= todo - 1;
        const uint32_t cn = static_cast<uint32_t>(__shfl(static_cast<int>(mycnt), u, LD_WAVE));
        const bool stored = cn != kOverflow;
        const uint32_t total = stored ? cn : static_cast<uint32_t>(kTile);
        const int64_t slot = static_cast<int64_t>(tile0 + u) * slot_of<ROW>(c);
        const int64_t tbase = tbase0 + static_cast<int64_t>(u) * kTile;
        begin(u);
        // kAhead batches of 64 are requested before the first is handed on: a tile read back from
        // the residual is 64 batches long, and one load at a time would wait for memory 64 times
        constexpr int kAhead = 4;
#pragma unroll 1
        for (uint32_t b0 = 0; b0 < total; b0 += kAhead * LD_WAVE) {
            bool have[kAhead];
            float v[kAhead];
            uint32_t x[kAhead];
#pragma unroll
            for (int a = 0; a < kAhead; ++a) {
                const uint32_t at = b0 + a * LD_WAVE + lane;
                have[a] = at < total;
                if (stored) {
                    v[a] = have[a] ? c.cval[slot + at] : 0.0f;
                    x[a] = (IDX && have[a]) ? c.cidx[slot + at] : 0u;
                } else {
                    const int64_t e = tbase + at;
                    have[a] = have[a] && e >= gr.lo && e < gr.hi;
                    v[a] = have[a] ? r[e] : 0.0f;
                    x[a] = at;
                }
            }
#pragma unroll
            for (int a = 0; a < kAhead; ++a) {
                if (b0 + a * LD_WAVE < total) {
                    const bool h = stored ? have[a] : (have[a] && ld_key(v[a]) >= tau);
                    item(h, v[a], x[a], stored);
                }
            }
        }
        end(u);
    }
}

__device__ __forceinline__ void mark_full(const Ctx& c, SegState* st, const GroupRange& gr, uint32_t* list0) {
    if (threadIdx.x == 0) {
        st->mode = kModeFull;
        *list0 = atomicAdd(c.fail_count + kSyncCount, static_cast<uint32_t>(gr.ngroup));
    }
    __syncthreads();
    for (int32_t q = threadIdx.x; q < gr.ngroup; q += blockDim.x) c.fail_groups[*list0 + q] = gr.group0 + q;
}

__device__ __forceinline__ GroupRange seg_range(const Ctx& c, int32_t s) {
    GroupRange r;
    const SegDesc d = c.desc[s];
    const SegDesc dn = c.desc[s + 1];
    r.seg = s;
    r.base = align_down4(d.off);
    r.lo = d.off;
    r.hi = dn.off;
    r.k = d.k;
    r.group0 = d.group0;
    r.ngroup = dn.group0 - d.group0;
    r.out0 = d.out0;
    r.tau = r.sh = r.test = r.tied = 0;
    return r;
}

// Fine-bin histogram of the candidates of kHistGroups consecutive groups (256 threads each),
// added to their segments'. Updates of one counter from many workgroups queue up behind one
// another, and the largest segment has hundreds of groups: the groups of a workgroup that
// belong to the same segment are summed in LDS first and added once.
constexpr int kHistGroups = 4;

template <int ROW>
__global__ __launch_bounds__(kHistGroups * kThreads) void k_hist(const float* __restrict__ r, Ctx c) {
    __shared__ uint32_t lh[kHistGroups][kBins];
    __shared__ int32_t qseg[kHistGroups];
    const int q = threadIdx.x / kThreads, tid = threadIdx.x % kThreads;
    const int32_t group = blockIdx.x * kHistGroups + q;
    const bool inside = group < c.n_group;
    const int32_t tile0 = group * kTilesPerGroup + wave_in_group() * kTilesPerWave;
    uint32_t mycnt = 0;
    GroupRange gr;
    gr.k = 0;
    TripRaw raw[kAhead];
    if (inside) {
        mycnt = wave_counts(c, group);
        gr = group_range(c, group);
        first_trips<false, ROW>(c, tile0, mycnt, raw);
    }
    const bool live = inside && gr.k != 0;
    const uint32_t tau = gr.tau, binsh = gr.sh;
    for (int b = tid; b < kBins; b += kThreads) lh[q][b] = 0;
    if (tid == 0) qseg[q] = live ? gr.seg : -1;
    __syncthreads();
    if (live) {
        // keys above the binned range all land in the top bin (a third of the candidates, more
        // at higher densities): counted in a register, added once per wave
        uint32_t top = 0;
        for_trips<false, ROW>(c, tile0, mycnt, raw, [&](const Trip& Q, int) {
#pragma unroll
            for (int j = 0; j < kPerLane; ++j) {
                if (static_cast<uint32_t>(j) < Q.have) {
                    const uint32_t bin = fine_bin(ld_key(Q.v[j]), tau, binsh);
                    if (bin == static_cast<uint32_t>(kTopBin)) ++top; else atomicAdd(&lh[q][bin], 1u);
                }
            }
        });
        slow_tiles<false, ROW>(
            c, r, gr, group, mycnt, tau, [](int) {},
            [&](bool have, float v, uint32_t, bool) {
                const uint32_t bin = fine_bin(ld_key(v), tau, binsh);
                const uint64_t any = __ballot(have);
                if (any == 0) return;
                // massive ties put a whole batch into one bin: one update instead of 64 on one counter
                const uint32_t lead = static_cast<uint32_t>(__shfl(static_cast<int>(bin), __builtin_ctzll(any), LD_WAVE));
                if (__ballot(have && bin == lead) == any) {
                    if (ld_lane() == 0) {
                        if (lead == static_cast<uint32_t>(kTopBin)) top += __popcll(any);
                        else atomicAdd(&lh[q][lead], static_cast<uint32_t>(__popcll(any)));
                    }
                } else if (have) {
                    if (bin == static_cast<uint32_t>(kTopBin)) ++top; else atomicAdd(&lh[q][bin], 1u);
                }
            },
            [](int) {});
        top = ld_wave_sum(top);
        if (ld_lane() == 0 && top) atomicAdd(&lh[q][kTopBin], top);
    }
    __syncthreads();
    if (!live || (q > 0 && qseg[q - 1] == gr.seg)) return;  // summed by the first group of the run
    int run = 1;
    while (q + run < kHistGroups && qseg[q + run] == gr.seg) ++run;
    uint32_t* h = c.hist + static_cast<int64_t>(gr.seg) * kBins;
    for (int b = tid; b < kBins; b += kThreads) {
        uint32_t x = 0;
        for (int j = 0; j < run; ++j) x += lh[q + j][b];
        if (x) atomicAdd(h + b, x);
    }
}

// One workgroup per segment: the fine bin that holds the k-th largest key, or
// the hand-over to the full path when the candidates are fewer than k.
__global__ __launch_bounds__(kThreads) void k_bin(Ctx c) {
    __shared__ uint32_t sh[kWaves];
    __shared__ uint32_t res[2];
    __shared__ uint32_t list0;
    const GroupRange gr = seg_range(c, blockIdx.x);
    if (gr.k == 0 || gr.ngroup == 0) return;
    SegState* st = c.state + gr.seg;
    uint32_t* h = c.hist + static_cast<int64_t>(gr.seg) * kBins;
    if (threadIdx.x == 0) { res[0] = 0; res[1] = 0; }
    __syncthreads();
    const uint32_t total = find_bin<kThreads, false>(h, static_cast<uint32_t>(gr.k), sh, res);
    for (int b = threadIdx.x; b < kBins; b += kThreads) h[b] = 0;  // the full path reuses the row
    if (total >= static_cast<uint32_t>(gr.k)) {
        if (threadIdx.x == 0) { st->prefix = res[0]; st->krem = res[1]; }
    } else if (st->tied) {
        // every candidate is selected; the rest must be ties of the repeated key (k_select checks)
        if (threadIdx.x == 0) {
            st->mode = kModeTies;
            st->prefix = st->tau - 1u;                          // T
            st->krem = static_cast<uint32_t>(gr.k) - total;     // m
        }
    } else {
        mark_full(c, st, gr, &list0);  // the candidate threshold was too high
    }
}

// Elements of the tile starting at tbase whose key is `key`, counted by the whole wave from the
// residual (which holds r + g wherever nothing was zeroed).
__device__ __forceinline__ uint32_t count_key_in_tile(const float* __restrict__ r, int64_t tbase, int64_t lo,
                                                      int64_t hi, uint32_t key) {
    uint32_t n = 0;
#pragma unroll 4
    for (int j = 0; j < kTile / (LD_WAVE * 4); ++j) {
        float x[4];
        const uint32_t mask = load4(r, tbase + (j * LD_WAVE + ld_lane()) * 4, lo, hi, x);
#pragma unroll
        for (int q = 0; q < 4; ++q) n += ((mask >> q) & 1u) && ld_key(x[q]) == key;
    }
    return ld_wave_sum(n);
}

// Keys of the threshold bin held by the lanes of a wave (bit j of `in`: candidate j of the lane)
// go to the segment's gather list: one reservation for the wave. Returns what found no room.
// Kept out of line: the loop around it is bound by instruction fetch, and this runs for a few
// keys per segment only.
struct Unplaced { uint32_t kmin, kmax; bool full; };

__device__ __attribute__((noinline)) Unplaced gather_lane_keys(SegState* st, uint32_t* gkey, int32_t* gtile,
                                                               uint32_t gcap, ld_f32x4 va, ld_f32x4 vb, uint32_t in,
                                                               int32_t tile, bool full) {
    const float v[kPerLane] = {va.x, va.y, va.z, va.w, vb.x, vb.y, vb.z, vb.w};
    Unplaced un{0xFFFFFFFFu, 0u, full};
    const int lane = ld_lane();
    const uint32_t n_in = __popc(in);
    const uint32_t inc = ld_wave_iscan(n_in);
    const uint32_t total = static_cast<uint32_t>(__shfl(static_cast<int>(inc), LD_WAVE - 1, LD_WAVE));
    uint32_t base = gcap;
    if (!full) {
        if (lane == 0) base = atomicAdd(&st->gcount, total);
        base = static_cast<uint32_t>(__shfl(static_cast<int>(base), 0, LD_WAVE));
        un.full = base + total > gcap;
    }
    uint32_t pos = base + inc - n_in;
#pragma unroll
    for (int j = 0; j < kPerLane; ++j) {
        if ((in >> j) & 1u) {
            const uint32_t key = ld_key(v[j]);
            if (pos < gcap) {
                gkey[pos] = key;
                gtile[pos] = tile;
            } else {
                un.kmin = umin(un.kmin, key);
                un.kmax = key > un.kmax ? key : un.kmax;
            }
            ++pos;
        }
    }
    return un;
}

// Per tile: candidates in bins above the threshold bin; the keys inside the bin
// are gathered per segment.
template <int ROW>
__global__ __launch_bounds__(kThreads) void k_gather(const float* __restrict__ r, Ctx c) {
    __shared__ uint32_t wsum[2][kWaves];
    const uint32_t mycnt = wave_counts(c, blockIdx.x);
    const GroupRange gr = group_range(c, blockIdx.x);
    TripRaw raw[kAhead];
    first_trips<false, ROW>(c, blockIdx.x * kTilesPerGroup + (threadIdx.x >> 6) * kTilesPerWave, mycnt, raw);
    SegState* st = c.state + gr.seg;
    const uint32_t mode = st->mode;
    if (gr.k == 0 || mode == kModeFull) return;
    // kModeTies: every candidate lies above the threshold and nothing is gathered; the ties of a
    // tile are what k_main counted
    const bool ties_mode = mode == kModeTies;
    const uint32_t tau = gr.tau, binsh = gr.sh, b1 = st->prefix;
    const int lane = ld_lane();
    const int w = threadIdx.x >> 6;
    uint32_t* gkey = c.gkey + gather_first(gr.seg, gr.lo);
    int32_t* gtile = c.gtile + gather_first(gr.seg, gr.lo);
    const uint32_t gcap = gather_cap(gr.lo, gr.hi);
    const int32_t tile0 = blockIdx.x * kTilesPerGroup + w * kTilesPerWave;
    // Keys of the threshold bin go to the segment's gather list, one reservation per wave and
    // batch. When the list is full (massive ties: millions of equal keys) nothing more is
    // reserved (a wave learns that from its first reservation that comes back beyond the end);
    // the keys that found no room only widen the segment's [kmin, kmax].
    bool full = false;
    uint32_t lmin = 0xFFFFFFFFu, lmax = 0;
    uint32_t part_gt = 0, part_eq = 0;  // fast path: the first lane of a row sums the row's tiles
    uint32_t wave_ties = 0;
    if (ties_mode) {  // the repeated key tau - 1, counted per tile in the residual
        const int tl0 = w * kTilesPerWave;
#pragma unroll 1
        for (int u = 0; u < kTilesPerWave; ++u) {
            const int64_t tbase = gr.base + static_cast<int64_t>(tl0 + u) * kTile;
            const uint32_t t = tbase < gr.hi ? count_key_in_tile(r, tbase, gr.lo, gr.hi, tau - 1u) : 0u;
            if (lane == 0) c.tile_eq[tile0 + u] = t;
            wave_ties += t;
        }
    }
    for_trips<false, ROW>(c, tile0, mycnt, raw, [&](const Trip& Q, int) {
        uint32_t cnt = 0, in = 0;
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) {
            const uint32_t bin = fine_bin(ld_key(Q.v[j]), tau, binsh);
            const bool valid = static_cast<uint32_t>(j) < Q.have;
            cnt += valid && (ties_mode || bin > b1);
            in |= static_cast<uint32_t>(valid && !ties_mode && bin == b1) << j;
        }
        const uint32_t n_in = __popc(in);
        const uint64_t who = __ballot(in != 0);
        if (who) {
            if (full || __popcll(who) >= 4) {  // massive ties: one reservation for the wave, or none
                const Unplaced un = gather_lane_keys(st, gkey, gtile, gcap, ld_f32x4{Q.v[0], Q.v[1], Q.v[2], Q.v[3]},
                                                     ld_f32x4{Q.v[4], Q.v[5], Q.v[6], Q.v[7]}, in, tile0 + Q.u, full);
                lmin = umin(lmin, un.kmin);
                lmax = un.kmax > lmax ? un.kmax : lmax;
                full = un.full;
            } else {  // the usual case: a key or two
#pragma unroll
                for (int j = 0; j < kPerLane; ++j) {
                    if ((in >> j) & 1u) {
                        const uint32_t key = ld_key(Q.v[j]);
                        const uint32_t pos = atomicAdd(&st->gcount, 1u);
                        if (pos < gcap) {
                            gkey[pos] = key;
                            gtile[pos] = tile0 + Q.u;
                        } else {
                            lmin = umin(lmin, key);
                            lmax = key > lmax ? key : lmax;
                        }
                    }
                }
            }
        }
        const uint32_t both = row_sum<ROW>(cnt | (n_in << 16));  // a tile holds at most 512 here
        cnt = both & 0xFFFFu;
        const uint32_t eqc = both >> 16;
        if ((lane & (ROW - 1)) == 0 && Q.cn <= Rows<ROW>::kFast) {
            c.tile_gt[tile0 + Q.u] = cnt;
            if (!ties_mode) c.tile_eq[tile0 + Q.u] = eqc;  // keys in the threshold bin; k_select takes out those that are not T
            part_gt += cnt;
            part_eq += eqc;
        }
    });
    uint32_t slow_gt = 0, slow_eq = 0, gt = 0, eq = 0;
    int32_t tile_of_item = 0;
    slow_tiles<false, ROW>(
        c, r, gr, blockIdx.x, mycnt, tau,
        [&](int u) {
            gt = 0;
            eq = 0;
            tile_of_item = tile0 + u;
        },
        [&](bool have, float v, uint32_t, bool) {
            const uint32_t key = ld_key(v);
            const uint32_t bin = have ? fine_bin(key, tau, binsh) : 0u;
            gt += __popcll(__ballot(have && (ties_mode || bin > b1)));
            const bool in = have && !ties_mode && bin == b1;
            const uint64_t min_ = __ballot(in);
            if (min_) {
                const uint32_t total = static_cast<uint32_t>(__popcll(min_));
                eq += total;
                uint32_t base = gcap;
                if (!full) {
                    if (lane == 0) base = atomicAdd(&st->gcount, total);
                    base = static_cast<uint32_t>(__shfl(static_cast<int>(base), 0, LD_WAVE));
                    full = base + total > gcap;
                }
                const uint32_t pos = base + mbcnt(min_);
                if (in) {
                    if (pos < gcap) {
                        gkey[pos] = key;
                        gtile[pos] = tile_of_item;
                    } else {
                        lmin = umin(lmin, key);
                        lmax = key > lmax ? key : lmax;
                    }
                }
            }
        },
        [&](int u) {
            if (lane == 0) {
                c.tile_gt[tile0 + u] = gt;
                if (!ties_mode) c.tile_eq[tile0 + u] = eq;
            }
            slow_gt += gt;
            slow_eq += eq;
        });
    if (__ballot(lmin <= lmax)) {  // some key of this wave found no room
#pragma unroll
        for (int d = LD_WAVE / 2; d > 0; d >>= 1) {
            lmin = umin(lmin, static_cast<uint32_t>(__shfl_xor(static_cast<int>(lmin), d, LD_WAVE)));
            const uint32_t o = static_cast<uint32_t>(__shfl_xor(static_cast<int>(lmax), d, LD_WAVE));
            lmax = o > lmax ? o : lmax;
        }
        if (lane == 0) {
            atomicMin(&st->kmin, lmin);
            atomicMax(&st->kmax, lmax);
        }
    }
    const uint32_t wave_gt = ld_wave_sum(part_gt) + slow_gt;
    const uint32_t wave_eq = ld_wave_sum(part_eq) + slow_eq + wave_ties;
    if (lane == 0) {
        wsum[0][w] = wave_gt;
        wsum[1][w] = wave_eq;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        c.group_gt[blockIdx.x] = wsum[0][0] + wsum[0][1] + wsum[0][2] + wsum[0][3];
        c.group_eq[blockIdx.x] = wsum[1][0] + wsum[1][1] + wsum[1][2] + wsum[1][3];
    }
}

// One workgroup per segment: the exact threshold T and the number m of its ties to
// keep, selected among the gathered keys; per-tile counts completed; group sums
// scanned into output offsets. All gathered keys lie in one fine bin, so the radix
// select runs on (key - first key of the bin): one 11-bit level per 11 bits of bin
// width, and the digits spread over the histogram instead of piling on one counter.
__global__ __launch_bounds__(kThreads) void k_select(Ctx c) {
    __shared__ uint32_t lh[kBins];
    __shared__ uint32_t sh[kWaves];
    __shared__ uint32_t res[2];
    __shared__ uint32_t list0;
    const GroupRange gr = seg_range(c, blockIdx.x);
    SegState* st = c.state + gr.seg;
    const uint32_t mode = st->mode;
    if (gr.k == 0 || gr.ngroup == 0 || mode == kModeFull) return;
    const uint32_t ng = st->gcount;
    const uint32_t* gkey = c.gkey + gather_first(gr.seg, gr.lo);
    const int32_t* gtile = c.gtile + gather_first(gr.seg, gr.lo);
    const uint32_t gcap = gather_cap(gr.lo, gr.hi);
    uint32_t T, m;
    uint32_t seen = 0;
    if (mode == kModeTies) {  // k_bin has found both: nothing to select
        T = st->prefix;
        m = st->krem;
    } else if (ng > gcap) {
        // More keys in the threshold bin than the list holds. If they are all one value (massive
        // ties: a frozen layer's zeros, values on a coarse grid) nothing has to be selected among
        // them: T is that value, and the rank left inside the bin is the number of ties to keep,
        // lowest index first. k_gather's per-tile counts of the bin are then the tie counts.
        if (threadIdx.x == 0) { res[0] = st->kmin; res[1] = st->kmax; }
        __syncthreads();
        uint32_t lmin = 0xFFFFFFFFu, lmax = 0;
#pragma unroll 1
        for (uint32_t p = threadIdx.x; p < gcap; p += kThreads) {
            const uint32_t key = gkey[p];
            lmin = umin(lmin, key);
            lmax = key > lmax ? key : lmax;
        }
        atomicMin(&res[0], lmin);
        atomicMax(&res[1], lmax);
        __syncthreads();
        if (res[0] != res[1]) {
            mark_full(c, st, gr, &list0);  // several values share an overfull bin
            return;
        }
        T = res[0];
        m = st->krem;
        __syncthreads();
    } else {
        const uint32_t b1 = st->prefix, binsh = st->sh;
        const uint32_t base = st->tau + (b1 << binsh);
        const int bits = (b1 == static_cast<uint32_t>(kTopBin)) ? 31 : static_cast<int>(binsh);  // the top bin is open-ended
        const int nlev = bits == 0 ? 1 : (bits + 10) / 11;
        uint32_t prefix = 0, krem = st->krem;
#pragma unroll 1
        for (int lev = 0; lev < nlev; ++lev) {
            const int shift = 11 * (nlev - 1 - lev);
            for (int b = threadIdx.x; b < kBins; b += kThreads) lh[b] = 0;
            __syncthreads();
#pragma unroll 1
            for (uint32_t p = threadIdx.x; p < ng; p += kThreads) {
                const uint32_t rel = gkey[p] - base;
                if (lev == 0 || ((rel ^ prefix) >> (shift + 11)) == 0) atomicAdd(&lh[(rel >> shift) & 0x7FFu], 1u);
            }
            __syncthreads();
            find_bin<kThreads, false>(lh, krem, sh, res);
            prefix |= res[0] << shift;
            krem = res[1];
            __syncthreads();
        }
        T = base + prefix;
        m = krem;
        // k_gather counted every key of the bin as a tie: move those above T to the counts of the
        // selected, drop those below. The group sums are read back below by this same workgroup.
        // The updates return their old value, so each has been performed when its result arrives;
        // with the barrier that orders them before the reads. (A device-scope fence would do too,
        // but it writes back the whole L2 and costs 30 us here.)
#pragma unroll 1
        for (uint32_t p = threadIdx.x; p < ng; p += kThreads) {
            const uint32_t key = gkey[p];
            if (key == T) continue;
            const int32_t tile = gtile[p];
            atomicSub(c.tile_eq + tile, 1u);
            seen |= atomicSub(c.group_eq + tile / kTilesPerGroup, 1u);
            if (key > T) {
                atomicAdd(c.tile_gt + tile, 1u);
                seen |= atomicAdd(c.group_gt + tile / kTilesPerGroup, 1u);
            }
        }
    }
    if (seen == 0xFFFFFFFFu) res[0] = seen;  // never true: keeps the results, and so the waits, alive
    __syncthreads();
    // exclusive scan over the segment's groups: records emitted / ties seen before each
    uint32_t carry_out = 0, carry_eq = 0;
#pragma unroll 1
    for (int32_t q0 = 0; q0 < gr.ngroup; q0 += kThreads) {
        const int32_t q = q0 + threadIdx.x;
        uint32_t cg = 0, ce = 0;
        if (q < gr.ngroup) {
            cg = ld_load_coherent(c.group_gt + gr.group0 + q);
            ce = ld_load_coherent(c.group_eq + gr.group0 + q);
        }
        uint32_t te, tg;
        const uint32_t eq_before = carry_eq + block_escan<kThreads>(ce, sh, te);
        const uint32_t take = umin(eq_before + ce, m) - umin(eq_before, m);  // ties kept: lowest index first
        const uint32_t out_before = carry_out + block_escan<kThreads>(cg + take, sh, tg);
        if (q < gr.ngroup) {
            c.group_gt[gr.group0 + q] = out_before;
            c.group_eq[gr.group0 + q] = eq_before;
        }
        carry_eq += te;
        carry_out += tg;
    }
    if (mode == kModeTies && carry_eq < m) {
        mark_full(c, st, gr, &list0);  // the repeated key does not fill k either: the threshold lies below it
        return;
    }
    if (threadIdx.x == 0) { st->prefix = T; st->krem = m; }
}

// Ordered emission of the records. k_main left +0 in the residual exactly where a
// stored candidate's key reaches T_est; only where that guess and the selection
// differ is the residual written again. A segment handed to the full path gets
// every pre-zeroed position back instead.
template <int ROW>
__global__ __launch_bounds__(kThreads) void k_emit(float* __restrict__ r, int32_t* __restrict__ out_idx,
                                                   float* __restrict__ out_val, Ctx c) {
    __shared__ uint32_t tile_out[kTilesPerGroup], tile_eqb[kTilesPerGroup], tile_take[kTilesPerGroup];
    constexpr int kTiles = Rows<ROW>::kTiles;
    constexpr uint32_t kFast = Rows<ROW>::kFast;
    __shared__ int32_t stage_i[kWaves][kTiles * kFast];
    __shared__ float stage_v[kWaves][kTiles * kFast];
    uint32_t mycnt = wave_counts(c, blockIdx.x);
    const GroupRange gr = group_range(c, blockIdx.x);
    TripRaw raw[kAhead];
    first_trips<true, ROW>(c, blockIdx.x * kTilesPerGroup + (threadIdx.x >> 6) * kTilesPerWave, mycnt, raw);
    const SegState* st = c.state + gr.seg;
    if (gr.k == 0) return;
    const uint32_t mode = st->mode;
    const uint32_t tau = gr.tau, test = gr.test, T = st->prefix, m = st->krem;
    const int lane = ld_lane();
    const int w = threadIdx.x >> 6;
    const int tl0 = w * kTilesPerWave;
    const int32_t tile0 = blockIdx.x * kTilesPerGroup + tl0;
    int64_t tbase = 0;
    if (mode == kModeFull) {
        for_trips<true, ROW>(c, tile0, mycnt, raw, [&](const Trip& Q, int) {
            float* rt = r + gr.base + static_cast<int64_t>(tl0 + Q.u) * kTile;
#pragma unroll
            for (int j = 0; j < kPerLane; ++j)
                if (static_cast<uint32_t>(j) < Q.have && ld_key(Q.v[j]) >= test) rt[Q.x[j]] = Q.v[j];
        });
        slow_tiles<true, ROW>(
            c, r, gr, blockIdx.x, mycnt, tau,
            [&](int u) { tbase = gr.base + static_cast<int64_t>(tl0 + u) * kTile; },
            [&](bool have, float v, uint32_t local, bool stored) {
                if (have && stored && ld_key(v) >= test) r[tbase + local] = v;
            },
            [](int) {});
        return;
    }
    if (w == 0) {  // offsets of the group's 64 tiles
        const int32_t tile = blockIdx.x * kTilesPerGroup + lane;
        const bool live = gr.base + static_cast<int64_t>(lane) * kTile < gr.hi;
        const uint32_t cg = live ? c.tile_gt[tile] : 0u, ce = live ? c.tile_eq[tile] : 0u;
        const uint32_t eq_before = c.group_eq[blockIdx.x] + ld_wave_iscan(ce) - ce;
        const uint32_t take = umin(eq_before + ce, m) - umin(eq_before, m);
        tile_out[lane] = c.group_gt[blockIdx.x] + ld_wave_iscan(cg + take) - (cg + take);
        tile_eqb[lane] = eq_before;
        tile_take[lane] = take;
    }
    __syncthreads();
    // kModeTies: the ties are not among the stored candidates. A tile that keeps some of them is
    // read back from the residual (nothing was pre-zeroed in a tied segment), where candidates and
    // ties come in index order; keys at or above T pass the filter there.
    const uint32_t keep_from = mode == kModeTies ? T : tau;
    if (mode == kModeTies && lane < kTilesPerWave && tile_take[tl0 + lane] > 0) mycnt = kOverflow;
    for_trips<true, ROW>(c, tile0, mycnt, raw, [&](const Trip& Q, int q) {
        const uint32_t out_tile = tile_out[tl0 + Q.u], eq_tile = tile_eqb[tl0 + Q.u];
        uint32_t gtm = 0, eqm = 0;
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) {
            const uint32_t key = ld_key(Q.v[j]);
            const bool valid = static_cast<uint32_t>(j) < Q.have;
            gtm |= static_cast<uint32_t>(valid && key > T) << j;
            eqm |= static_cast<uint32_t>(valid && key == T) << j;
        }
        const uint32_t mine = __popc(gtm) | (__popc(eqm) << 16);  // a tile holds at most 512 here
        const uint32_t before = row_iscan<ROW>(mine) - mine;
        uint32_t gt_before = before & 0xFFFFu;
        uint32_t eq_rank = eq_tile + (before >> 16);
        float* rt = r + gr.base + static_cast<int64_t>(tl0 + Q.u) * kTile;
        const int32_t e0 = static_cast<int32_t>(gr.base + static_cast<int64_t>(tl0 + Q.u) * kTile);
        // the records of a row's tile are staged in LDS at their rank inside the tile and then
        // written out as contiguous runs (stores of single records from scattered lanes cost
        // three times as much)
        int32_t* si = stage_i[w] + (lane / ROW) * kFast;
        float* sv = stage_v[w] + (lane / ROW) * kFast;
        uint32_t rank = 0;
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) {
            const bool is_gt = (gtm >> j) & 1u, is_eq = (eqm >> j) & 1u;
            const bool selected = is_gt || (is_eq && eq_rank < m);
            rank = gt_before + (umin(eq_rank, m) - umin(eq_tile, m));
            if (selected) {
                si[rank] = e0 + static_cast<int32_t>(Q.x[j]);
                sv[rank] = Q.v[j];
            }
            const bool zeroed = ld_key(Q.v[j]) >= test;
            if (static_cast<uint32_t>(j) < Q.have && selected != zeroed) rt[Q.x[j]] = selected ? 0.0f : Q.v[j];
            gt_before += is_gt;
            eq_rank += is_eq;
        }
        rank = gt_before + (umin(eq_rank, m) - umin(eq_tile, m));  // in a row's last lane: records of the tile
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
#pragma unroll
        for (int row = 0; row < kTiles; ++row) {
            const uint32_t cnt = static_cast<uint32_t>(__shfl(static_cast<int>(rank), row * ROW + ROW - 1, LD_WAVE));
            const int64_t o0 = gr.out0 + tile_out[tl0 + kTiles * q + row];
            for (uint32_t i = lane; i < cnt; i += LD_WAVE) {
                // streamed past the caches: the records are read much later, by another call
                __builtin_nontemporal_store(stage_i[w][row * kFast + i], out_idx + o0 + i);
                __builtin_nontemporal_store(stage_v[w][row * kFast + i], out_val + o0 + i);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    });
    uint32_t run_out = 0;  // records of the segment emitted before this point
    uint32_t run_eq = 0;   // ties seen before this point
    slow_tiles<true, ROW>(
        c, r, gr, blockIdx.x, mycnt, keep_from,
        [&](int u) {
            run_out = tile_out[tl0 + u];
            run_eq = tile_eqb[tl0 + u];
            tbase = gr.base + static_cast<int64_t>(tl0 + u) * kTile;
        },
        [&](bool have, float v, uint32_t local, bool stored) {
            const uint32_t key = ld_key(v);
            const bool is_gt = have && key > T;
            const bool is_eq = have && key == T;
            const uint64_t mg = __ballot(is_gt), me = __ballot(is_eq);
            const uint32_t eq_rank = run_eq + mbcnt(me);
            const bool selected = is_gt || (is_eq && eq_rank < m);
            const int64_t e = tbase + local;
            if (selected) {
                const int64_t pos = gr.out0 + run_out + mbcnt(mg) + (umin(eq_rank, m) - umin(run_eq, m));
                out_idx[pos] = static_cast<int32_t>(e);
                out_val[pos] = v;
            }
            const bool zeroed = stored && key >= test;
            if (have && selected != zeroed) r[e] = selected ? 0.0f : v;
            const uint32_t eq_end = run_eq + __popcll(me);
            run_out += __popcll(mg) + (umin(eq_end, m) - umin(run_eq, m));
            run_eq = eq_end;
        },
        [](int) {});
}

// ------------------------------------------ full-segment path (kModeFull only)
// Plain three-level radix select over every element of the listed groups.

struct FullRange { GroupRange gr; int64_t cs, ce; };

__device__ __forceinline__ FullRange full_range(const Ctx& c, int32_t g) {
    FullRange f;
    f.gr = group_range(c, g);
    f.cs = f.gr.base < f.gr.lo ? f.gr.lo : f.gr.base;
    f.ce = (f.gr.base + kGroup) > f.gr.hi ? f.gr.hi : (f.gr.base + kGroup);
    return f;
}

template <int LEVEL>
__device__ __forceinline__ void full_level(const float* __restrict__ r, const Ctx& c, uint32_t nlist, uint32_t* lh,
                                           uint32_t* sh, uint32_t* res) {
    constexpr int match_shift = (LEVEL == 1) ? 31 : (LEVEL == 2 ? kShift1 : kShift2);
    constexpr int digit_shift = (LEVEL == 1) ? kShift1 : (LEVEL == 2 ? kShift2 : 0);
    constexpr uint32_t digit_mask = (LEVEL == 3) ? 0x1FFu : 0x7FFu;
    for (uint32_t li = blockIdx.x; li < nlist; li += gridDim.x) {
        const FullRange fr = full_range(c, c.fail_groups[li]);
        SegState* st = c.state + fr.gr.seg;
        const uint32_t prefix = (LEVEL == 1) ? 0u : st->prefix;
        const uint32_t krem = (LEVEL == 1) ? static_cast<uint32_t>(fr.gr.k) : st->krem;
        for (int b = threadIdx.x; b < kBins; b += kThreads) lh[b] = 0;
        __syncthreads();
        for (int64_t t = fr.gr.base; t < fr.ce; t += kThreads * 4) {
            float x[4];
            const uint32_t mask = load4(r, t + threadIdx.x * 4, fr.cs, fr.ce, x);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t key = ld_key(x[q]);
                if (((mask >> q) & 1u) && (key >> match_shift) == (prefix >> match_shift))
                    atomicAdd(&lh[(key >> digit_shift) & digit_mask], 1u);
            }
        }
        __syncthreads();
        uint32_t* h = c.hist + static_cast<int64_t>(fr.gr.seg) * kBins;
        flush_hist(h, lh);
        if (last_block(&st->fdone[LEVEL - 1], static_cast<uint32_t>(fr.gr.ngroup))) {
            find_bin<kThreads, true>(h, krem, sh, res);
            for (int b = threadIdx.x; b < kBins; b += kThreads) h[b] = 0;
            if (threadIdx.x == 0) {
                st->prefix = prefix | (res[0] << digit_shift);
                st->krem = res[1];
            }
        }
        __syncthreads();
    }
}

__device__ __forceinline__ void full_count(const float* __restrict__ r, const Ctx& c, uint32_t nlist, uint32_t* sh) {
    for (uint32_t li = blockIdx.x; li < nlist; li += gridDim.x) {
        const int32_t g = c.fail_groups[li];
        const FullRange fr = full_range(c, g);
        SegState* st = c.state + fr.gr.seg;
        const uint32_t T = st->prefix, m = st->krem;
        uint32_t gt = 0, eq = 0;
        for (int64_t t = fr.gr.base; t < fr.ce; t += kThreads * 4) {
            float x[4];
            const uint32_t mask = load4(r, t + threadIdx.x * 4, fr.cs, fr.ce, x);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t key = ld_key(x[q]);
                if ((mask >> q) & 1u) { gt += (key > T); eq += (key == T); }
            }
        }
        uint32_t tot_gt, tot_eq;
        block_escan<kThreads>(gt, sh, tot_gt);
        block_escan<kThreads>(eq, sh, tot_eq);
        if (threadIdx.x == 0) { c.group_gt[g] = tot_gt; c.group_eq[g] = tot_eq; }
        if (last_block(&st->fdone[3], static_cast<uint32_t>(fr.gr.ngroup))) {
            uint32_t carry_out = 0, carry_eq = 0;
            for (int32_t q0 = 0; q0 < fr.gr.ngroup; q0 += kThreads) {
                const int32_t q = q0 + threadIdx.x;
                uint32_t cg = 0, ce = 0;
                if (q < fr.gr.ngroup) {
                    cg = ld_load_coherent(c.group_gt + fr.gr.group0 + q);
                    ce = ld_load_coherent(c.group_eq + fr.gr.group0 + q);
                }
                uint32_t te, tg;
                const uint32_t eq_before = carry_eq + block_escan<kThreads>(ce, sh, te);
                const uint32_t take = umin(eq_before + ce, m) - umin(eq_before, m);
                const uint32_t out_before = carry_out + block_escan<kThreads>(cg + take, sh, tg);
                if (q < fr.gr.ngroup) {
                    c.group_gt[fr.gr.group0 + q] = out_before;
                    c.group_eq[fr.gr.group0 + q] = eq_before;
                }
                carry_eq += te;
                carry_out += tg;
            }
        }
        __syncthreads();
    }
}

__device__ __forceinline__ void full_emit(float* __restrict__ r, int32_t* __restrict__ out_idx,
                                          float* __restrict__ out_val, const Ctx& c, uint32_t nlist,
                                          uint32_t (*part)[kWaves]) {  // part: packed (above | ties << 16) per wave
    const int lane = ld_lane();
    const int wv = threadIdx.x >> 6;
    for (uint32_t li = blockIdx.x; li < nlist; li += gridDim.x) {
        const int32_t g = c.fail_groups[li];
        const FullRange fr = full_range(c, g);
        const SegState* st = c.state + fr.gr.seg;
        const uint32_t T = st->prefix, m = st->krem;
        uint32_t run_out = c.group_gt[g], run_eq = c.group_eq[g];
        int buf = 0;
        // element order inside a step of 1024: (thread, component)
        for (int64_t t = fr.gr.base; t < fr.ce; t += kThreads * 4, buf ^= 1) {
            const int64_t e0 = t + threadIdx.x * 4;
            float x[4];
            const uint32_t mask = load4(r, e0, fr.cs, fr.ce, x);
            uint32_t fg = 0, fe = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t key = ld_key(x[q]);
                if ((mask >> q) & 1u) {
                    fg |= static_cast<uint32_t>(key > T) << q;
                    fe |= static_cast<uint32_t>(key == T) << q;
                }
            }
            const uint32_t cg = __popc(fg), ce = __popc(fe);
            const uint32_t inc = ld_wave_iscan(cg | (ce << 16));
            if (lane == LD_WAVE - 1) part[buf][wv] = inc;
            __syncthreads();
            uint32_t base_gt = 0, base_eq = 0, tot_gt = 0, tot_eq = 0;
#pragma unroll
            for (int u = 0; u < kWaves; ++u) {
                const uint32_t p = part[buf][u];
                if (u < wv) { base_gt += p & 0xFFFFu; base_eq += p >> 16; }
                tot_gt += p & 0xFFFFu;
                tot_eq += p >> 16;
            }
            uint32_t gt_before = base_gt + (inc & 0xFFFFu) - cg;
            uint32_t eq_rank = run_eq + base_eq + (inc >> 16) - ce;
            bool touched = false;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bool is_gt = (fg >> q) & 1u, is_eq = (fe >> q) & 1u;
                if (is_gt || (is_eq && eq_rank < m)) {
                    const int64_t pos = fr.gr.out0 + run_out + gt_before + (umin(eq_rank, m) - umin(run_eq, m));
                    out_idx[pos] = static_cast<int32_t>(e0 + q);
                    out_val[pos] = x[q];
                    x[q] = 0.0f;
                    touched = true;
                }
                gt_before += is_gt;
                eq_rank += is_eq;
            }
            if (touched) store4(r, e0, mask, x);
            const uint32_t eq_end = run_eq + tot_eq;
            run_out += tot_gt + (umin(eq_end, m) - umin(run_eq, m));
            run_eq = eq_end;
        }
        __syncthreads();
    }
}

// Barrier across the grid of k_full: every workgroup adds one arrival and waits until `target`
// have come. Needs every workgroup of the grid resident at once (the host sizes the grid for
// that). The wait is bounded: a workgroup that has polled kSpinLimit times (seconds; a barrier
// takes microseconds) raises the give-up flag, and every workgroup that sees the flag leaves the
// kernel, so the grid always drains. Returns false when the kernel is to be left.
constexpr uint32_t kSpinLimit = 1u << 21;

__device__ __forceinline__ bool grid_barrier(uint32_t* sync, uint32_t target) {
    __shared__ uint32_t go;
    __syncthreads();
    if (threadIdx.x == 0) {
        __hip_atomic_fetch_add(sync + kSyncArrived, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        uint32_t ok = 1, spins = 0;
        while (__hip_atomic_load(sync + kSyncArrived, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < target) {
            if (__hip_atomic_load(sync + kSyncGaveUp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0 ||
                ++spins > kSpinLimit) {
                __hip_atomic_store(sync + kSyncGaveUp, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ok = 0;
                break;
            }
            __builtin_amdgcn_s_sleep(64);
        }
        go = ok;
    }
    __syncthreads();
    const bool ok = go != 0;
    if (ok) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    __syncthreads();
    return ok;
}

// The whole full-segment path in one launch: nothing listed (the usual case), nothing done.
__global__ __launch_bounds__(kThreads) void k_full(float* __restrict__ r, int32_t* __restrict__ out_idx,
                                                   float* __restrict__ out_val, Ctx c) {
    __shared__ uint32_t lh[kBins];
    __shared__ uint32_t sh[kWaves];
    __shared__ uint32_t res[2];
    __shared__ uint32_t part[2][kWaves];
    const uint32_t nlist = c.fail_count[kSyncCount];
    if (nlist == 0) return;
    full_level<1>(r, c, nlist, lh, sh, res);
    if (!grid_barrier(c.fail_count, 1 * gridDim.x)) return;
    full_level<2>(r, c, nlist, lh, sh, res);
    if (!grid_barrier(c.fail_count, 2 * gridDim.x)) return;
    full_level<3>(r, c, nlist, lh, sh, res);
    if (!grid_barrier(c.fail_count, 3 * gridDim.x)) return;
    full_count(r, c, nlist, sh);
    if (!grid_barrier(c.fail_count, 4 * gridDim.x)) return;
    full_emit(r, out_idx, out_val, c, nlist, part);
}

// ---------------------------------------------------------------- host side

struct Layout {
    size_t desc, gdesc, state, hist, cnt, cval, cidx, tile_gt, tile_eq, group_gt, group_eq, gkey, gtile,
        fail_groups, fail_count, total;
};

Layout layout(int32_t n_seg, int64_t n_group, int32_t slot) {
    Layout L;
    size_t o = 0;
    const size_t ns = static_cast<size_t>(n_seg), ng = static_cast<size_t>(n_group), nt = ng * kTilesPerGroup;
    auto take = [&](size_t bytes) { const size_t at = o; o += ld_round_up(bytes, 256); return at; };
    L.desc = take(sizeof(SegDesc) * (ns + 1));
    L.gdesc = take(sizeof(GroupDesc) * ng);
    L.state = take(sizeof(SegState) * ns);
    L.hist = take(sizeof(uint32_t) * kBins * ns);
    L.cnt = take(4 * nt);
    L.tile_gt = take(4 * nt);
    L.tile_eq = take(4 * nt);
    L.group_gt = take(4 * ng);
    L.group_eq = take(4 * ng);
    const size_t gather_entries = static_cast<size_t>(kGatherBase) * ns + nt * (kTile / kGatherPer) + 1;
    L.gkey = take(4 * gather_entries);
    L.gtile = take(4 * gather_entries);
    L.fail_groups = take(4 * ng);
    L.fail_count = take(4 * kSyncWords);
    L.cval = take(4 * nt * static_cast<size_t>(slot));  // the two arrays whose size depends on `slot` come last
    L.cidx = take(2 * nt * static_cast<size_t>(slot));
    L.total = o;
    return L;
}

// Counts groups; returns -1 on a malformed offset table.
int64_t count_groups(int32_t n_seg, const int64_t* seg_off) {
    if (n_seg < 0 || (n_seg > 0 && !seg_off)) return -1;
    if (n_seg > 0 && seg_off[0] != 0) return -1;
    int64_t total = 0;
    for (int32_t s = 0; s < n_seg; ++s) {
        if (seg_off[s + 1] < seg_off[s]) return -1;
        total += groups_of(seg_off[s], seg_off[s + 1]);
    }
    return total;
}

// Slot size that holds the candidates of a tile in all but a few tiles: the candidate threshold
// of k_prep sits at sample rank x = a + z*sqrt(x) (a = k * kSample / n_s expected hits), i.e. a
// fraction x / kSample of the elements are candidates, plus five sigmas of a tile's own count.
// Taken over the segments of at least 16 tiles (the tiles of smaller ones may overflow into the
// residual re-read: there are few of them).
int32_t wanted_slot(int32_t n_seg, const int64_t* seg_off, const int32_t* seg_k, int32_t* per_tile = nullptr) {
    double most = 0.0;
    for (int32_t s = 0; s < n_seg; ++s) {
        const int64_t ns = seg_off[s + 1] - seg_off[s];
        if (ns < 16 * kTile || seg_k[s] <= 0) continue;
        const double a = static_cast<double>(seg_k[s]) * kSample / static_cast<double>(ns);
        const double sq = 0.5 * (kSampleZ + sqrt(kSampleZ * kSampleZ + 4.0 * a));
        const double x = sq * sq + 2.0;
        if (x >= kSample) continue;  // no estimate for this segment: every element is a candidate
        const double per_tile = x * kTile / kSample;
        const double need = per_tile + 5.0 * sqrt(per_tile) + 8.0;
        if (need > most) most = need;
    }
    if (per_tile) *per_tile = static_cast<int32_t>(most);
    int64_t slot = (static_cast<int64_t>(most) + 63) / 64 * 64;
    if (slot < kSlotMin) slot = kSlotMin;
    if (slot > kSlotMax) slot = kSlotMax;
    return static_cast<int32_t>(slot);
}

Ctx make_ctx(void* workspace, const Layout& L, int32_t n_seg, int64_t n_group, int32_t slot) {
    char* ws = static_cast<char*>(workspace);
    Ctx c;
    c.desc = reinterpret_cast<SegDesc*>(ws + L.desc);
    c.gdesc = reinterpret_cast<GroupDesc*>(ws + L.gdesc);
    c.state = reinterpret_cast<SegState*>(ws + L.state);
    c.hist = reinterpret_cast<uint32_t*>(ws + L.hist);
    c.cnt = reinterpret_cast<uint32_t*>(ws + L.cnt);
    c.cval = reinterpret_cast<float*>(ws + L.cval);
    c.cidx = reinterpret_cast<uint16_t*>(ws + L.cidx);
    c.tile_gt = reinterpret_cast<uint32_t*>(ws + L.tile_gt);
    c.tile_eq = reinterpret_cast<uint32_t*>(ws + L.tile_eq);
    c.group_gt = reinterpret_cast<uint32_t*>(ws + L.group_gt);
    c.group_eq = reinterpret_cast<uint32_t*>(ws + L.group_eq);
    c.gkey = reinterpret_cast<uint32_t*>(ws + L.gkey);
    c.gtile = reinterpret_cast<int32_t*>(ws + L.gtile);
    c.fail_groups = reinterpret_cast<int32_t*>(ws + L.fail_groups);
    c.fail_count = reinterpret_cast<uint32_t*>(ws + L.fail_count);
    c.n_seg = n_seg;
    c.n_group = static_cast<int32_t>(n_group);
    c.slot = slot;
    return c;
}

// One workgroup per segment: the path the last call took for it, and how many of its tiles
// overflowed their candidate slot.
__global__ __launch_bounds__(kThreads) void k_paths(Ctx c, int32_t* __restrict__ paths, int32_t* __restrict__ overflowed) {
    __shared__ uint32_t sh[kWaves];
    const int32_t s = blockIdx.x;
    const SegDesc d = c.desc[s], dn = c.desc[s + 1];
    uint32_t over = 0;
    if (d.k > 0) {
        const int64_t t0 = static_cast<int64_t>(d.group0) * kTilesPerGroup, t1 = static_cast<int64_t>(dn.group0) * kTilesPerGroup;
        for (int64_t t = t0 + threadIdx.x; t < t1; t += kThreads) over += c.cnt[t] == kOverflow;
    }
    uint32_t total;
    block_escan<kThreads>(over, sh, total);
    if (threadIdx.x == 0) {
        const SegState st = c.state[s];
        paths[s] = static_cast<int32_t>(st.mode | (st.tied ? 0x100u : 0u) |
                                        (c.fail_count[kSyncGaveUp] ? 0x10000u : 0u));
        if (overflowed) overflowed[s] = static_cast<int32_t>(total);
    }
}

// Packs the segment table for k_prep's arguments; false when it has too many segments or too
// many distinct (length, k) pairs.
bool pack_table(int32_t n_seg, const int64_t* seg_off, const int32_t* seg_k, PackedTable& pt) {
    pt.n_seg = 0;
    if (n_seg > kDictSegs) return false;
    int used = 0, last = 0;
    for (int32_t s = 0; s < n_seg; ++s) {
        const uint32_t len = static_cast<uint32_t>(seg_off[s + 1] - seg_off[s]), k = static_cast<uint32_t>(seg_k[s]);
        int code = -1;
        if (used > 0 && pt.len[last] == len && pt.k[last] == k) code = last;  // runs of equal tensors are common
        for (int d = 0; code < 0 && d < used; ++d)
            if (pt.len[d] == len && pt.k[d] == k) code = d;
        if (code < 0) {
            if (used == kDictMax) return false;
            code = used++;
            pt.len[code] = len;
            pt.k[code] = k;
        }
        pt.code[s] = static_cast<uint8_t>(code);
        last = code;
    }
    int64_t out0 = 0, group0 = 0;
    for (int32_t b = 0; b < kDictSegs / LD_WAVE; ++b) {
        const int32_t s0 = b * LD_WAVE < n_seg ? b * LD_WAVE : n_seg;
        pt.off0[b] = static_cast<uint32_t>(seg_off[s0]);
        pt.out0[b] = static_cast<uint32_t>(out0);
        pt.group0[b] = static_cast<uint32_t>(group0);
        for (int32_t s = s0; s < n_seg && s < s0 + LD_WAVE; ++s) {
            out0 += seg_k[s];
            group0 += groups_of(seg_off[s], seg_off[s + 1]);
        }
    }
    for (int d = used; d < kDictMax; ++d) pt.len[d] = pt.k[d] = 0;
    for (int32_t s = n_seg; s < kDictSegs; ++s) pt.code[s] = 0;
    pt.n_seg = n_seg;
    return true;
}

// Workgroups of k_full that the current device keeps resident at once, halved to leave room for
// whatever else runs (looked up once per device: a property of the device and of the kernel, not
// state of a call). 0 on failure.
int32_t full_grid_limit() {
    constexpr int kMaxDevices = 64;
    static std::atomic<int32_t> limit[kMaxDevices];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
    int32_t v = limit[dev].load(std::memory_order_acquire);
    if (v == 0) {
        int cus = 0, per_cu = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_full, kThreads, 0) != hipSuccess) return 0;
        if (cus <= 0 || per_cu <= 0) return 0;
        const int64_t all = static_cast<int64_t>(cus) * per_cu / 2;
        v = static_cast<int32_t>(all < 1 ? 1 : (all > kFullGrid ? kFullGrid : all));
        limit[dev].store(v, std::memory_order_release);
    }
    return v;
}

}  // namespace

extern "C" size_t ld_compress_topk_workspace(int32_t n_seg, const int64_t* seg_off) {
    const int64_t n_group = count_groups(n_seg, seg_off);
    if (n_group < 0) return 0;
    return layout(n_seg, n_group, kSlotMin).total;
}

extern "C" size_t ld_compress_topk_workspace_for(int32_t n_seg, const int64_t* seg_off, const int32_t* seg_k) {
    const int64_t n_group = count_groups(n_seg, seg_off);
    if (n_group < 0 || (n_seg > 0 && !seg_k)) return 0;
    return layout(n_seg, n_group, wanted_slot(n_seg, seg_off, seg_k)).total;
}

extern "C" ld_status ld_compress_topk_strategy(const float* grad, float* residual, const int64_t* seg_off,
                                               const int32_t* seg_k, int32_t n_seg, int32_t* out_idx,
                                               float* out_val, void* workspace, size_t workspace_bytes,
                                               ld_stream stream, int32_t strategy) {
    if (n_seg < 0 || (strategy != LD_COMPRESS_AUTO && strategy != LD_COMPRESS_FULL)) return LD_ERR_RANGE;
    if (n_seg == 0) return LD_OK;
    if (!seg_off || !seg_k) return LD_ERR_NULL;
    const int64_t n_group = count_groups(n_seg, seg_off);
    if (n_group < 0 || n_group > INT32_MAX / kTilesPerGroup) return LD_ERR_RANGE;
    const int64_t n = seg_off[n_seg];
    if (n > INT32_MAX) return LD_ERR_RANGE;
    int64_t K = 0;
    for (int32_t s = 0; s < n_seg; ++s) {
        if (seg_k[s] < 0 || seg_k[s] > seg_off[s + 1] - seg_off[s]) return LD_ERR_RANGE;
        K += seg_k[s];
    }
    if (n == 0) return LD_OK;
    if (!grad || !residual) return LD_ERR_NULL;
    if (K > 0 && (!out_idx || !out_val)) return LD_ERR_NULL;
    if (!ld_aligned(grad, 16) || !ld_aligned(residual, 16) || !ld_aligned(out_idx, 4) ||
        !ld_aligned(out_val, 4))
        return LD_ERR_ALIGN;
    if (!workspace || !ld_aligned(workspace, 256) || workspace_bytes < layout(n_seg, n_group, kSlotMin).total)
        return LD_ERR_WORKSPACE;
    // the largest slot, up to the one this call's densities ask for, that the workspace holds
    int32_t per_tile = 0;
    int32_t slot = wanted_slot(n_seg, seg_off, seg_k, &per_tile);
    while (slot > kSlotMin && layout(n_seg, n_group, slot).total > workspace_bytes) slot -= 64;
    const Layout L = layout(n_seg, n_group, slot);

    hipStream_t st = static_cast<hipStream_t>(stream);
    const Ctx c = make_ctx(workspace, L, n_seg, n_group, slot);

    ld_begin_call();
    // The segment table travels as kernel arguments: packed into k_prep's own when it has few
    // distinct (length, k) pairs, else through k_upload launches of kSegPerLaunch segments each.
    PackedTable pt;
    if (!pack_table(n_seg, seg_off, seg_k, pt)) {
        int64_t out0 = 0;
        int32_t group0 = 0;
        for (int32_t s0 = 0; s0 < n_seg; s0 += kSegPerLaunch) {
            UploadBatch ub;
            const int32_t cnt = (n_seg - s0) < kSegPerLaunch ? (n_seg - s0) : kSegPerLaunch;
            ub.out0 = out0;
            ub.group0 = group0;
            ub.first = s0;
            ub.count = cnt;
            ub.n_seg = n_seg;
            for (int32_t j = 0; j <= kSegPerLaunch; ++j) {
                const int32_t q = (s0 + j <= n_seg) ? (s0 + j) : n_seg;
                ub.off[j] = static_cast<int32_t>(seg_off[q]);
                if (j < kSegPerLaunch) ub.k[j] = (s0 + j < n_seg) ? seg_k[s0 + j] : 0;
            }
            for (int32_t j = 0; j < cnt; ++j) {
                out0 += seg_k[s0 + j];
                group0 += groups_of(seg_off[s0 + j], seg_off[s0 + j + 1]);
            }
            k_upload<<<dim3(1), dim3(512), 0, st>>>(ub, c);
            if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
        }
    }
    const dim3 block(kThreads);
    const dim3 sgrid(static_cast<uint32_t>(n_seg));
    k_prep<<<sgrid, dim3(kPrepThreads), 0, st>>>(grad, residual, c, strategy == LD_COMPRESS_FULL ? 1 : 0, pt);
    if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    if (n_group == 0) return LD_OK;
    const dim3 grid(static_cast<uint32_t>(n_group));
    const dim3 mgrid(static_cast<uint32_t>(n_group * kTilesPerGroup)), mblock(kMainWaves * LD_WAVE);
    if (slot == kSlotMin) k_main<true><<<mgrid, mblock, 0, st>>>(grad, residual, c);
    else k_main<false><<<mgrid, mblock, 0, st>>>(grad, residual, c);
    if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    if (K == 0) return LD_OK;
    const dim3 hgrid(static_cast<uint32_t>((n_group + kHistGroups - 1) / kHistGroups)), hblock(kHistGroups * kThreads);
    // lanes per tile in the candidate passes: enough for the candidates a tile is expected to hold
    const int row = (per_tile <= 128 && slot == kSlotMin) ? 16 : (per_tile <= 256 ? 32 : 64);  // 16 implies the minimum slot
    if (row == 16) k_hist<16><<<hgrid, hblock, 0, st>>>(residual, c);
    else if (row == 32) k_hist<32><<<hgrid, hblock, 0, st>>>(residual, c);
    else k_hist<64><<<hgrid, hblock, 0, st>>>(residual, c);
    if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    k_bin<<<sgrid, block, 0, st>>>(c);
    if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    if (row == 16) k_gather<16><<<grid, block, 0, st>>>(residual, c);
    else if (row == 32) k_gather<32><<<grid, block, 0, st>>>(residual, c);
    else k_gather<64><<<grid, block, 0, st>>>(residual, c);
    if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    k_select<<<sgrid, block, 0, st>>>(c);
    if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    if (row == 16) k_emit<16><<<grid, block, 0, st>>>(residual, out_idx, out_val, c);
    else if (row == 32) k_emit<32><<<grid, block, 0, st>>>(residual, out_idx, out_val, c);
    else k_emit<64><<<grid, block, 0, st>>>(residual, out_idx, out_val, c);
    if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    // segments handed to the full path (normally none: the launch returns at once). Its grid must be
    // resident as a whole (the phases hand over through a barrier across it).
    const int32_t resident = full_grid_limit();
    if (resident <= 0) return LD_ERR_HIP;
    const dim3 fgrid(static_cast<uint32_t>(n_group < resident ? n_group : resident));
    k_full<<<fgrid, block, 0, st>>>(residual, out_idx, out_val, c);
    return ld_launch_status();
}

extern "C" ld_status ld_compress_topk_paths(const void* workspace, size_t workspace_bytes, int32_t n_seg,
                                            const int64_t* seg_off, int32_t* paths, int32_t* overflowed_tiles,
                                            ld_stream stream) {
    if (n_seg < 0) return LD_ERR_RANGE;
    if (n_seg == 0) return LD_OK;
    if (!seg_off || !paths) return LD_ERR_NULL;
    const int64_t n_group = count_groups(n_seg, seg_off);
    if (n_group < 0 || n_group > INT32_MAX / kTilesPerGroup) return LD_ERR_RANGE;
    if (!ld_aligned(paths, 4) || !ld_aligned(overflowed_tiles, 4)) return LD_ERR_ALIGN;
    const Layout L = layout(n_seg, n_group, kSlotMin);  // the slot size only moves the candidate arrays
    if (!workspace || !ld_aligned(workspace, 256) || workspace_bytes < L.total) return LD_ERR_WORKSPACE;
    const Ctx c = make_ctx(const_cast<void*>(workspace), L, n_seg, n_group, kSlotMin);
    ld_begin_call();
    k_paths<<<dim3(static_cast<uint32_t>(n_seg)), dim3(kThreads), 0, static_cast<hipStream_t>(stream)>>>(
        c, paths, overflowed_tiles);
    return ld_launch_status();
}

extern "C" ld_status ld_compress_topk(const float* grad, float* residual, const int64_t* seg_off,
                                      const int32_t* seg_k, int32_t n_seg, int32_t* out_idx,
                                      float* out_val, void* workspace, size_t workspace_bytes,
                                      ld_stream stream) {
    return ld_compress_topk_strategy(grad, residual, seg_off, seg_k, n_seg, out_idx, out_val, workspace,
                                     workspace_bytes, stream, LD_COMPRESS_AUTO);
}
