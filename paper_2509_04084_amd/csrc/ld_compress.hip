// ld_compress_topk: per-segment exact top-k sparsification with error feedback.
//
// Comp of Algorithm 1 (Sec. IV-B) at ratio rho (Sec. II-C, Sec. VII-A): the
// compressed gradient that is reused as the differential checkpoint.  The
// selection rule (|r+g| descending on the bit pattern, ties to the lower index,
// records ascending, selected residuals zeroed) is stated in lowdiff.h.
//
// Design: ONE streaming pass over the gradient and the residual.
//
//   k_prep   one workgroup per segment: writes the segment descriptor, clears its
//            state, and estimates a candidate threshold tau from a strided sample
//            of |r+g| (exact for segments that fit in the sample): tau is the
//            sample's key at a rank chosen high enough that, with overwhelming
//            probability, at least k elements of the segment lie at or above it.
//   k_main   a = r + g -> residual (12 bytes per element, the only full pass).
//            Each wave owns a contiguous 16K-element range and appends, in index
//            order, every element with key >= tau to its own candidate slot; the
//            first digit of the candidates' keys is histogrammed in LDS.
//   k_level  two more radix-select levels over the candidates only
//   k_count  per wave range: #candidates above / equal to the exact threshold;
//            the last workgroup of a segment scans them into output offsets
//   k_emit   ordered emission of (idx, val) from the candidates; residual[idx] <- +0
//
// The estimate can never make the result wrong, only slower:
//   * a wave whose slot fills up stops collecting; the rest of its range (the
//     "suffix") is re-read from the residual by the later kernels;
//   * a segment that ends up with fewer than k candidates is handed to the
//     k_full_* kernels, a plain three-level radix select over the whole segment.
// Per-segment digit histograms live in global memory and are resolved by the
// workgroup that finishes a segment's phase last (ticket counter + release /
// acquire at device scope), so no phase needs an extra launch.
#include <math.h>

#include <vector>

#include "ld_common.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / LD_WAVE;
constexpr int kRows = 4;                          // float4 rows per lane per wave tile
constexpr int kWaveTile = LD_WAVE * 4 * kRows;    // 1024 elements
constexpr int kWChunk = 16384;                    // elements owned by one wave
constexpr int kChunk = kWaves * kWChunk;          // 65536 elements per workgroup
constexpr int kCapW = 1024;                       // candidate slots per wave range (6.25 %)
constexpr int kBins = 2048;
constexpr int kShift1 = 20, kShift2 = 9;          // digit positions: [30:20] [19:9] [8:0]
constexpr int kPrepThreads = 1024;
constexpr int kSampleItems = 8;
constexpr int kSample = kPrepThreads * kSampleItems;  // 8192 sampled elements per segment
constexpr int kSampleRuns = kSample / LD_WAVE;        // as 128 runs of 64 consecutive elements
constexpr float kSampleZ = 6.5f;                  // safety margin of the rank estimate, in sigmas
constexpr int kSegPerLaunch = 448;
constexpr int kFullGrid = 1024;                   // workgroups of the (normally idle) k_full_* kernels
constexpr uint32_t kModeCand = 0, kModeFull = 1;

struct SegDesc {        // one per segment plus a sentinel
    int64_t off;        // first element
    int64_t out0;       // first output record
    int32_t k;          // records to keep
    int32_t chunk0;     // first chunk
};

struct SegState {       // 64 bytes
    uint32_t tau;       // candidate threshold (key); 0: every element, 0xFFFFFFFF: none
    uint32_t prefix;    // key bits fixed so far; after level 3 the exact threshold T
    uint32_t krem;      // rank still to resolve; after level 3 the number of ties to keep
    uint32_t ncand;     // elements with key >= tau
    uint32_t mode;      // kModeCand | kModeFull
    uint32_t done[4];   // tickets: main, level 2, level 3, count
    uint32_t fdone[4];  // tickets of the full-segment path: level 1, 2, 3, count
    uint32_t pad[3];
};

struct Ctx {
    SegDesc* desc;          // [n_seg + 1]
    SegState* state;        // [n_seg]
    uint32_t* hist;         // [n_seg][kBins]
    int32_t* chunk_seg;     // [n_chunk]
    int32_t* cand_idx;      // [n_chunk * kWaves][kCapW]
    float* cand_val;        // same shape
    uint32_t* wc_cnt;       // [n_chunk * kWaves] stored candidates
    int32_t* wc_ovf;        // [n_chunk * kWaves] first element of the un-collected suffix (range end if none)
    uint32_t* wc_gt;        // [n_chunk * kWaves] #above threshold -> records emitted before this range
    uint32_t* wc_eq;        // [n_chunk * kWaves] #equal -> ties before this range
    uint32_t* ch_gt;        // [n_chunk] the same two per chunk, full-segment path
    uint32_t* ch_eq;
    int32_t* fail_chunks;   // [n_chunk] chunks of segments in kModeFull
    uint32_t* fail_count;   // [1]
    int32_t n_seg;
    int32_t n_chunk;
};

struct PrepBatch {
    int32_t off[kSegPerLaunch + 1];
    int32_t k[kSegPerLaunch];
    int64_t out0;     // records before the first segment of the batch
    int32_t chunk0;   // chunks before it
    int32_t first;    // index of the batch's first segment
    int32_t count;
    int32_t n_seg;
    int32_t no_estimate;  // LD_COMPRESS_FULL: collect no candidates, select over whole segments
};

__host__ __device__ inline int64_t align_down4(int64_t x) { return x & ~static_cast<int64_t>(3); }

__host__ __device__ inline int32_t chunks_of(int64_t off, int64_t end) {
    if (end <= off) return 0;
    return static_cast<int32_t>((end - align_down4(off) + kChunk - 1) / kChunk);
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
// of `expected`. Everything the other workgroups published before their ticket
// (atomics, or plain stores read back with ld_load_coherent) is visible to it.
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

// Finds the digit d with #(digit > d) < krem <= #(digit >= d) in the global
// histogram `h`, folds it into the segment's prefix and clears `h`.
template <int NT>
__device__ void resolve_level(uint32_t* h, SegState* st, int shift, uint32_t krem_in, uint32_t prefix_in,
                              uint32_t* sh) {
    constexpr int per = kBins / NT;
    const int top = kBins - 1 - threadIdx.x * per;  // this thread's highest digit
    uint32_t v[per], sum = 0;
#pragma unroll
    for (int i = 0; i < per; ++i) {
        v[i] = ld_load_coherent(h + top - i);
        sum += v[i];
    }
    uint32_t total;
    uint32_t above = block_escan<NT>(sum, sh, total);
#pragma unroll
    for (int i = 0; i < per; ++i) {
        if (above < krem_in && krem_in <= above + v[i]) {
            st->prefix = prefix_in | (static_cast<uint32_t>(top - i) << shift);
            st->krem = krem_in - above;
        }
        above += v[i];
    }
#pragma unroll
    for (int i = 0; i < per; ++i) h[top - i] = 0;
}

__device__ __forceinline__ void flush_hist(uint32_t* h, const uint32_t* lh) {
    for (int b = threadIdx.x; b < kBins; b += blockDim.x) {
        const uint32_t x = lh[b];
        if (x) atomicAdd(h + b, x);
    }
}

__device__ __forceinline__ uint32_t mbcnt(uint64_t mask) {  // set bits of `mask` below this lane
    return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
}

__device__ __forceinline__ uint32_t umin(uint32_t a, uint32_t b) { return a < b ? a : b; }

// ------------------------------------------------------------------ geometry

struct ChunkRange {
    int32_t seg;
    int64_t cs, ce;      // element range of this chunk
    int64_t t0;          // start of the chunk's first tile (multiple of 4; may precede cs)
    int32_t k;
    int32_t nchunk;      // chunks in the segment
    int32_t chunk0;
    int64_t out0;
};

__device__ __forceinline__ ChunkRange chunk_range(const Ctx& c, int32_t chunk) {
    ChunkRange r;
    r.seg = c.chunk_seg[chunk];
    const SegDesc d = c.desc[r.seg];
    const SegDesc dn = c.desc[r.seg + 1];
    const int64_t base = align_down4(d.off);
    r.t0 = base + static_cast<int64_t>(chunk - d.chunk0) * kChunk;
    r.cs = r.t0 < d.off ? d.off : r.t0;
    r.ce = (r.t0 + kChunk) > dn.off ? dn.off : (r.t0 + kChunk);
    r.k = d.k;
    r.chunk0 = d.chunk0;
    r.nchunk = dn.chunk0 - d.chunk0;
    r.out0 = d.out0;
    return r;
}

// The range of wave `w` inside a chunk: [ws, we), tiles start at wt0.
__device__ __forceinline__ void wave_range(const ChunkRange& cr, int w, int64_t& wt0, int64_t& ws, int64_t& we) {
    wt0 = cr.t0 + static_cast<int64_t>(w) * kWChunk;
    ws = wt0 < cr.cs ? cr.cs : wt0;
    we = (wt0 + kWChunk) > cr.ce ? cr.ce : (wt0 + kWChunk);
    if (we < ws) we = ws;
}

// Loads the 4 elements at e0..e0+3 that lie inside [lo, hi); returns the mask of
// valid components. e0 is a multiple of 4 and `p` is 16-byte aligned.
template <bool NT>
__device__ __forceinline__ uint32_t load4(const float* __restrict__ p, int64_t e0, int64_t lo, int64_t hi,
                                          float (&x)[4]) {
    if (e0 >= lo && e0 + 4 <= hi) {
        ld_f32x4 q;
        if (NT) q = ld_nt_load(reinterpret_cast<const ld_f32x4*>(p + e0));
        else q = *reinterpret_cast<const ld_f32x4*>(p + e0);
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

template <bool NT>
__device__ __forceinline__ void store4(float* __restrict__ p, int64_t e0, uint32_t mask, const float (&x)[4]) {
    if (mask == 0xF) {
        const ld_f32x4 q = {x[0], x[1], x[2], x[3]};
        if (NT) ld_nt_store(q, reinterpret_cast<ld_f32x4*>(p + e0));
        else *reinterpret_cast<ld_f32x4*>(p + e0) = q;
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

// Key at rank `rank` (1 = largest) among the valid keys held in registers by
// the 1024 threads of the workgroup.
__device__ uint32_t block_select(const uint32_t (&key)[kSampleItems], uint32_t valid_mask, uint32_t rank,
                                 uint32_t* lh, uint32_t* sh, uint32_t* res) {
    uint32_t prefix = 0, krem = rank;
#pragma unroll 1
    for (int level = 0; level < 3; ++level) {
        const int match_shift = (level == 0) ? 31 : (level == 1 ? kShift1 : kShift2);
        const int digit_shift = (level == 0) ? kShift1 : (level == 1 ? kShift2 : 0);
        const uint32_t digit_mask = (level == 2) ? 0x1FFu : 0x7FFu;
        for (int b = threadIdx.x; b < kBins; b += kPrepThreads) lh[b] = 0;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kSampleItems; ++i)
            if (((valid_mask >> i) & 1u) && (key[i] >> match_shift) == (prefix >> match_shift))
                atomicAdd(&lh[(key[i] >> digit_shift) & digit_mask], 1u);
        __syncthreads();
        constexpr int per = kBins / kPrepThreads;  // 2
        const int top = kBins - 1 - threadIdx.x * per;
        uint32_t v[per], sum = 0;
#pragma unroll
        for (int i = 0; i < per; ++i) { v[i] = lh[top - i]; sum += v[i]; }
        uint32_t total;
        uint32_t above = block_escan<kPrepThreads>(sum, sh, total);
#pragma unroll
        for (int i = 0; i < per; ++i) {
            if (above < krem && krem <= above + v[i]) {
                res[0] = prefix | (static_cast<uint32_t>(top - i) << digit_shift);
                res[1] = krem - above;
            }
            above += v[i];
        }
        __syncthreads();
        prefix = res[0];
        krem = res[1];
        __syncthreads();
    }
    return prefix;
}

__global__ __launch_bounds__(kPrepThreads) void k_prep(const float* __restrict__ g,
                                                       const float* __restrict__ r, PrepBatch pb, Ctx c) {
    __shared__ uint32_t lh[kBins];
    __shared__ uint32_t sh[kPrepThreads / LD_WAVE];
    __shared__ uint32_t res[2];
    __shared__ long long sums[2];
    const int j = blockIdx.x;
    const int s = pb.first + j;
    // descriptor: prefix sums over the batch entries before this one
    if (threadIdx.x == 0) { sums[0] = 0; sums[1] = 0; }
    __syncthreads();
    long long my_chunks = 0, my_k = 0;
    for (int i = threadIdx.x; i < j; i += kPrepThreads) {
        my_chunks += chunks_of(pb.off[i], pb.off[i + 1]);
        my_k += pb.k[i];
    }
    if (my_chunks) atomicAdd(reinterpret_cast<unsigned long long*>(&sums[0]), static_cast<unsigned long long>(my_chunks));
    if (my_k) atomicAdd(reinterpret_cast<unsigned long long*>(&sums[1]), static_cast<unsigned long long>(my_k));
    __syncthreads();
    const int64_t off = pb.off[j], end = pb.off[j + 1];
    const int32_t k = pb.k[j];
    const int32_t chunk0 = pb.chunk0 + static_cast<int32_t>(sums[0]);
    const int64_t out0 = pb.out0 + sums[1];
    const int32_t nchunk = chunks_of(off, end);
    if (threadIdx.x == 0) {
        c.desc[s] = SegDesc{off, out0, k, chunk0};
        if (s == pb.n_seg - 1) c.desc[s + 1] = SegDesc{end, out0 + k, 0, chunk0 + nchunk};
        if (s == 0) *c.fail_count = 0;
    }
    if (threadIdx.x < sizeof(SegState) / 4) reinterpret_cast<uint32_t*>(&c.state[s])[threadIdx.x] = 0;
    for (int b = threadIdx.x; b < kBins; b += kPrepThreads) c.hist[static_cast<int64_t>(s) * kBins + b] = 0;
    for (int32_t q = threadIdx.x; q < nchunk; q += kPrepThreads) c.chunk_seg[chunk0 + q] = s;

    // candidate threshold from a sample of |r + g|
    const int64_t ns = end - off;
    uint32_t tau;
    if (k == 0 || pb.no_estimate) {
        tau = 0xFFFFFFFFu;
    } else {
        uint32_t key[kSampleItems];
        uint32_t valid = 0;
        const bool whole = ns <= kSample;
        const int lane = threadIdx.x & 63;
        const int64_t stride = ns / kSampleRuns;
#pragma unroll
        for (int i = 0; i < kSampleItems; ++i) {
            int64_t e;
            if (whole) {
                e = off + i * kPrepThreads + threadIdx.x;
            } else {
                const int run = i * (kPrepThreads / LD_WAVE) + (threadIdx.x >> 6);
                const int64_t jitter = hash32(static_cast<uint32_t>(run) * 2654435761u + static_cast<uint32_t>(s)) %
                                       static_cast<uint32_t>(stride - LD_WAVE + 1);
                e = off + run * stride + jitter + lane;
            }
            key[i] = 0;
            if (e < end) {
                key[i] = ld_key(__fadd_rn(r[e], g[e]));
                valid |= 1u << i;
            }
        }
        uint32_t rank;
        if (whole) {
            rank = static_cast<uint32_t>(k);  // the sample is the segment: tau is the exact threshold
        } else {
            // expected sample hits a = k * kSample / ns; take the rank x with x = a + z*sqrt(x)
            const float a = static_cast<float>(k) * (static_cast<float>(kSample) / static_cast<float>(ns));
            const float sq = 0.5f * (kSampleZ + sqrtf(kSampleZ * kSampleZ + 4.0f * a));
            rank = static_cast<uint32_t>(sq * sq) + 2u;
        }
        const uint32_t navail = whole ? static_cast<uint32_t>(ns) : static_cast<uint32_t>(kSample);
        if (rank >= navail && !whole) tau = 0;  // k too large for an estimate: everything is a candidate
        else tau = block_select(key, valid, rank, lh, sh, res);
    }
    if (threadIdx.x == 0) c.state[s].tau = tau;
}

// -------------------------------------------------------------------- k_main

__global__ __launch_bounds__(kThreads) void k_main(const float* __restrict__ g, float* __restrict__ r, Ctx c) {
    __shared__ uint32_t lh[kBins];
    __shared__ uint32_t sh[kWaves];
    __shared__ uint32_t ncand_blk;
    const ChunkRange cr = chunk_range(c, blockIdx.x);
    SegState* st = c.state + cr.seg;
    const uint32_t tau = st->tau;
    for (int b = threadIdx.x; b < kBins; b += kThreads) lh[b] = 0;
    if (threadIdx.x == 0) ncand_blk = 0;
    __syncthreads();

    const int lane = ld_lane();
    const int w = threadIdx.x >> 6;
    int64_t wt0, ws, we;
    wave_range(cr, w, wt0, ws, we);
    const int64_t wc = static_cast<int64_t>(blockIdx.x) * kWaves + w;
    int32_t* slot_idx = c.cand_idx + wc * kCapW;
    float* slot_val = c.cand_val + wc * kCapW;
    uint32_t cnt = 0;         // candidates stored (wave-uniform)
    uint32_t ncand = 0;       // per-lane count of keys >= tau
    int64_t ovf = we;         // start of the suffix that was not collected
    bool collecting = true;

    for (int64_t t = wt0; t < we; t += kWaveTile) {
        float a[kRows][4];
        uint32_t mask[kRows], flag[kRows];
        uint32_t any = 0;
        if (t >= ws && t + kWaveTile <= we) {  // interior tile: unconditional 16-byte streaming accesses
            const ld_f32x4* g4 = reinterpret_cast<const ld_f32x4*>(g + t) + lane;
            ld_f32x4* r4 = reinterpret_cast<ld_f32x4*>(r + t) + lane;
            ld_f32x4 gq[kRows], rq[kRows];
#pragma unroll
            for (int j = 0; j < kRows; ++j) gq[j] = ld_nt_load(g4 + j * LD_WAVE);
#pragma unroll
            for (int j = 0; j < kRows; ++j) rq[j] = ld_nt_load(r4 + j * LD_WAVE);
#pragma unroll
            for (int j = 0; j < kRows; ++j) {
                a[j][0] = __fadd_rn(rq[j].x, gq[j].x);
                a[j][1] = __fadd_rn(rq[j].y, gq[j].y);
                a[j][2] = __fadd_rn(rq[j].z, gq[j].z);
                a[j][3] = __fadd_rn(rq[j].w, gq[j].w);
                ld_nt_store(ld_f32x4{a[j][0], a[j][1], a[j][2], a[j][3]}, r4 + j * LD_WAVE);
                mask[j] = 0xF;
            }
        } else {
#pragma unroll
            for (int j = 0; j < kRows; ++j) {
                const int64_t e0 = t + (j * LD_WAVE + lane) * 4;
                float gv[4], rv[4];
                mask[j] = load4<false>(g, e0, ws, we, gv);
                load4<false>(r, e0, ws, we, rv);
#pragma unroll
                for (int q = 0; q < 4; ++q) a[j][q] = __fadd_rn(rv[q], gv[q]);
                store4<false>(r, e0, mask[j], a[j]);
            }
        }
#pragma unroll
        for (int j = 0; j < kRows; ++j) {
            flag[j] = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                flag[j] |= static_cast<uint32_t>(ld_key(a[j][q]) >= tau) << q;
            flag[j] &= mask[j];
            any |= flag[j];
            ncand += __popc(flag[j]);
        }
        if (collecting) {
            if (__ballot(any != 0) == 0) continue;
            // ordered positions: element order in the tile is (row, lane, component)
            uint32_t below[kRows];   // candidates of lower lanes in the same row
            uint32_t rowbase[kRows]; // candidates of earlier rows
            uint32_t total = 0;
#pragma unroll
            for (int j = 0; j < kRows; ++j) {
                rowbase[j] = total;
                below[j] = 0;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint64_t m = __ballot((flag[j] >> q) & 1u);
                    below[j] += mbcnt(m);
                    total += __popcll(m);
                }
            }
            if (cnt + total <= kCapW) {
#pragma unroll
                for (int j = 0; j < kRows; ++j) {
                    if (flag[j] == 0) continue;
                    const int64_t e0 = t + (j * LD_WAVE + lane) * 4;
                    uint32_t pos = cnt + rowbase[j] + below[j];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if ((flag[j] >> q) & 1u) {
                            slot_idx[pos] = static_cast<int32_t>(e0 + q);
                            slot_val[pos] = a[j][q];
                            atomicAdd(&lh[ld_key(a[j][q]) >> kShift1], 1u);
                            ++pos;
                        }
                    }
                }
                cnt += total;
                continue;
            }
            collecting = false;  // slot full: this tile and the rest of the range form the suffix
            ovf = t < ws ? ws : t;
        }
        // suffix: every element takes part in the selection, read back from the residual later
#pragma unroll
        for (int j = 0; j < kRows; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if ((mask[j] >> q) & 1u) atomicAdd(&lh[ld_key(a[j][q]) >> kShift1], 1u);
    }
    ncand = ld_wave_sum(ncand);
    if (lane == 0) {
        c.wc_cnt[wc] = cnt;
        c.wc_ovf[wc] = static_cast<int32_t>(ovf);
        if (ncand) atomicAdd(&ncand_blk, ncand);
    }
    __syncthreads();
    flush_hist(c.hist + static_cast<int64_t>(cr.seg) * kBins, lh);
    if (threadIdx.x == 0 && ncand_blk) atomicAdd(&st->ncand, ncand_blk);
    if (!last_block(&st->done[0], static_cast<uint32_t>(cr.nchunk))) return;
    uint32_t* h = c.hist + static_cast<int64_t>(cr.seg) * kBins;
    const uint32_t total_cand = ld_load_coherent(&st->ncand);
    if (cr.k == 0) {
        if (threadIdx.x == 0) { st->prefix = 0xFFFFFFFFu; st->krem = 0; }
        for (int b = threadIdx.x; b < kBins; b += kThreads) h[b] = 0;
    } else if (total_cand >= static_cast<uint32_t>(cr.k)) {
        resolve_level<kThreads>(h, st, kShift1, static_cast<uint32_t>(cr.k), 0u, sh);
    } else {
        // the estimate was too high: hand the whole segment to the k_full_* kernels
        __shared__ uint32_t list0;
        if (threadIdx.x == 0) {
            st->mode = kModeFull;
            list0 = atomicAdd(c.fail_count, static_cast<uint32_t>(cr.nchunk));
        }
        for (int b = threadIdx.x; b < kBins; b += kThreads) h[b] = 0;
        __syncthreads();
        for (int32_t q = threadIdx.x; q < cr.nchunk; q += kThreads) c.fail_chunks[list0 + q] = cr.chunk0 + q;
    }
}

// ------------------------------------------------- candidate-based selection

// Visits every element that takes part in the selection of one wave range:
// first the stored candidates, then the un-collected suffix (from the residual).
// f(key) is called once per element, in no particular order.
template <class F>
__device__ __forceinline__ void for_each_key(const Ctx& c, const float* __restrict__ r, int64_t wc,
                                             int64_t we, F&& f) {
    const int lane = ld_lane();
    const uint32_t cnt = c.wc_cnt[wc];
    const int64_t ovf = c.wc_ovf[wc];
    const float* val = c.cand_val + wc * kCapW;
    for (uint32_t i = lane; i < cnt; i += LD_WAVE) f(ld_key(val[i]));
    for (int64_t e = ovf + lane; e < we; e += LD_WAVE) f(ld_key(r[e]));
}

template <int LEVEL>
__global__ __launch_bounds__(kThreads) void k_level(const float* __restrict__ r, Ctx c) {
    __shared__ uint32_t lh[kBins];
    __shared__ uint32_t sh[kWaves];
    const ChunkRange cr = chunk_range(c, blockIdx.x);
    SegState* st = c.state + cr.seg;
    if (cr.k == 0 || st->mode != kModeCand) return;
    const uint32_t prefix = st->prefix, krem = st->krem;
    constexpr int match_shift = (LEVEL == 2) ? kShift1 : kShift2;
    constexpr int digit_shift = (LEVEL == 2) ? kShift2 : 0;
    constexpr uint32_t digit_mask = (LEVEL == 2) ? 0x7FFu : 0x1FFu;
    for (int b = threadIdx.x; b < kBins; b += kThreads) lh[b] = 0;
    __syncthreads();
    const int w = threadIdx.x >> 6;
    int64_t wt0, ws, we;
    wave_range(cr, w, wt0, ws, we);
    for_each_key(c, r, static_cast<int64_t>(blockIdx.x) * kWaves + w, we, [&](uint32_t key) {
        if ((key >> match_shift) == (prefix >> match_shift))
            atomicAdd(&lh[(key >> digit_shift) & digit_mask], 1u);
    });
    __syncthreads();
    uint32_t* h = c.hist + static_cast<int64_t>(cr.seg) * kBins;
    flush_hist(h, lh);
    if (last_block(&st->done[LEVEL - 1], static_cast<uint32_t>(cr.nchunk)))
        resolve_level<kThreads>(h, st, digit_shift, krem, prefix, sh);
}

__global__ __launch_bounds__(kThreads) void k_count(const float* __restrict__ r, Ctx c) {
    __shared__ uint32_t sh[kWaves];
    const ChunkRange cr = chunk_range(c, blockIdx.x);
    SegState* st = c.state + cr.seg;
    if (cr.k == 0 || st->mode != kModeCand) return;
    const uint32_t T = st->prefix, m = st->krem;
    const int w = threadIdx.x >> 6;
    const int64_t wc = static_cast<int64_t>(blockIdx.x) * kWaves + w;
    int64_t wt0, ws, we;
    wave_range(cr, w, wt0, ws, we);
    uint32_t gt = 0, eq = 0;
    for_each_key(c, r, wc, we, [&](uint32_t key) {
        gt += (key > T);
        eq += (key == T);
    });
    gt = ld_wave_sum(gt);
    eq = ld_wave_sum(eq);
    if (ld_lane() == 0) {
        c.wc_gt[wc] = gt;
        c.wc_eq[wc] = eq;
    }
    if (!last_block(&st->done[3], static_cast<uint32_t>(cr.nchunk))) return;
    // exclusive scan over the segment's wave ranges: records emitted / ties seen before each
    const int64_t wc0 = static_cast<int64_t>(cr.chunk0) * kWaves;
    const int32_t nwc = cr.nchunk * kWaves;
    uint32_t carry_out = 0, carry_eq = 0;
    for (int32_t q0 = 0; q0 < nwc; q0 += kThreads) {
        const int32_t q = q0 + threadIdx.x;
        uint32_t cg = 0, ce = 0;
        if (q < nwc) {
            cg = ld_load_coherent(c.wc_gt + wc0 + q);
            ce = ld_load_coherent(c.wc_eq + wc0 + q);
        }
        uint32_t te, tg;
        const uint32_t eq_before = carry_eq + block_escan<kThreads>(ce, sh, te);
        const uint32_t take = umin(eq_before + ce, m) - umin(eq_before, m);  // ties kept: lowest index first
        const uint32_t out_before = carry_out + block_escan<kThreads>(cg + take, sh, tg);
        if (q < nwc) {
            c.wc_gt[wc0 + q] = out_before;
            c.wc_eq[wc0 + q] = eq_before;
        }
        carry_eq += te;
        carry_out += tg;
    }
}

__global__ __launch_bounds__(kThreads) void k_emit(float* __restrict__ r, int32_t* __restrict__ out_idx,
                                                   float* __restrict__ out_val, Ctx c) {
    const ChunkRange cr = chunk_range(c, blockIdx.x);
    const SegState* st = c.state + cr.seg;
    if (cr.k == 0 || st->mode != kModeCand) return;
    const uint32_t T = st->prefix, m = st->krem;
    const int lane = ld_lane();
    const int w = threadIdx.x >> 6;
    const int64_t wc = static_cast<int64_t>(blockIdx.x) * kWaves + w;
    int64_t wt0, ws, we;
    wave_range(cr, w, wt0, ws, we);
    uint32_t run_out = c.wc_gt[wc];  // records of the segment emitted before this point
    uint32_t run_eq = c.wc_eq[wc];   // ties seen before this point
    const uint32_t cnt = c.wc_cnt[wc];
    const int64_t ovf = c.wc_ovf[wc];
    const int32_t* cidx = c.cand_idx + wc * kCapW;
    const float* cval = c.cand_val + wc * kCapW;
    // one batch of up to 64 elements, in index order across the lanes
    auto emit = [&](bool have, int32_t idx, float val) {
        const uint32_t key = ld_key(val);
        const bool is_gt = have && key > T;
        const bool is_eq = have && key == T;
        const uint64_t mg = __ballot(is_gt), me = __ballot(is_eq);
        const uint32_t eq_rank = run_eq + mbcnt(me);
        if (is_gt || (is_eq && eq_rank < m)) {
            const int64_t pos = cr.out0 + run_out + mbcnt(mg) + (umin(eq_rank, m) - umin(run_eq, m));
            out_idx[pos] = idx;
            out_val[pos] = val;
            r[idx] = 0.0f;
        }
        const uint32_t eq_end = run_eq + __popcll(me);
        run_out += __popcll(mg) + (umin(eq_end, m) - umin(run_eq, m));
        run_eq = eq_end;
    };
    for (uint32_t i0 = 0; i0 < cnt; i0 += LD_WAVE) {
        const bool have = i0 + lane < cnt;
        emit(have, have ? cidx[i0 + lane] : 0, have ? cval[i0 + lane] : 0.0f);
    }
    for (int64_t e0 = ovf; e0 < we; e0 += LD_WAVE) {
        const bool have = e0 + lane < we;
        emit(have, static_cast<int32_t>(e0 + lane), have ? r[e0 + lane] : 0.0f);
    }
}

// ------------------------------------------ full-segment path (kModeFull only)
// Plain three-level radix select over every element of the listed chunks.

template <int LEVEL>
__global__ __launch_bounds__(kThreads) void k_full_level(const float* __restrict__ r, Ctx c) {
    __shared__ uint32_t lh[kBins];
    __shared__ uint32_t sh[kWaves];
    const uint32_t nlist = *c.fail_count;
    constexpr int match_shift = (LEVEL == 1) ? 31 : (LEVEL == 2 ? kShift1 : kShift2);
    constexpr int digit_shift = (LEVEL == 1) ? kShift1 : (LEVEL == 2 ? kShift2 : 0);
    constexpr uint32_t digit_mask = (LEVEL == 3) ? 0x1FFu : 0x7FFu;
    for (uint32_t li = blockIdx.x; li < nlist; li += gridDim.x) {
        const ChunkRange cr = chunk_range(c, c.fail_chunks[li]);
        SegState* st = c.state + cr.seg;
        const uint32_t prefix = (LEVEL == 1) ? 0u : st->prefix;
        const uint32_t krem = (LEVEL == 1) ? static_cast<uint32_t>(cr.k) : st->krem;
        for (int b = threadIdx.x; b < kBins; b += kThreads) lh[b] = 0;
        __syncthreads();
        for (int64_t t = cr.t0; t < cr.ce; t += kThreads * 4) {
            const int64_t e0 = t + threadIdx.x * 4;
            float x[4];
            const uint32_t mask = load4<false>(r, e0, cr.cs, cr.ce, x);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t key = ld_key(x[q]);
                if (((mask >> q) & 1u) && (key >> match_shift) == (prefix >> match_shift))
                    atomicAdd(&lh[(key >> digit_shift) & digit_mask], 1u);
            }
        }
        __syncthreads();
        uint32_t* h = c.hist + static_cast<int64_t>(cr.seg) * kBins;
        flush_hist(h, lh);
        if (last_block(&st->fdone[LEVEL - 1], static_cast<uint32_t>(cr.nchunk)))
            resolve_level<kThreads>(h, st, digit_shift, krem, prefix, sh);
        __syncthreads();
    }
}

__global__ __launch_bounds__(kThreads) void k_full_count(const float* __restrict__ r, Ctx c) {
    __shared__ uint32_t sh[kWaves];
    const uint32_t nlist = *c.fail_count;
    for (uint32_t li = blockIdx.x; li < nlist; li += gridDim.x) {
        const int32_t chunk = c.fail_chunks[li];
        const ChunkRange cr = chunk_range(c, chunk);
        SegState* st = c.state + cr.seg;
        const uint32_t T = st->prefix, m = st->krem;
        uint32_t gt = 0, eq = 0;
        for (int64_t t = cr.t0; t < cr.ce; t += kThreads * 4) {
            float x[4];
            const uint32_t mask = load4<false>(r, t + threadIdx.x * 4, cr.cs, cr.ce, x);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t key = ld_key(x[q]);
                if ((mask >> q) & 1u) { gt += (key > T); eq += (key == T); }
            }
        }
        uint32_t tot_gt, tot_eq;
        block_escan<kThreads>(gt, sh, tot_gt);
        block_escan<kThreads>(eq, sh, tot_eq);
        if (threadIdx.x == 0) { c.ch_gt[chunk] = tot_gt; c.ch_eq[chunk] = tot_eq; }
        if (last_block(&st->fdone[3], static_cast<uint32_t>(cr.nchunk))) {
            uint32_t carry_out = 0, carry_eq = 0;
            for (int32_t q0 = 0; q0 < cr.nchunk; q0 += kThreads) {
                const int32_t q = q0 + threadIdx.x;
                uint32_t cg = 0, ce = 0;
                if (q < cr.nchunk) {
                    cg = ld_load_coherent(c.ch_gt + cr.chunk0 + q);
                    ce = ld_load_coherent(c.ch_eq + cr.chunk0 + q);
                }
                uint32_t te, tg;
                const uint32_t eq_before = carry_eq + block_escan<kThreads>(ce, sh, te);
                const uint32_t take = umin(eq_before + ce, m) - umin(eq_before, m);
                const uint32_t out_before = carry_out + block_escan<kThreads>(cg + take, sh, tg);
                if (q < cr.nchunk) {
                    c.ch_gt[cr.chunk0 + q] = out_before;
                    c.ch_eq[cr.chunk0 + q] = eq_before;
                }
                carry_eq += te;
                carry_out += tg;
            }
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(kThreads) void k_full_emit(float* __restrict__ r, int32_t* __restrict__ out_idx,
                                                        float* __restrict__ out_val, Ctx c) {
    __shared__ uint32_t part[2][kWaves];  // packed (above | ties << 16) per wave
    const uint32_t nlist = *c.fail_count;
    const int lane = ld_lane();
    const int wv = threadIdx.x >> 6;
    for (uint32_t li = blockIdx.x; li < nlist; li += gridDim.x) {
        const int32_t chunk = c.fail_chunks[li];
        const ChunkRange cr = chunk_range(c, chunk);
        const SegState* st = c.state + cr.seg;
        const uint32_t T = st->prefix, m = st->krem;
        uint32_t run_out = c.ch_gt[chunk], run_eq = c.ch_eq[chunk];
        int buf = 0;
        // element order inside a tile of 1024: (thread, component)
        for (int64_t t = cr.t0; t < cr.ce; t += kThreads * 4, buf ^= 1) {
            const int64_t e0 = t + threadIdx.x * 4;
            float x[4];
            const uint32_t mask = load4<false>(r, e0, cr.cs, cr.ce, x);
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
                    const int64_t pos = cr.out0 + run_out + gt_before + (umin(eq_rank, m) - umin(run_eq, m));
                    out_idx[pos] = static_cast<int32_t>(e0 + q);
                    out_val[pos] = x[q];
                    x[q] = 0.0f;
                    touched = true;
                }
                gt_before += is_gt;
                eq_rank += is_eq;
            }
            if (touched) store4<false>(r, e0, mask, x);
            const uint32_t eq_end = run_eq + tot_eq;
            run_out += tot_gt + (umin(eq_end, m) - umin(run_eq, m));
            run_eq = eq_end;
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------- host side

struct Layout {
    size_t desc, state, hist, chunk_seg, cand_idx, cand_val, wc_cnt, wc_ovf, wc_gt, wc_eq, ch_gt, ch_eq,
        fail_chunks, fail_count, total;
};

Layout layout(int32_t n_seg, int64_t n_chunk) {
    Layout L;
    size_t o = 0;
    const size_t ns = static_cast<size_t>(n_seg), nc = static_cast<size_t>(n_chunk), nw = nc * kWaves;
    auto take = [&](size_t bytes) { const size_t at = o; o += ld_round_up(bytes, 256); return at; };
    L.desc = take(sizeof(SegDesc) * (ns + 1));
    L.state = take(sizeof(SegState) * ns);
    L.hist = take(sizeof(uint32_t) * kBins * ns);
    L.chunk_seg = take(4 * nc);
    L.cand_idx = take(4 * nw * kCapW);
    L.cand_val = take(4 * nw * kCapW);
    L.wc_cnt = take(4 * nw);
    L.wc_ovf = take(4 * nw);
    L.wc_gt = take(4 * nw);
    L.wc_eq = take(4 * nw);
    L.ch_gt = take(4 * nc);
    L.ch_eq = take(4 * nc);
    L.fail_chunks = take(4 * nc);
    L.fail_count = take(4);
    L.total = o;
    return L;
}

// Counts chunks; returns -1 on a malformed offset table.
int64_t count_chunks(int32_t n_seg, const int64_t* seg_off) {
    if (n_seg < 0 || (n_seg > 0 && !seg_off)) return -1;
    if (n_seg > 0 && seg_off[0] != 0) return -1;
    int64_t total = 0;
    for (int32_t s = 0; s < n_seg; ++s) {
        if (seg_off[s + 1] < seg_off[s]) return -1;
        total += chunks_of(seg_off[s], seg_off[s + 1]);
    }
    return total;
}

}  // namespace

extern "C" size_t ld_compress_topk_workspace(int32_t n_seg, const int64_t* seg_off) {
    const int64_t n_chunk = count_chunks(n_seg, seg_off);
    if (n_chunk < 0) return 0;
    return layout(n_seg, n_chunk).total;
}

extern "C" ld_status ld_compress_topk_strategy(const float* grad, float* residual, const int64_t* seg_off,
                                               const int32_t* seg_k, int32_t n_seg, int32_t* out_idx,
                                               float* out_val, void* workspace, size_t workspace_bytes,
                                               ld_stream stream, int32_t strategy) {
    if (n_seg < 0 || (strategy != LD_COMPRESS_AUTO && strategy != LD_COMPRESS_FULL)) return LD_ERR_RANGE;
    if (n_seg == 0) return LD_OK;
    if (!seg_off || !seg_k) return LD_ERR_NULL;
    const int64_t n_chunk = count_chunks(n_seg, seg_off);
    if (n_chunk < 0 || n_chunk > INT32_MAX / kWaves) return LD_ERR_RANGE;
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
    const Layout L = layout(n_seg, n_chunk);
    if (!workspace || !ld_aligned(workspace, 256) || workspace_bytes < L.total) return LD_ERR_WORKSPACE;

    hipStream_t st = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    Ctx c;
    c.desc = reinterpret_cast<SegDesc*>(ws + L.desc);
    c.state = reinterpret_cast<SegState*>(ws + L.state);
    c.hist = reinterpret_cast<uint32_t*>(ws + L.hist);
    c.chunk_seg = reinterpret_cast<int32_t*>(ws + L.chunk_seg);
    c.cand_idx = reinterpret_cast<int32_t*>(ws + L.cand_idx);
    c.cand_val = reinterpret_cast<float*>(ws + L.cand_val);
    c.wc_cnt = reinterpret_cast<uint32_t*>(ws + L.wc_cnt);
    c.wc_ovf = reinterpret_cast<int32_t*>(ws + L.wc_ovf);
    c.wc_gt = reinterpret_cast<uint32_t*>(ws + L.wc_gt);
    c.wc_eq = reinterpret_cast<uint32_t*>(ws + L.wc_eq);
    c.ch_gt = reinterpret_cast<uint32_t*>(ws + L.ch_gt);
    c.ch_eq = reinterpret_cast<uint32_t*>(ws + L.ch_eq);
    c.fail_chunks = reinterpret_cast<int32_t*>(ws + L.fail_chunks);
    c.fail_count = reinterpret_cast<uint32_t*>(ws + L.fail_count);
    c.n_seg = n_seg;
    c.n_chunk = static_cast<int32_t>(n_chunk);

    // segment table travels as kernel arguments, kSegPerLaunch segments per launch
    {
        int64_t out0 = 0;
        int32_t chunk0 = 0;
        for (int32_t s0 = 0; s0 < n_seg; s0 += kSegPerLaunch) {
            PrepBatch pb;
            const int32_t cnt = (n_seg - s0) < kSegPerLaunch ? (n_seg - s0) : kSegPerLaunch;
            pb.out0 = out0;
            pb.chunk0 = chunk0;
            pb.first = s0;
            pb.count = cnt;
            pb.n_seg = n_seg;
            pb.no_estimate = (strategy == LD_COMPRESS_FULL);
            for (int32_t j = 0; j <= kSegPerLaunch; ++j) {
                const int32_t q = (s0 + j <= n_seg) ? (s0 + j) : n_seg;
                pb.off[j] = static_cast<int32_t>(seg_off[q]);
                if (j < kSegPerLaunch) pb.k[j] = (s0 + j < n_seg) ? seg_k[s0 + j] : 0;
            }
            for (int32_t j = 0; j < cnt; ++j) {
                out0 += seg_k[s0 + j];
                chunk0 += chunks_of(seg_off[s0 + j], seg_off[s0 + j + 1]);
            }
            k_prep<<<dim3(cnt), dim3(kPrepThreads), 0, st>>>(grad, residual, pb, c);
            if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
        }
    }
    if (n_chunk == 0) return LD_OK;
    const dim3 grid(static_cast<uint32_t>(n_chunk)), block(kThreads);
    k_main<<<grid, block, 0, st>>>(grad, residual, c);
    if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    if (K == 0) return LD_OK;
    k_level<2><<<grid, block, 0, st>>>(residual, c);
    k_level<3><<<grid, block, 0, st>>>(residual, c);
    k_count<<<grid, block, 0, st>>>(residual, c);
    k_emit<<<grid, block, 0, st>>>(residual, out_idx, out_val, c);
    if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    // segments whose candidate estimate failed (normally none: these exit at once)
    const dim3 fgrid(static_cast<uint32_t>(n_chunk < kFullGrid ? n_chunk : kFullGrid));
    k_full_level<1><<<fgrid, block, 0, st>>>(residual, c);
    k_full_level<2><<<fgrid, block, 0, st>>>(residual, c);
    k_full_level<3><<<fgrid, block, 0, st>>>(residual, c);
    k_full_count<<<fgrid, block, 0, st>>>(residual, c);
    k_full_emit<<<fgrid, block, 0, st>>>(residual, out_idx, out_val, c);
    return ld_launch_status();
}

extern "C" ld_status ld_compress_topk(const float* grad, float* residual, const int64_t* seg_off,
                                      const int32_t* seg_k, int32_t n_seg, int32_t* out_idx,
                                      float* out_val, void* workspace, size_t workspace_bytes,
                                      ld_stream stream) {
    return ld_compress_topk_strategy(grad, residual, seg_off, seg_k, n_seg, out_idx, out_val, workspace,
                                     workspace_bytes, stream, LD_COMPRESS_AUTO);
}
