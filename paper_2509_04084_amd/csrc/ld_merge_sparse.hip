// ld_merge_sparse: ordered replay of a window of sparse diffs onto w.
//
// Recovery loop of Algorithm 1 (Sec. IV-B) and Eq. (6): M_{j+1} = M_j + merge(diff j)
// for j in iteration order, with the diffs of a batch kept apart and replayed one
// after another (Sec. IV-C, "Batched write semantics").  Update rule per record:
// p = fl32(lr*val); w[idx] = fl32(w[idx] - p).
//
// Two strategies with identical results:
//  * sweep   - one streaming pass over w.  A wave owns an 8192-element sub-tile
//              held in LDS, pulls the records of every diff that fall into it and
//              applies them diff after diff.  LDS operations of one wave execute
//              in issue order, so the cross-diff order on an element needs no
//              barrier.  Where a diff's records for the sub-tile start is not
//              looked up in a table: a small kernel finds the record range of
//              every chunk of 6 sub-tiles by binary search, the wave
//              interpolates inside its chunk, loads a 128-record window a little
//              before the guess and keeps the records that fall into its
//              sub-tile.  The guess is checked (the window must begin before the
//              sub-tile does, and end after it); a miss costs a binary search
//              inside the chunk or one more window, never a wrong result.
//              HBM traffic: 8n + 8*sum(K) bytes + the chunk table.
//  * scatter - one kernel per diff, one thread per record; for windows that
//              touch only a small part of w.
#include <atomic>

#include "ld_sparse_common.h"

namespace {

constexpr int kSub = 8192;                 // elements per wave sub-tile (32 KB of LDS, 5 waves per CU)
constexpr int kChunkSubs = 6;              // sub-tiles per chunk of the range table
static_assert(static_cast<int64_t>(kSub) * kChunkSubs == kChunk, "sub-tiles must tile a chunk");
constexpr int kMargin = 24;                // records the window starts before the interpolated position
constexpr int kSweepGroup = kTableMax;     // diffs per sweep: a lane keeps the chunk ranges of two of them
// Windows loaded ahead, as <diffs per batch, 64-record windows per diff>: 10 x 2 for the usual
// densities (~80 records per diff and sub-tile at 1 %), 20 x 1 for long windows of very sparse
// diffs (a handful of records each: half as many rounds of loads, each a memory round trip).

__device__ __forceinline__ void apply_record(float* tile, int32_t local, float val, float lr) {
    const float p = __fmul_rn(lr, val);        // rounded product: never fused
    tile[local] = __fsub_rn(tile[local], p);
}

// N records per lane of ONE diff (so no two of the wave's 64 N records name the same element):
// those inside [lo, hi) are all read before any is written - one round trip to LDS instead of N.
template <int N>
__device__ __forceinline__ void apply_records(float* tile, const int32_t (&i)[N], const float (&v)[N], int32_t lo,
                                              int32_t hi, float lr) {
    float cur[N];
#pragma unroll
    for (int u = 0; u < N; ++u) cur[u] = (i[u] >= lo && i[u] < hi) ? tile[i[u] - lo] : 0.0f;
#pragma unroll
    for (int u = 0; u < N; ++u)
        if (i[u] >= lo && i[u] < hi) tile[i[u] - lo] = __fsub_rn(cur[u], __fmul_rn(lr, v[u]));   // rounded product: never fused
}

// Applies the records of one diff at positions [p, end) that fall into [lo, hi), up to the
// first record at or beyond hi. kDeep loads of 64 records are in flight together: a dense
// diff has many such batches per sub-tile, and one at a time would leave the wave waiting
// for memory once per batch.
constexpr int kDeep = 8;

__device__ __forceinline__ void apply_from(float* tile, const int32_t* __restrict__ idx,
                                           const float* __restrict__ val, int32_t p, int32_t end,
                                           int32_t lo, int32_t hi, float lr, int lane) {
    for (; p < end; p += kDeep * LD_WAVE) {
        int32_t i[kDeep];
        float v[kDeep];
#pragma unroll
        for (int u = 0; u < kDeep; ++u) {
            const int32_t q = p + u * LD_WAVE + lane;
            const bool have = q < end;
            i[u] = have ? idx[q] : INT_MAX;
            v[u] = have ? val[q] : 0.0f;
        }
        apply_records(tile, i, v, lo, hi, lr);
        if (__ballot(i[kDeep - 1] >= hi)) break;
    }
}

// Chunk range [c0, c1) and guessed start of diff t (lanes 0..63) and, in sweeps of more than 64
// diffs (SETS = 2), of diff t + 64.
template <int SETS>
struct Ranges {
    int32_t c0[SETS], c1[SETS], start[SETS];
};

template <int SETS>
__device__ __forceinline__ int32_t of_diff(const int32_t (&x)[SETS], int t) {
    if (SETS == 1) return __builtin_amdgcn_readlane(x[0], t);
    return t < LD_WAVE ? __builtin_amdgcn_readlane(x[0], t) : __builtin_amdgcn_readlane(x[SETS - 1], t - LD_WAVE);
}

// The first WIN * 64 records of PRE consecutive diffs at and after the guessed positions.
template <int PRE, int WIN>
struct Batch {
    int32_t s[PRE], e[PRE], b[PRE];   // window start, end of the chunk's records, their begin (wave-uniform)
    int32_t ri[PRE][WIN];
    float rv[PRE][WIN];
};

template <int PRE, int WIN, int SETS>
__device__ __forceinline__ void load_batch(Batch<PRE, WIN>& X, const DiffTable& tb, int32_t W, int32_t t0,
                                           const Ranges<SETS>& R, int lane) {
#pragma unroll
    for (int g = 0; g < PRE; ++g) {
        const int t = (t0 + g < W) ? t0 + g : 0;
        X.s[g] = of_diff(R.start, t);
        X.b[g] = of_diff(R.c0, t);
        X.e[g] = (t0 + g < W) ? of_diff(R.c1, t) : X.s[g];  // past W: an empty window
        const int32_t* __restrict__ ip = tb.idx[t];
        const float* __restrict__ vp = tb.val[t];
#pragma unroll
        for (int u = 0; u < WIN; ++u) {
            const int32_t p = X.s[g] + u * LD_WAVE + lane;
            const bool h = p < X.e[g];
            X.ri[g][u] = h ? ip[p] : INT_MAX;
            X.rv[g][u] = h ? vp[p] : 0.0f;
        }
    }
}

template <int PRE, int WIN, int SETS>
__global__ __launch_bounds__(LD_WAVE) void k_merge_sweep(float* __restrict__ w, int64_t n, int32_t nchunk,
                                                         DiffTable tb, int32_t W,
                                                         const int32_t* __restrict__ ctab, float lr) {
    __shared__ float tile[kSub];
    const int lane = threadIdx.x;
    // consecutive workgroups go to different XCDs (each with an L2 of its own): give every XCD one
    // contiguous eighth of w, so that the overlapping record windows of neighbouring sub-tiles hit its L2
    const int64_t per = (static_cast<int64_t>(gridDim.x) + 7) / 8;
    const int64_t sub = static_cast<int64_t>(blockIdx.x % 8) * per + blockIdx.x / 8;
    if (sub * kSub >= n) return;
    const int64_t lo64 = sub * kSub;
    const int32_t len = static_cast<int32_t>((n - lo64) < kSub ? (n - lo64) : kSub);
    const int32_t lo = static_cast<int32_t>(lo64), hi = lo + len;  // n <= INT_MAX
    const bool full = (len == kSub);

    ld_f32x4 x[kSub / 4 / LD_WAVE];
    if (full) {
        const ld_f32x4* src = reinterpret_cast<const ld_f32x4*>(w + lo64);
#pragma unroll
        for (int j = 0; j < kSub / 4 / LD_WAVE; ++j) x[j] = ld_nt_load(src + j * LD_WAVE + lane);
    }

    // lane t: where the records of diffs t and t + 64 lie in this chunk, and the guesses for this sub-tile
    const int32_t chunk = static_cast<int32_t>(sub / kChunkSubs), part = static_cast<int32_t>(sub % kChunkSubs);
    Ranges<SETS> R;
#pragma unroll
    for (int h = 0; h < SETS; ++h) {
        const int t = h * LD_WAVE + lane;
        R.c0[h] = R.c1[h] = 0;
        if (t < W) {
            const int32_t* row = ctab + static_cast<int64_t>(t) * (nchunk + 1) + chunk;
            R.c0[h] = row[0];
            R.c1[h] = row[1];
        }
        R.start[h] = R.c0[h] + ((R.c1[h] - R.c0[h]) * part) / kChunkSubs - kMargin;
        if (R.start[h] < R.c0[h]) R.start[h] = R.c0[h];
    }

    // The windows of the first PRE diffs are requested before the tile goes to LDS. (Requesting
    // every next batch while the current one is applied made the sweep 10 % slower.)
    Batch<PRE, WIN> A;
    load_batch(A, tb, W, 0, R, lane);

    if (full) {
#pragma unroll
        for (int j = 0; j < kSub / 4 / LD_WAVE; ++j) reinterpret_cast<ld_f32x4*>(tile)[j * LD_WAVE + lane] = x[j];
    } else {
        for (int32_t e = lane; e < len; e += LD_WAVE) tile[e] = w[lo64 + e];
    }
    __syncthreads();  // one wave: only orders the vector fill before the scalar updates

    for (int32_t t0 = 0; t0 < W; t0 += PRE) {
        if (t0 > 0) load_batch(A, tb, W, t0, R, lane);
#pragma unroll
        for (int g = 0; g < PRE; ++g) {
            if (A.s[g] < A.e[g]) {
                const int t = t0 + g;
                const int32_t first = __builtin_amdgcn_readfirstlane(A.ri[g][0]);
                if (A.s[g] == A.b[g] || first <= lo) {
                    // the window begins before the sub-tile's records do; ascending indices: a record
                    // at or beyond hi (or the padding past the chunk's end) in the last window says
                    // that nothing of this sub-tile follows
                    apply_records(tile, A.ri[g], A.rv[g], lo, hi, lr);
                    const bool more = !__ballot(A.ri[g][WIN - 1] >= hi);
                    if (more) apply_from(tile, tb.idx[t], tb.val[t], A.s[g] + WIN * LD_WAVE, A.e[g], lo, hi, lr, lane);
                } else {
                    // guess too late: find the first record of the sub-tile inside the chunk
                    const int32_t p = lower_bound_idx(tb.idx[t], A.b[g], A.s[g], lo);
                    apply_from(tile, tb.idx[t], tb.val[t], p, A.e[g], lo, hi, lr, lane);
                }
            }
            __builtin_amdgcn_wave_barrier();  // keep diff g's LDS traffic ahead of diff g+1's
        }
    }

    __syncthreads();
    if (full) {
        ld_f32x4* dst = reinterpret_cast<ld_f32x4*>(w + lo64);
#pragma unroll
        for (int j = 0; j < kSub / 4 / LD_WAVE; ++j)
            ld_nt_store(reinterpret_cast<const ld_f32x4*>(tile)[j * LD_WAVE + lane], dst + j * LD_WAVE + lane);
    } else {
        for (int32_t e = lane; e < len; e += LD_WAVE) w[lo64 + e] = tile[e];
    }
}

// ------------------------------------------------------- thin long windows: a lane per diff
//
// A long window of very sparse diffs (config 3: 100 diffs of 0.1 %, eight records per diff and
// sub-tile) leaves the sweep above with a wave's 64 lanes serving eight records at a time, a
// hundred times in a row. Here the roles are turned round: lane t holds ALL the records of diff t
// (and t + 64) that fall into the wave's sub-tile and the diffs are applied side by side. Where
// exactly a diff's records for a sub-tile begin comes from a table of its own (k_subtab: one
// streaming pass over the index arrays, which are small when diffs are this sparse).
//
// Order: an element that only one diff of the window touches can be updated at any time. Elements
// touched by several diffs are found first (two bitmaps in LDS: seen, seen again) and their
// records are held back; these are then applied in rounds: every pending record bids for its
// element's slot of a small owner table with (diff, element) as the key, the smallest key wins the
// slot (atomic minimum), applies its update and leaves; so the updates of one element go through
// in diff order whatever else shares the slot.
#ifndef LD_THIN_SUB
#define LD_THIN_SUB 4096
#endif
#ifndef LD_THIN_CAP
#define LD_THIN_CAP 24
#endif
#ifndef LD_THIN_OWNER
#define LD_THIN_OWNER 128
#endif
constexpr int kThinSub = LD_THIN_SUB;    // elements of a wave's sub-tile in this kernel
constexpr int kThinCap = LD_THIN_CAP;    // records of one diff in one sub-tile that a lane can hold
constexpr int kThinSlots = (kThinCap + 3 + 3) / 4 * 4;  // register slots: the records come in aligned blocks of four
constexpr int kConfLane = 4;             // held-back records a lane can keep
constexpr int kBitWords = kThinSub / 32;
constexpr int kOwner = LD_THIN_OWNER;    // slots of the owner table
static_assert(kThinSub % (4 * LD_WAVE) == 0 && kThinSub % 32 == 0 && kThinSub <= 8192, "whole rows of 16-byte accesses; 13 bits of element in a key");

// tab[t * (nsub + 1) + s] = number of records of diff t with idx < s * kThinSub, s = 0 .. nsub.
// A thread looks at four consecutive records (one 16-byte load; the arrays of this path are
// 16-byte aligned) and at the one before them, and fills the entries between the sub-tiles of
// neighbouring records; the thread that meets record K closes the row.
constexpr int kSubtabPer = 4;

__global__ __launch_bounds__(256) void k_subtab(DiffTable tb, int32_t nsub, int32_t* __restrict__ tab) {
    const int t = blockIdx.y;
    const int32_t K = tb.K[t];
    const int32_t* __restrict__ idx = tb.idx[t];
    const int32_t j0 = (static_cast<int32_t>(blockIdx.x) * 256 + static_cast<int32_t>(threadIdx.x)) * kSubtabPer;
    if (j0 > K) return;
    // the block of four that holds record j0 lies inside the array's last 16 bytes at worst
    ld_u32x4 q = {0u, 0u, 0u, 0u};
    if (j0 < K) q = *reinterpret_cast<const ld_u32x4*>(idx + j0);
    const int32_t v[kSubtabPer] = {static_cast<int32_t>(q.x), static_cast<int32_t>(q.y), static_cast<int32_t>(q.z),
                                   static_cast<int32_t>(q.w)};
    int32_t a = j0 == 0 ? -1 : idx[j0 - 1] / kThinSub;
    int32_t* row = tab + static_cast<int64_t>(t) * (nsub + 1);
#pragma unroll
    for (int c = 0; c < kSubtabPer; ++c) {
        const int32_t j = j0 + c;
        if (j > K) break;
        int32_t b = j == K ? nsub : v[c] / kThinSub;
        if (a >= nsub) a = nsub - 1;   // an index outside [0, n) breaks the caller's contract: stay inside the row
        if (a < -1) a = -1;
        if (b > nsub) b = nsub;
        for (int32_t s = a + 1; s <= b; ++s) row[s] = j;
        a = b;
    }
}

__device__ __forceinline__ int32_t wave_max(int32_t x) {
#pragma unroll
    for (int d = LD_WAVE / 2; d > 0; d >>= 1) {
        const int32_t y = __shfl_xor(x, d, LD_WAVE);
        x = y > x ? y : x;
    }
    return x;
}

template <int SETS>
__global__ __launch_bounds__(LD_WAVE) void k_merge_thin(float* __restrict__ w, int64_t n, int32_t nsub,
                                                        DiffTable tb, int32_t W, const int32_t* __restrict__ tab,
                                                        float lr) {
    __shared__ float tile[kThinSub];
    __shared__ uint32_t seen[kBitWords], multi[kBitWords];
    __shared__ uint32_t owner[kOwner];
    const int lane = threadIdx.x;
    const int64_t per = (static_cast<int64_t>(gridDim.x) + 7) / 8;   // each XCD walks one contiguous eighth of w
    const int64_t sub = static_cast<int64_t>(blockIdx.x % 8) * per + blockIdx.x / 8;
    if (sub * kThinSub >= n) return;
    const int64_t lo64 = sub * kThinSub;
    const int32_t len = static_cast<int32_t>((n - lo64) < kThinSub ? (n - lo64) : kThinSub);
    const int32_t lo = static_cast<int32_t>(lo64);
    const bool full = (len == kThinSub);

    ld_f32x4 x[kThinSub / 4 / LD_WAVE];
    if (full) {
        const ld_f32x4* src = reinterpret_cast<const ld_f32x4*>(w + lo64);
#pragma unroll
        for (int j = 0; j < kThinSub / 4 / LD_WAVE; ++j) x[j] = ld_nt_load(src + j * LD_WAVE + lane);
    }
    // lane t: the records of diffs t (and t + 64) inside this sub-tile
    int32_t p0[SETS], cnt[SETS];
    const int32_t* ip[SETS];
    const float* vp[SETS];
    int32_t most = 0, slots = 0;
#pragma unroll
    for (int h = 0; h < SETS; ++h) {
        const int t = h * LD_WAVE + lane;
        p0[h] = cnt[h] = 0;
        ip[h] = nullptr;
        vp[h] = nullptr;
        if (t < W) {
            const int32_t* row = tab + static_cast<int64_t>(t) * (nsub + 1) + sub;
            p0[h] = row[0];
            cnt[h] = row[1] - p0[h];
            ip[h] = tb.idx[t];
            vp[h] = tb.val[t];
        }
        most = cnt[h] > most ? cnt[h] : most;
        const int32_t used = (p0[h] & 3) + cnt[h];   // slots of 16-byte blocks the lane's records reach into
        slots = used > slots ? used : slots;
    }
    most = wave_max(most);
    slots = wave_max(slots);
    if (full) {
#pragma unroll
        for (int j = 0; j < kThinSub / 4 / LD_WAVE; ++j) reinterpret_cast<ld_f32x4*>(tile)[j * LD_WAVE + lane] = x[j];
    } else {
        for (int32_t e = lane; e < len; e += LD_WAVE) tile[e] = w[lo64 + e];
    }
    for (int q = lane; q < kOwner; q += LD_WAVE) owner[q] = 0xFFFFFFFFu;
    __syncthreads();  // one wave: orders the fills before what follows

    if (most > kThinCap) {
        // some diff has more records here than a lane holds: diff after diff, the lanes sharing
        // the records of one diff (no two of them touch the same element)
        for (int t = 0; t < W; ++t) {
            const int h = t / LD_WAVE, l = t % LD_WAVE;
            const int32_t b = __shfl(SETS == 1 ? p0[0] : (h == 0 ? p0[0] : p0[SETS - 1]), l, LD_WAVE);
            const int32_t c = __shfl(SETS == 1 ? cnt[0] : (h == 0 ? cnt[0] : cnt[SETS - 1]), l, LD_WAVE);
            const int32_t* __restrict__ di = tb.idx[t];
            const float* __restrict__ dv = tb.val[t];
            for (int32_t q = lane; q < c; q += LD_WAVE) {
                const int32_t e = di[b + q] - lo;
                if (static_cast<uint32_t>(e) < static_cast<uint32_t>(len)) apply_record(tile, e, dv[b + q], lr);
            }
            __builtin_amdgcn_wave_barrier();
        }
    } else {
        // The lane's records, fetched as whole 16-byte blocks of four (the index and value arrays
        // of this path are 16-byte aligned): slot j holds record (p0 & ~3) + j; slots before p0 or
        // past the lane's count are marked empty (a negative index). (Single 4-byte loads, one
        // record per lane and instruction, pulled a cache line per lane and record from L2.) Both
        // sets of diffs are requested before the first is worked on.
        int32_t ri_[SETS][kThinSlots];
        float rp_[SETS][kThinSlots];
#pragma unroll
        for (int h = 0; h < SETS; ++h) {
            const int32_t k0 = p0[h] & ~3, sh = p0[h] - k0;
#pragma unroll
            for (int v = 0; v < kThinSlots / 4; ++v) {
                ld_u32x4 qi = {0u, 0u, 0u, 0u};
                ld_f32x4 qv = {0.0f, 0.0f, 0.0f, 0.0f};
                if (4 * v < slots) {  // wave-uniform
                    if (4 * v < sh + cnt[h]) {
                        qi = *reinterpret_cast<const ld_u32x4*>(ip[h] + k0 + 4 * v);
                        qv = *reinterpret_cast<const ld_f32x4*>(vp[h] + k0 + 4 * v);
                    }
                }
                const uint32_t ei[4] = {qi.x, qi.y, qi.z, qi.w};
                const float ev[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int j = 4 * v + c;
                    const int32_t e = static_cast<int32_t>(ei[c]) - lo;
                    const bool have = j >= sh && j < sh + cnt[h] && static_cast<uint32_t>(e) < static_cast<uint32_t>(len);
                    ri_[h][j] = have ? e : -1;  // ascending, in-range indices never fail the last test
                    rp_[h][j] = ev[c];
                }
            }
        }
#pragma unroll
        for (int h = 0; h < SETS; ++h) {
            const uint32_t t = static_cast<uint32_t>(h * LD_WAVE + lane);
            const int32_t (&ri)[kThinSlots] = ri_[h];
            const float (&rp)[kThinSlots] = rp_[h];
            for (int q = lane; q < kBitWords; q += LD_WAVE) {
                seen[q] = 0;
                multi[q] = 0;
            }
            __builtin_amdgcn_wave_barrier();
            // which elements do several diffs of this set touch?
            uint32_t again = 0;
#pragma unroll
            for (int i = 0; i < kThinSlots; ++i) {
                if (i < slots && ri[i] >= 0) {
                    const uint32_t bit = 1u << (ri[i] & 31);
                    if (atomicOr(&seen[ri[i] >> 5], bit) & bit) again |= 1u << i;
                }
            }
#pragma unroll
            for (int i = 0; i < kThinSlots; ++i)
                if ((again >> i) & 1u) atomicOr(&multi[ri[i] >> 5], 1u << (ri[i] & 31));
            __builtin_amdgcn_wave_barrier();
            // elements of one diff only: updated now; the others are held back
            int32_t ce[kConfLane];
            float cp[kConfLane];
            int nc = 0;
#pragma unroll
            for (int q = 0; q < kConfLane; ++q) { ce[q] = 0; cp[q] = 0.0f; }
#pragma unroll
            for (int i = 0; i < kThinSlots; ++i) {
                if (i < slots && ri[i] >= 0) {
                    const float p = __fmul_rn(lr, rp[i]);   // rounded product: never fused
                    if ((multi[ri[i] >> 5] >> (ri[i] & 31)) & 1u) {
#pragma unroll
                        for (int q = 0; q < kConfLane; ++q)
                            if (nc == q) { ce[q] = ri[i]; cp[q] = p; }
                        ++nc;
                    } else {
                        tile[ri[i]] = __fsub_rn(tile[ri[i]], p);
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
            if (__ballot(nc > kConfLane)) {
                // more held back than a lane keeps (heavily overlapping diffs): the lanes take turns in
                // diff order, each applying what it holds back
                uint64_t turn = __ballot(nc > 0);
                while (turn) {
                    const int l = __builtin_ctzll(turn);
                    turn &= turn - 1;
                    if (lane == l) {
#pragma unroll
                        for (int i = 0; i < kThinSlots; ++i) {
                            if (i < slots && ri[i] >= 0 && ((multi[ri[i] >> 5] >> (ri[i] & 31)) & 1u))
                                tile[ri[i]] = __fsub_rn(tile[ri[i]], __fmul_rn(lr, rp[i]));
                        }
                    }
                    __builtin_amdgcn_wave_barrier();
                }
            } else {
                uint32_t pend = (1u << nc) - 1u;
                while (__ballot(pend != 0)) {
#pragma unroll
                    for (int q = 0; q < kConfLane; ++q)
                        if ((pend >> q) & 1u) atomicMin(&owner[ce[q] & (kOwner - 1)], (t << 13) | static_cast<uint32_t>(ce[q]));
                    __builtin_amdgcn_wave_barrier();
                    uint32_t won = 0;
#pragma unroll
                    for (int q = 0; q < kConfLane; ++q) {
                        if (((pend >> q) & 1u) && owner[ce[q] & (kOwner - 1)] == ((t << 13) | static_cast<uint32_t>(ce[q]))) {
                            tile[ce[q]] = __fsub_rn(tile[ce[q]], cp[q]);
                            won |= 1u << q;
                        }
                    }
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int q = 0; q < kConfLane; ++q)
                        if ((won >> q) & 1u) owner[ce[q] & (kOwner - 1)] = 0xFFFFFFFFu;
                    __builtin_amdgcn_wave_barrier();
                    pend &= ~won;
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }

    __syncthreads();
    if (full) {
        ld_f32x4* dst = reinterpret_cast<ld_f32x4*>(w + lo64);
#pragma unroll
        for (int j = 0; j < kThinSub / 4 / LD_WAVE; ++j)
            ld_nt_store(reinterpret_cast<const ld_f32x4*>(tile)[j * LD_WAVE + lane], dst + j * LD_WAVE + lane);
    } else {
        for (int32_t e = lane; e < len; e += LD_WAVE) w[lo64 + e] = tile[e];
    }
}

__global__ __launch_bounds__(256) void k_merge_scatter(float* __restrict__ w,
                                                       const int32_t* __restrict__ idx,
                                                       const float* __restrict__ val, int32_t K,
                                                       float lr) {
    const int32_t j = blockIdx.x * 256 + threadIdx.x;
    if (j >= K) return;
    const int32_t i = idx[j];
    const float p = __fmul_rn(lr, val[j]);
    w[i] = __fsub_rn(w[i], p);
}

int32_t sub_tiles(int64_t n) { return static_cast<int32_t>((n + kSub - 1) / kSub); }

}  // namespace

namespace {

// A group of `gw` diffs whose largest holds `most` records is "thin" when a diff brings at most ~16
// records to a sub-tile and the group is long: it then runs a lane per diff (k_merge_thin).
bool thin_group(int64_t n, int32_t gw, int64_t most) { return gw > 10 && most * kSub <= 16 * n; }

size_t chunk_table_bytes(int64_t n, int32_t W) {
    const int64_t group = W < kSweepGroup ? W : kSweepGroup;
    return ld_round_up(static_cast<size_t>(group) * (static_cast<size_t>(chunks(n)) + 1) * 4, 256);
}

size_t sub_table_bytes(int64_t n, int32_t gw) {
    return ld_round_up(static_cast<size_t>(gw) * (static_cast<size_t>((n + kThinSub - 1) / kThinSub) + 1) * 4, 256);
}

}  // namespace

// The chunk table always; for thin groups (when K is given) the larger per-sub-tile table, without
// which they run as ordinary sweeps.
extern "C" size_t ld_merge_sparse_workspace(int64_t n, int32_t W, const int64_t* K) {
    if (n <= 0 || W <= 0) return 256;
    size_t need = chunk_table_bytes(n, W);
    if (K && n <= INT32_MAX && W <= LD_MAX_WINDOW) {
        for (int32_t g0 = 0; g0 < W; g0 += kSweepGroup) {
            const int32_t gw = (W - g0) < kSweepGroup ? (W - g0) : kSweepGroup;
            int64_t most = 0;
            for (int32_t t = g0; t < g0 + gw; ++t) most = K[t] > most ? K[t] : most;
            if (thin_group(n, gw, most) && sub_table_bytes(n, gw) > need) need = sub_table_bytes(n, gw);
        }
    }
    return need;
}

namespace {

ld_status merge_sparse_impl(float* w, int64_t n, const int32_t* const* idx, const float* const* val,
                            const int64_t* K, int32_t W, float lr, void* workspace, size_t workspace_bytes,
                            ld_stream stream, int32_t strategy) {
    const ld_status st = check_diff_args(w, n, idx, val, K, W);
    if (st != LD_OK) return st;
    if (strategy < LD_MERGE_AUTO || strategy > LD_MERGE_SCATTER) return LD_ERR_RANGE;
    if (W == 0 || n == 0) return LD_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    ld_begin_call();

    int64_t total = 0;
    for (int32_t t = 0; t < W; ++t) total += K[t];
    if (total == 0) return LD_OK;
    // measured on 1.56 G elements: a scattered record costs 46 ps, the sweep 1.35 ps per element of w
    // plus little per record: they meet where the window holds n / 34 records
    if (strategy == LD_MERGE_AUTO)
        strategy = (total * 32 >= n) ? LD_MERGE_SWEEP : LD_MERGE_SCATTER;

    if (strategy == LD_MERGE_SCATTER) {
        for (int32_t t = 0; t < W; ++t) {
            if (K[t] == 0) continue;
            const int32_t k = static_cast<int32_t>(K[t]);
            k_merge_scatter<<<dim3((k + 255) / 256), dim3(256), 0, s>>>(w, idx[t], val[t], k, lr);
            if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
        }
        return LD_OK;
    }

    if (!workspace || !ld_aligned(workspace, 256) || workspace_bytes < chunk_table_bytes(n, W))
        return LD_ERR_WORKSPACE;
    const int32_t nsub = sub_tiles(n), nchunk = chunks(n);
    int32_t* ctab = static_cast<int32_t*>(workspace);
    for (int32_t g0 = 0; g0 < W; g0 += kSweepGroup) {
        const int32_t gw = (W - g0) < kSweepGroup ? (W - g0) : kSweepGroup;
        DiffTable tb = {};
        int64_t most = 0;
        bool aligned16 = true;
        for (int32_t t = 0; t < kTableMax; ++t) {
            const bool live = t < gw;
            tb.idx[t] = live ? idx[g0 + t] : nullptr;
            tb.val[t] = live ? val[g0 + t] : nullptr;
            tb.K[t] = live ? static_cast<int32_t>(K[g0 + t]) : 0;
            if (live && K[g0 + t] > most) most = K[g0 + t];
            if (live && !(ld_aligned(idx[g0 + t], 16) && ld_aligned(val[g0 + t], 16))) aligned16 = false;
        }
        const dim3 grid((nsub + 7) / 8 * 8), wave(LD_WAVE);
        const bool thin = thin_group(n, gw, most);
        if (thin && aligned16 && workspace_bytes >= sub_table_bytes(n, gw)) {  // a lane per diff (else: the sweep below)
            const int32_t tsub = static_cast<int32_t>((n + kThinSub - 1) / kThinSub);
            const dim3 tgrid((tsub + 7) / 8 * 8);
            k_subtab<<<dim3(static_cast<uint32_t>(most / (256 * kSubtabPer) + 1), gw), dim3(256), 0, s>>>(tb, tsub, ctab);
            if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
            if (gw <= LD_WAVE) k_merge_thin<1><<<tgrid, wave, 0, s>>>(w, n, tsub, tb, gw, ctab, lr);
            else k_merge_thin<2><<<tgrid, wave, 0, s>>>(w, n, tsub, tb, gw, ctab, lr);
            if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
            continue;
        }
        launch_chunks(tb, gw, n, nchunk, ctab, s);
        if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
        // at most ~16 records per diff and sub-tile: one window per diff is plenty
        if (gw <= LD_WAVE) {
            if (thin) k_merge_sweep<20, 1, 1><<<grid, wave, 0, s>>>(w, n, nchunk, tb, gw, ctab, lr);
            else k_merge_sweep<10, 2, 1><<<grid, wave, 0, s>>>(w, n, nchunk, tb, gw, ctab, lr);
        } else {
            if (thin) k_merge_sweep<20, 1, 2><<<grid, wave, 0, s>>>(w, n, nchunk, tb, gw, ctab, lr);
            else k_merge_sweep<10, 2, 2><<<grid, wave, 0, s>>>(w, n, nchunk, tb, gw, ctab, lr);
        }
        if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    }
    return LD_OK;
}

}  // namespace

extern "C" ld_status ld_merge_sparse_strategy(float* w, int64_t n, const int32_t* const* idx,
                                              const float* const* val, const int64_t* K, int32_t W,
                                              float lr, void* workspace, size_t workspace_bytes,
                                              ld_stream stream, int32_t strategy) {
    return merge_sparse_impl(w, n, idx, val, K, W, lr, workspace, workspace_bytes, stream, strategy);
}

extern "C" ld_status ld_merge_sparse(float* w, int64_t n, const int32_t* const* idx,
                                     const float* const* val, const int64_t* K, int32_t W, float lr,
                                     void* workspace, size_t workspace_bytes, ld_stream stream) {
    return ld_merge_sparse_strategy(w, n, idx, val, K, W, lr, workspace, workspace_bytes, stream,
                                    LD_MERGE_AUTO);
}

// ------------------------------------------------ the entry point that allocates nothing
//
// The chunk table is the only scratch memory of the merge. Here it lives in a file-scope
// device array instead of a caller's workspace: one copy per GPU, held until the process
// ends, shared by every call on that GPU. Nothing in it has to start at zero (k_chunks
// writes every entry the sweep reads), so nothing is cleared between calls.
static __device__ __align__(256) unsigned char scratch[LD_MERGE_STATIC_SCRATCH];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<void*> scratch_ptr[kMaxDevices];  // per device: the address of ITS copy of `scratch`

// Device address of the current device's scratch array (looked up once per device; the array's
// name is only a host-side handle and is never passed to a kernel).
ld_status static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LD_ERR_HIP;
    void* p = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LD_ERR_HIP;
        scratch_ptr[dev].store(p, std::memory_order_release);  // every thread finds the same address
    }
    *out = p;
    return LD_OK;
}

}  // namespace

extern "C" size_t ld_merge_sparse_static_limit(void) { return LD_MERGE_STATIC_SCRATCH; }

extern "C" ld_status ld_merge_sparse_static(float* w, int64_t n, const int32_t* const* idx,
                                            const float* const* val, const int64_t* K, int32_t W, float lr,
                                            ld_stream stream) {
    const ld_status st = check_diff_args(w, n, idx, val, K, W);
    if (st != LD_OK) return st;
    if (chunk_table_bytes(n, W) > LD_MERGE_STATIC_SCRATCH) return LD_ERR_WORKSPACE;
    if (W == 0 || n == 0) return LD_OK;
    void* ptr = nullptr;
    const ld_status sp = static_scratch(&ptr);
    if (sp != LD_OK) return sp;
    return merge_sparse_impl(w, n, idx, val, K, W, lr, ptr, LD_MERGE_STATIC_SCRATCH, stream, LD_MERGE_AUTO);
}
