// ld_compress_topk: per-segment exact top-k sparsification with error feedback.
//
// Comp of Algorithm 1 (Sec. IV-B) at ratio rho (Sec. II-C, Sec. VII-A): the
// compressed gradient that is reused as the differential checkpoint.  The
// selection rule (|r+g| descending on the bit pattern, ties to the lower index,
// records ascending, selected residuals zeroed) is stated in lowdiff.h.
//
// Every segment is cut into chunks of kChunk elements, one workgroup per chunk.
// The k-th largest key of a segment is found by a three-level radix select
// (11 + 11 + 9 bits of the 31-bit magnitude key); the per-segment digit
// histogram lives in global memory, is fed from per-workgroup LDS histograms,
// and is resolved by whichever workgroup finishes a segment's level last
// (ticket counter), so no level needs a launch of its own:
//
//   k_accum   a = r + g -> residual; level-1 histogram
//   k_level   level-2, then level-3 histogram over keys matching the prefix
//   k_count   per chunk: #keys above the threshold, #keys equal to it; the last
//             workgroup of a segment turns them into per-chunk output offsets
//   k_emit    ordered compaction of (idx, val); selected residuals <- +0
#include <vector>

#include "ld_common.h"

namespace {

constexpr int kThreads = 256;
constexpr int kRows = 4;                          // float4 rows per thread per tile
constexpr int kTile = kThreads * 4 * kRows;       // 4096 elements
constexpr int kChunk = 65536;                     // elements per workgroup
constexpr int kBins = 2048;
constexpr int kShift1 = 20, kShift2 = 9;          // digit positions: [30:20] [19:9] [8:0]
constexpr int kDescPerLaunch = 160;

struct SegDesc {        // one per segment plus a sentinel; written by k_upload
    int64_t off;        // first element
    int64_t out0;       // first output record
    int32_t k;          // records to keep
    int32_t chunk0;     // first chunk
};

struct SegState {       // selection progress of one segment
    uint32_t prefix;    // key bits fixed so far (0xFFFFFFFF: keep nothing)
    uint32_t krem;      // rank still to resolve inside the prefix bucket
    uint32_t done[4];   // ticket counters: level 1, 2, 3, count
    uint32_t pad[2];
};

struct Ctx {
    SegDesc* desc;        // [n_seg + 1]
    SegState* state;      // [n_seg]
    uint32_t* hist;       // [n_seg][kBins]
    int32_t* chunk_seg;   // [n_chunk]
    uint32_t* chunk_gt;   // [n_chunk] keys above threshold -> exclusive output offset in segment
    uint32_t* chunk_eq;   // [n_chunk] keys equal to threshold -> exclusive tie rank in segment
    int32_t n_seg;
    int32_t n_chunk;
};

struct UploadBatch {
    SegDesc d[kDescPerLaunch];
    int32_t first;  // index of d[0] in the descriptor table
    int32_t count;
    int32_t n_seg;
};

__host__ __device__ inline int64_t align_down4(int64_t x) { return x & ~static_cast<int64_t>(3); }

__host__ __device__ inline int32_t chunks_of(int64_t off, int64_t end) {
    if (end <= off) return 0;
    return static_cast<int32_t>((end - align_down4(off) + kChunk - 1) / kChunk);
}

// Writes the descriptors of a batch of segments, clears their selection state
// and histogram, and fills the chunk -> segment map. One workgroup per entry.
__global__ __launch_bounds__(kThreads) void k_upload(UploadBatch ub, Ctx c) {
    const int j = blockIdx.x;
    const int s = ub.first + j;
    const SegDesc d = ub.d[j];
    if (threadIdx.x == 0) c.desc[s] = d;
    if (s >= ub.n_seg) return;  // sentinel
    if (threadIdx.x < 8) reinterpret_cast<uint32_t*>(&c.state[s])[threadIdx.x] = 0;
    for (int b = threadIdx.x; b < kBins; b += kThreads) c.hist[static_cast<int64_t>(s) * kBins + b] = 0;
    const int32_t nchunk = ub.d[j + 1].chunk0 - d.chunk0;
    for (int32_t q = threadIdx.x; q < nchunk; q += kThreads) c.chunk_seg[d.chunk0 + q] = s;
}

struct ChunkRange {
    int32_t seg;
    int64_t cs, ce;      // element range of this chunk
    int64_t t0;          // first tile start (multiple of 4)
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
    const int64_t q = chunk - d.chunk0;
    r.cs = base + q * kChunk;
    r.ce = r.cs + kChunk;
    r.t0 = r.cs;
    if (r.cs < d.off) r.cs = d.off;
    if (r.ce > dn.off) r.ce = dn.off;
    r.k = d.k;
    r.chunk0 = d.chunk0;
    r.nchunk = dn.chunk0 - d.chunk0;
    r.out0 = d.out0;
    return r;
}

// Loads the 4 elements at e0..e0+3 that lie inside [cs, ce); returns the mask of
// valid components. e0 is a multiple of 4 and `p` is 16-byte aligned.
__device__ __forceinline__ uint32_t load4(const float* __restrict__ p, int64_t e0, int64_t cs,
                                          int64_t ce, float (&x)[4]) {
    if (e0 >= cs && e0 + 4 <= ce) {
        const float4 q = *reinterpret_cast<const float4*>(p + e0);
        x[0] = q.x; x[1] = q.y; x[2] = q.z; x[3] = q.w;
        return 0xF;
    }
    uint32_t mask = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        x[c] = 0.0f;
        if (e0 + c >= cs && e0 + c < ce) {
            x[c] = p[e0 + c];
            mask |= 1u << c;
        }
    }
    return mask;
}

__device__ __forceinline__ void store4(float* __restrict__ p, int64_t e0, uint32_t mask,
                                       const float (&x)[4]) {
    if (mask == 0xF) {
        *reinterpret_cast<float4*>(p + e0) = make_float4(x[0], x[1], x[2], x[3]);
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (mask & (1u << c)) p[e0 + c] = x[c];
    }
}

// After a workgroup has pushed its contribution for `phase` of segment `seg`:
// returns true in exactly one workgroup per (segment, phase) - the last one -
// and only after every other workgroup's contribution is visible to it.
__device__ __forceinline__ bool last_of_segment(const Ctx& c, int32_t seg, int phase, int32_t nchunk) {
    __shared__ uint32_t ticket;
    __threadfence();  // every thread publishes its own contribution
    __syncthreads();
    if (threadIdx.x == 0) ticket = atomicAdd(&c.state[seg].done[phase], 1u);
    __syncthreads();
    const bool last = (ticket == static_cast<uint32_t>(nchunk - 1));
    if (last) __threadfence();
    return last;
}

// The last workgroup of a level: finds the digit d with
//   #(digit > d) < krem <= #(digit >= d)
// in the segment's histogram, folds it into the prefix, and clears the histogram.
__device__ void resolve_level(const Ctx& c, int32_t seg, int shift, uint32_t krem_in, uint32_t prefix_in,
                              uint32_t* sh /* >= 4 words */) {
    uint32_t* h = c.hist + static_cast<int64_t>(seg) * kBins;
    // thread t owns the 8 digits 8t .. 8t+7, scanned from the top digit down
    const int top = kBins - 1 - threadIdx.x * 8;
    uint32_t v[8], sum = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        v[i] = ld_load_coherent(h + top - i);
        sum += v[i];
    }
    uint32_t total;
    uint32_t above = ld_block_escan256(sum, sh, total);  // keys with a higher digit than my first
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        if (above < krem_in && krem_in <= above + v[i]) {
            c.state[seg].prefix = prefix_in | (static_cast<uint32_t>(top - i) << shift);
            c.state[seg].krem = krem_in - above;
        }
        above += v[i];
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) h[top - i] = 0;
}

__device__ __forceinline__ void flush_hist(const Ctx& c, int32_t seg, uint32_t* lh) {
    uint32_t* h = c.hist + static_cast<int64_t>(seg) * kBins;
    for (int b = threadIdx.x; b < kBins; b += kThreads) {
        const uint32_t x = lh[b];
        if (x) atomicAdd(h + b, x);
    }
}

// Pass 1: a = r + g -> residual, level-1 histogram.
__global__ __launch_bounds__(kThreads) void k_accum(const float* __restrict__ g, float* __restrict__ r,
                                                    Ctx c) {
    __shared__ uint32_t lh[kBins];
    __shared__ uint32_t sh[4];
    const ChunkRange cr = chunk_range(c, blockIdx.x);
    for (int b = threadIdx.x; b < kBins; b += kThreads) lh[b] = 0;
    __syncthreads();
    for (int64_t t = cr.t0; t < cr.ce; t += kTile) {
        float a[kRows][4];
        uint32_t mask[kRows];
#pragma unroll
        for (int j = 0; j < kRows; ++j) {
            const int64_t e0 = t + (j * kThreads + threadIdx.x) * 4;
            float gv[4], rv[4];
            mask[j] = load4(g, e0, cr.cs, cr.ce, gv);
            load4(r, e0, cr.cs, cr.ce, rv);
#pragma unroll
            for (int q = 0; q < 4; ++q) a[j][q] = __fadd_rn(rv[q], gv[q]);
        }
#pragma unroll
        for (int j = 0; j < kRows; ++j) {
            const int64_t e0 = t + (j * kThreads + threadIdx.x) * 4;
            store4(r, e0, mask[j], a[j]);
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (mask[j] & (1u << q)) atomicAdd(&lh[ld_key(a[j][q]) >> kShift1], 1u);
        }
    }
    __syncthreads();
    flush_hist(c, cr.seg, lh);
    if (last_of_segment(c, cr.seg, 0, cr.nchunk)) {
        if (cr.k == 0) {
            if (threadIdx.x == 0) { c.state[cr.seg].prefix = 0xFFFFFFFFu; c.state[cr.seg].krem = 0; }
            uint32_t* h = c.hist + static_cast<int64_t>(cr.seg) * kBins;
            for (int b = threadIdx.x; b < kBins; b += kThreads) h[b] = 0;
        } else {
            resolve_level(c, cr.seg, kShift1, static_cast<uint32_t>(cr.k), 0u, sh);
        }
    }
}

// Levels 2 and 3: histogram of the next digit over keys that match the prefix.
template <int LEVEL>
__global__ __launch_bounds__(kThreads) void k_level(const float* __restrict__ r, Ctx c) {
    __shared__ uint32_t lh[kBins];
    __shared__ uint32_t sh[4];
    const ChunkRange cr = chunk_range(c, blockIdx.x);
    if (cr.k == 0) return;
    const uint32_t prefix = c.state[cr.seg].prefix;
    const uint32_t krem = c.state[cr.seg].krem;
    constexpr int match_shift = (LEVEL == 2) ? kShift1 : kShift2;
    constexpr int digit_shift = (LEVEL == 2) ? kShift2 : 0;
    constexpr uint32_t digit_mask = (LEVEL == 2) ? 0x7FFu : 0x1FFu;
    for (int b = threadIdx.x; b < kBins; b += kThreads) lh[b] = 0;
    __syncthreads();
    for (int64_t t = cr.t0; t < cr.ce; t += kTile) {
#pragma unroll
        for (int j = 0; j < kRows; ++j) {
            const int64_t e0 = t + (j * kThreads + threadIdx.x) * 4;
            float x[4];
            const uint32_t mask = load4(r, e0, cr.cs, cr.ce, x);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t key = ld_key(x[q]);
                if ((mask & (1u << q)) && (key >> match_shift) == (prefix >> match_shift))
                    atomicAdd(&lh[(key >> digit_shift) & digit_mask], 1u);
            }
        }
    }
    __syncthreads();
    flush_hist(c, cr.seg, lh);
    if (last_of_segment(c, cr.seg, LEVEL - 1, cr.nchunk))
        resolve_level(c, cr.seg, digit_shift, krem, prefix, sh);
}

// Per chunk: keys above / equal to the threshold; the last workgroup of the
// segment converts the per-chunk counts into exclusive offsets.
__global__ __launch_bounds__(kThreads) void k_count(const float* __restrict__ r, Ctx c) {
    __shared__ uint32_t sh[4];
    const ChunkRange cr = chunk_range(c, blockIdx.x);
    const uint32_t T = c.state[cr.seg].prefix;
    const uint32_t m = c.state[cr.seg].krem;
    uint32_t gt = 0, eq = 0;
    for (int64_t t = cr.t0; t < cr.ce; t += kTile) {
#pragma unroll
        for (int j = 0; j < kRows; ++j) {
            const int64_t e0 = t + (j * kThreads + threadIdx.x) * 4;
            float x[4];
            const uint32_t mask = load4(r, e0, cr.cs, cr.ce, x);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t key = ld_key(x[q]);
                if (mask & (1u << q)) {
                    gt += (key > T);
                    eq += (key == T);
                }
            }
        }
    }
    uint32_t tot_gt, tot_eq;
    ld_block_escan256(gt, sh, tot_gt);
    ld_block_escan256(eq, sh, tot_eq);
    if (threadIdx.x == 0) {
        c.chunk_gt[blockIdx.x] = tot_gt;
        c.chunk_eq[blockIdx.x] = tot_eq;
    }
    if (!last_of_segment(c, cr.seg, 3, cr.nchunk)) return;
    // exclusive scan over the segment's chunks, 256 at a time
    uint32_t carry_out = 0, carry_eq = 0;
    for (int32_t q0 = 0; q0 < cr.nchunk; q0 += kThreads) {
        const int32_t q = q0 + threadIdx.x;
        uint32_t cg = 0, ce = 0;
        if (q < cr.nchunk) {
            cg = ld_load_coherent(c.chunk_gt + cr.chunk0 + q);
            ce = ld_load_coherent(c.chunk_eq + cr.chunk0 + q);
        }
        uint32_t te, tg;
        const uint32_t eq_before = carry_eq + ld_block_escan256(ce, sh, te);
        // ties taken from this chunk: those with tie rank < m
        uint32_t take = 0;
        if (eq_before < m) take = (m - eq_before < ce) ? (m - eq_before) : ce;
        const uint32_t out_before = carry_out + ld_block_escan256(cg + take, sh, tg);
        if (q < cr.nchunk) {
            c.chunk_gt[cr.chunk0 + q] = out_before;
            c.chunk_eq[cr.chunk0 + q] = eq_before;
        }
        carry_eq += te;
        carry_out += tg;
    }
}

// Ordered compaction: element order inside a tile is (row, thread, component).
__global__ __launch_bounds__(kThreads) void k_emit(float* __restrict__ r, int32_t* __restrict__ out_idx,
                                                   float* __restrict__ out_val, Ctx c) {
    __shared__ uint32_t part[2][kRows * 4];  // packed (selected | ties << 16) per (row, wave)
    const ChunkRange cr = chunk_range(c, blockIdx.x);
    if (cr.k == 0) return;
    const uint32_t T = c.state[cr.seg].prefix;
    const uint32_t m = c.state[cr.seg].krem;
    uint32_t run_out = c.chunk_gt[blockIdx.x];  // records of this segment emitted before this chunk
    uint32_t run_eq = c.chunk_eq[blockIdx.x];   // ties seen before this chunk
    const int lane = ld_lane();
    const int wv = threadIdx.x >> 6;
    int buf = 0;
    for (int64_t t = cr.t0; t < cr.ce; t += kTile, buf ^= 1) {
        float x[kRows][4];
        uint32_t mask[kRows];
        uint32_t fl_gt[kRows], fl_eq[kRows];   // 4-bit component flags
        uint32_t pre_gt[kRows], pre_eq[kRows]; // exclusive prefix inside the wave row
#pragma unroll
        for (int j = 0; j < kRows; ++j) {
            const int64_t e0 = t + (j * kThreads + threadIdx.x) * 4;
            mask[j] = load4(r, e0, cr.cs, cr.ce, x[j]);
            fl_gt[j] = fl_eq[j] = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t key = ld_key(x[j][q]);
                if (mask[j] & (1u << q)) {
                    fl_gt[j] |= static_cast<uint32_t>(key > T) << q;
                    fl_eq[j] |= static_cast<uint32_t>(key == T) << q;
                }
            }
            const uint32_t cg = __popc(fl_gt[j]), ce = __popc(fl_eq[j]);
            const uint32_t inc = ld_wave_iscan(cg | (ce << 16));
            pre_gt[j] = (inc & 0xFFFFu) - cg;
            pre_eq[j] = (inc >> 16) - ce;
            if (lane == LD_WAVE - 1) part[buf][j * 4 + wv] = inc;
        }
        __syncthreads();
        // (row, wave) slots in element order: row-major, wave-minor
        uint32_t acc_gt = 0, acc_eq = 0;
        uint32_t base_gt[kRows], base_eq[kRows];
#pragma unroll
        for (int j = 0; j < kRows; ++j) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (u == wv) { base_gt[j] = acc_gt; base_eq[j] = acc_eq; }
                const uint32_t p = part[buf][j * 4 + u];
                acc_gt += p & 0xFFFFu;
                acc_eq += p >> 16;
            }
        }
        // positions: a tie is taken iff its rank among the segment's ties is < m
        // selected-before = gt-before + min(ties-before, m) (ties are taken lowest index first)
        const uint32_t tile_eq0 = run_eq;
        const uint32_t tile_out0 = run_out;
#pragma unroll
        for (int j = 0; j < kRows; ++j) {
            const int64_t e0 = t + (j * kThreads + threadIdx.x) * 4;
            uint32_t gt_before = base_gt[j] + pre_gt[j];
            uint32_t eq_before = tile_eq0 + base_eq[j] + pre_eq[j];
            bool touched = false;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bool is_gt = (fl_gt[j] >> q) & 1u;
                const bool is_eq = (fl_eq[j] >> q) & 1u;
                const bool sel = is_gt || (is_eq && eq_before < m);
                if (sel) {
                    const uint32_t ties_taken_before = (eq_before < m ? eq_before : m) - (tile_eq0 < m ? tile_eq0 : m);
                    const int64_t pos = cr.out0 + tile_out0 + gt_before + ties_taken_before;
                    out_idx[pos] = static_cast<int32_t>(e0 + q);
                    out_val[pos] = x[j][q];
                    x[j][q] = 0.0f;
                    touched = true;
                }
                gt_before += is_gt;
                eq_before += is_eq;
            }
            if (touched) store4(r, e0, mask[j], x[j]);
        }
        const uint32_t eq_end = tile_eq0 + acc_eq;
        run_out += acc_gt + ((eq_end < m ? eq_end : m) - (tile_eq0 < m ? tile_eq0 : m));
        run_eq = eq_end;
    }
}

struct Layout {
    size_t desc, state, hist, chunk_seg, chunk_gt, chunk_eq, total;
};

Layout layout(int32_t n_seg, int64_t n_chunk) {
    Layout L;
    size_t o = 0;
    L.desc = o;      o += ld_round_up(sizeof(SegDesc) * (static_cast<size_t>(n_seg) + 1), 256);
    L.state = o;     o += ld_round_up(sizeof(SegState) * static_cast<size_t>(n_seg), 256);
    L.hist = o;      o += ld_round_up(sizeof(uint32_t) * kBins * static_cast<size_t>(n_seg), 256);
    L.chunk_seg = o; o += ld_round_up(sizeof(int32_t) * static_cast<size_t>(n_chunk), 256);
    L.chunk_gt = o;  o += ld_round_up(sizeof(uint32_t) * static_cast<size_t>(n_chunk), 256);
    L.chunk_eq = o;  o += ld_round_up(sizeof(uint32_t) * static_cast<size_t>(n_chunk), 256);
    L.total = o + 256;
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

extern "C" ld_status ld_compress_topk(const float* grad, float* residual, const int64_t* seg_off,
                                      const int32_t* seg_k, int32_t n_seg, int32_t* out_idx,
                                      float* out_val, void* workspace, size_t workspace_bytes,
                                      ld_stream stream) {
    if (n_seg < 0) return LD_ERR_RANGE;
    if (n_seg == 0) return LD_OK;
    if (!seg_off || !seg_k) return LD_ERR_NULL;
    const int64_t n_chunk = count_chunks(n_seg, seg_off);
    if (n_chunk < 0 || n_chunk > INT32_MAX) return LD_ERR_RANGE;
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
    c.chunk_gt = reinterpret_cast<uint32_t*>(ws + L.chunk_gt);
    c.chunk_eq = reinterpret_cast<uint32_t*>(ws + L.chunk_eq);
    c.n_seg = n_seg;
    c.n_chunk = static_cast<int32_t>(n_chunk);

    // Descriptor table: n_seg entries + a sentinel. A launch writes up to
    // kDescPerLaunch - 1 entries and also carries the entry after its last one,
    // whose chunk0 tells how many chunks that last entry has.
    {
        std::vector<SegDesc> desc(static_cast<size_t>(n_seg) + 1);
        int64_t out0 = 0;
        int32_t chunk0 = 0;
        for (int32_t s = 0; s <= n_seg; ++s) {
            desc[s].off = seg_off[s];
            desc[s].out0 = out0;
            desc[s].chunk0 = chunk0;
            desc[s].k = (s < n_seg) ? seg_k[s] : 0;
            if (s < n_seg) {
                out0 += seg_k[s];
                chunk0 += chunks_of(seg_off[s], seg_off[s + 1]);
            }
        }
        constexpr int32_t per = kDescPerLaunch - 1;
        for (int32_t s = 0; s <= n_seg; s += per) {
            UploadBatch ub;
            const int32_t own = (n_seg + 1 - s) < per ? (n_seg + 1 - s) : per;
            for (int32_t j = 0; j < kDescPerLaunch; ++j) {
                const int32_t q = (s + j <= n_seg) ? (s + j) : n_seg;
                ub.d[j] = desc[q];
            }
            ub.first = s;
            ub.count = own;
            ub.n_seg = n_seg;
            k_upload<<<dim3(own), dim3(kThreads), 0, st>>>(ub, c);
            if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
        }
    }
    if (n_chunk == 0) return LD_OK;
    const dim3 grid(static_cast<uint32_t>(n_chunk)), block(kThreads);
    k_accum<<<grid, block, 0, st>>>(grad, residual, c);
    if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    if (K == 0) return LD_OK;
    k_level<2><<<grid, block, 0, st>>>(residual, c);
    if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    k_level<3><<<grid, block, 0, st>>>(residual, c);
    if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    k_count<<<grid, block, 0, st>>>(residual, c);
    if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    k_emit<<<grid, block, 0, st>>>(residual, out_idx, out_val, c);
    return ld_launch_status();
}
