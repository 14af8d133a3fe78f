// ld_merge_sparse_adam: ordered replay of a window of sparse diffs through Adam.
//
// Recovery loop of Algorithm 1 (Sec. IV-B) with the update the paper names there:
// for every diff j of the window, in iteration order, decompress it (Comp^-1: a dense
// gradient that is val at the recorded positions and zero elsewhere) and merge it with
// M_{j+1} = M_j + Adam(G_j) (Eq. (4)) into the model AND the optimizer state. Every
// element takes every step: a zero gradient still decays m and v and moves w.
//
// One streaming pass over (w, m, v): 24 n bytes + the records, whatever the window
// length. A wave owns a 2048-element sub-tile: its w, m, v live in registers (32
// elements per lane), the decompressed gradient of the current step in an 8 KB LDS
// tile that is zero except where the step's records were scattered. Per step: scatter
// the records that fall into the sub-tile, read the tile back, apply the shared Adam
// step to all 32 elements, clear the scattered positions again. The records are found
// as in ld_merge_sparse: chunk table + interpolated 128-record windows, verified.
// With W = 20 the arithmetic (20 x 14 flops per element, with a square root and a
// reciprocal each) outweighs the 24 bytes per element: this kernel is bound by the
// vector ALUs, not by HBM.
#include "ld_sparse_common.h"

namespace {

constexpr int kSub = 2048;                 // elements per wave sub-tile
constexpr int kChunkSubs = 24;             // sub-tiles per chunk of the range table
static_assert(static_cast<int64_t>(kSub) * kChunkSubs == kChunk, "sub-tiles must tile a chunk");
constexpr int kRows = kSub / 4 / LD_WAVE;  // 16-byte vectors per lane and array: 8
constexpr int kWin = 2;                    // 64-record windows per diff loaded ahead
constexpr int kMargin = 24;                // records the window starts before the interpolated position

// Writes (or clears) the records of [p, end) that fall into [lo, hi) into the gradient tile.
__device__ __forceinline__ void scatter_from(float* tile, const int32_t* __restrict__ idx,
                                             const float* __restrict__ val, int32_t p, int32_t end,
                                             int32_t lo, int32_t hi, bool clear, int lane) {
    for (; p < end; p += LD_WAVE) {
        const bool have = p + lane < end;
        const int32_t i = have ? idx[p + lane] : INT_MAX;
        const float v = (have && !clear) ? val[p + lane] : 0.0f;
        if (i >= lo && i < hi) tile[i - lo] = v;
        if (__ballot(i >= hi)) break;
    }
}

template <bool TINY_EPS>
__global__ __launch_bounds__(LD_WAVE) void k_sparse_adam(float* __restrict__ w, float* __restrict__ m,
                                                         float* __restrict__ v, int64_t n, int32_t nchunk,
                                                         DiffTable tb, int32_t W, LdAdamSteps a,
                                                         const int32_t* __restrict__ ctab) {
    __shared__ float tile[kSub];
    const int lane = threadIdx.x;
    // consecutive workgroups go to different XCDs: each XCD walks one contiguous eighth of the arrays
    const int64_t per = (static_cast<int64_t>(gridDim.x) + 7) / 8;
    const int64_t sub = static_cast<int64_t>(blockIdx.x % 8) * per + blockIdx.x / 8;
    if (sub * kSub >= n) return;
    const int64_t lo64 = sub * kSub;
    const int32_t len = static_cast<int32_t>((n - lo64) < kSub ? (n - lo64) : kSub);
    const int32_t lo = static_cast<int32_t>(lo64), hi = lo + len;  // n <= INT_MAX
    const bool full = (len == kSub);

    // state of the lane's 32 elements: vector j covers elements (j*64 + lane)*4 .. +3 of the sub-tile
    float ww[kRows][4], mm[kRows][4], vv[kRows][4];
#pragma unroll
    for (int j = 0; j < kRows; ++j) {
        const int32_t e = (j * LD_WAVE + lane) * 4;
        if (full) {
            const ld_f32x4 a4 = ld_nt_load(reinterpret_cast<const ld_f32x4*>(w + lo64 + e));
            const ld_f32x4 b4 = ld_nt_load(reinterpret_cast<const ld_f32x4*>(m + lo64 + e));
            const ld_f32x4 c4 = ld_nt_load(reinterpret_cast<const ld_f32x4*>(v + lo64 + e));
            ww[j][0] = a4.x; ww[j][1] = a4.y; ww[j][2] = a4.z; ww[j][3] = a4.w;
            mm[j][0] = b4.x; mm[j][1] = b4.y; mm[j][2] = b4.z; mm[j][3] = b4.w;
            vv[j][0] = c4.x; vv[j][1] = c4.y; vv[j][2] = c4.z; vv[j][3] = c4.w;
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bool in = e + q < len;
                ww[j][q] = in ? w[lo64 + e + q] : 0.0f;
                mm[j][q] = in ? m[lo64 + e + q] : 0.0f;
                vv[j][q] = in ? v[lo64 + e + q] : 0.0f;
            }
        }
    }

    // lane t: where diff t's records of this chunk lie, and the guess for this sub-tile
    const int32_t chunk = static_cast<int32_t>(sub / kChunkSubs), part = static_cast<int32_t>(sub % kChunkSubs);
    int32_t c0 = 0, c1 = 0;
    if (lane < W) {
        const int32_t* row = ctab + static_cast<int64_t>(lane) * (nchunk + 1) + chunk;
        c0 = row[0];
        c1 = row[1];
    }
    int32_t start = c0 + ((c1 - c0) * part) / kChunkSubs - kMargin;
    if (start < c0) start = c0;

#pragma unroll
    for (int j = 0; j < kRows; ++j)
        reinterpret_cast<ld_f32x4*>(tile)[j * LD_WAVE + lane] = ld_f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    __syncthreads();  // one wave: only orders the vector fill before the scalar scatters

    // One trip per diff; the record window of the next diff is requested before the current
    // one is applied (an Adam step over the sub-tile takes longer than a memory round trip).
    struct Window {
        int32_t s, e, b;        // first position of the window, end and begin of the chunk's records
        int32_t ri[kWin];
        float rv[kWin];
    };
    auto fetch = [&](int32_t t, Window& x) {
        const int tt = t < W ? t : 0;
        x.s = __builtin_amdgcn_readlane(start, tt);
        x.b = __builtin_amdgcn_readlane(c0, tt);
        x.e = t < W ? __builtin_amdgcn_readlane(c1, tt) : x.s;  // past W: an empty window
        const int32_t* __restrict__ ip = tb.idx[tt];
        const float* __restrict__ vp = tb.val[tt];
#pragma unroll
        for (int u = 0; u < kWin; ++u) {
            const int32_t p = x.s + u * LD_WAVE + lane;
            const bool h = p < x.e;
            x.ri[u] = h ? ip[p] : INT_MAX;
            x.rv[u] = h ? vp[p] : 0.0f;
        }
    };
    Window cur, nxt;
    fetch(0, cur);
#pragma unroll 1
    for (int32_t t = 0; t < W; ++t) {
        fetch(t + 1, nxt);
        int32_t p_slow = -1;  // where the sub-tile's records begin, when the window missed them
#pragma unroll 1
        for (int pass = 0; pass < 2; ++pass) {  // 0: scatter the records, 1: clear them again
            const bool clear = pass == 1;
            if (cur.s < cur.e) {
                const int32_t first = __builtin_amdgcn_readfirstlane(cur.ri[0]);
                if (cur.s == cur.b || first <= lo) {
                    // the window begins before the sub-tile's records do
                    bool more = true;
#pragma unroll
                    for (int u = 0; u < kWin; ++u) {
                        if (more) {
                            if (cur.ri[u] >= lo && cur.ri[u] < hi) tile[cur.ri[u] - lo] = clear ? 0.0f : cur.rv[u];
                            more = !__ballot(cur.ri[u] >= hi);
                        }
                    }
                    if (more)
                        scatter_from(tile, tb.idx[t], tb.val[t], cur.s + kWin * LD_WAVE, cur.e, lo, hi, clear, lane);
                } else {
                    // guess too late: find the first record of the sub-tile inside the chunk
                    if (p_slow < 0) p_slow = lower_bound_idx(tb.idx[t], cur.b, cur.s, lo);
                    scatter_from(tile, tb.idx[t], tb.val[t], p_slow, cur.e, lo, hi, clear, lane);
                }
            }
            if (!clear) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                const float lr_bc1 = a.lr_over_bc1[t], ibc2 = a.inv_bc2[t];
#pragma unroll
                for (int j = 0; j < kRows; ++j) {
                    const ld_f32x4 g4 = reinterpret_cast<const ld_f32x4*>(tile)[j * LD_WAVE + lane];
                    const float gq[4] = {g4.x, g4.y, g4.z, g4.w};
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        ld_adam_step<TINY_EPS>(ww[j][q], mm[j][q], vv[j][q], gq[q], a.beta1, a.one_m_beta1, a.beta2,
                                     a.one_m_beta2, a.eps, lr_bc1, ibc2);
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        }
        cur = nxt;
    }

#pragma unroll
    for (int j = 0; j < kRows; ++j) {
        const int32_t e = (j * LD_WAVE + lane) * 4;
        if (full) {
            ld_nt_store(ld_f32x4{ww[j][0], ww[j][1], ww[j][2], ww[j][3]}, reinterpret_cast<ld_f32x4*>(w + lo64 + e));
            ld_nt_store(ld_f32x4{mm[j][0], mm[j][1], mm[j][2], mm[j][3]}, reinterpret_cast<ld_f32x4*>(m + lo64 + e));
            ld_nt_store(ld_f32x4{vv[j][0], vv[j][1], vv[j][2], vv[j][3]}, reinterpret_cast<ld_f32x4*>(v + lo64 + e));
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (e + q < len) {
                    w[lo64 + e + q] = ww[j][q];
                    m[lo64 + e + q] = mm[j][q];
                    v[lo64 + e + q] = vv[j][q];
                }
            }
        }
    }
}

}  // namespace

extern "C" size_t ld_merge_sparse_adam_workspace(int64_t n, int32_t W, const int64_t* K) {
    (void)K;
    if (n <= 0 || W <= 0) return 256;
    const int64_t group = W < kGroupMax ? W : kGroupMax;
    return ld_round_up(static_cast<size_t>(group) * (static_cast<size_t>(chunks(n)) + 1) * 4, 256);
}

extern "C" ld_status ld_merge_sparse_adam(float* w, float* m, float* v, int64_t n,
                                          const int32_t* const* idx, const float* const* val,
                                          const int64_t* K, int32_t W, int64_t step0, float lr,
                                          float beta1, float beta2, float eps, void* workspace,
                                          size_t workspace_bytes, ld_stream stream) {
    const ld_status st = check_diff_args(w, n, idx, val, K, W);
    if (st != LD_OK) return st;
    if (step0 < 0) return LD_ERR_RANGE;
    if (!(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f)) return LD_ERR_RANGE;
    if (W == 0 || n == 0) return LD_OK;
    if (!m || !v) return LD_ERR_NULL;
    if (!ld_aligned(m, 16) || !ld_aligned(v, 16)) return LD_ERR_ALIGN;
    if (!workspace || !ld_aligned(workspace, 256) ||
        workspace_bytes < ld_merge_sparse_adam_workspace(n, W, K))
        return LD_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    ld_begin_call();
    const int32_t nsub = static_cast<int32_t>((n + kSub - 1) / kSub), nchunk = chunks(n);
    int32_t* ctab = static_cast<int32_t*>(workspace);
    static_assert(kGroupMax <= LD_MAX_ADAM_STEPS, "step table too small");
    for (int32_t g0 = 0; g0 < W; g0 += kGroupMax) {
        const int32_t gw = (W - g0) < kGroupMax ? (W - g0) : kGroupMax;
        DiffTable tb = {};
        for (int32_t t = 0; t < kGroupMax; ++t) {
            const bool live = t < gw;
            tb.idx[t] = live ? idx[g0 + t] : nullptr;
            tb.val[t] = live ? val[g0 + t] : nullptr;
            tb.K[t] = live ? static_cast<int32_t>(K[g0 + t]) : 0;
        }
        LdAdamSteps a;
        ld_fill_adam_steps(a, gw, step0 + g0, lr, beta1, beta2, eps);
        launch_chunks(tb, gw, n, nchunk, ctab, s);
        if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
        if (ld_adam_careful(eps))
            k_sparse_adam<true><<<dim3((nsub + 7) / 8 * 8), dim3(LD_WAVE), 0, s>>>(w, m, v, n, nchunk, tb, gw, a, ctab);
        else
            k_sparse_adam<false><<<dim3((nsub + 7) / 8 * 8), dim3(LD_WAVE), 0, s>>>(w, m, v, n, nchunk, tb, gw, a, ctab);
        if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    }
    return LD_OK;
}
