// ld_merge_sparse: ordered replay of a window of sparse diffs onto w.
//
// Recovery loop of Algorithm 1 (Sec. IV-B) and Eq. (6): M_{j+1} = M_j + merge(diff j)
// for j in iteration order, with the diffs of a batch kept apart and replayed one
// after another (Sec. IV-C, "Batched write semantics").  Update rule per record:
// p = fl32(lr*val); w[idx] = fl32(w[idx] - p).
//
// Two strategies with identical results:
//  * sweep   - one streaming pass over w.  A wave owns a 4096-element sub-tile
//              held in LDS, pulls the records of every diff that fall into it
//              (ranges precomputed by a binary-search kernel) and applies them
//              diff after diff.  LDS operations of one wave execute in issue
//              order, so the cross-diff order on an element needs no barrier.
//              HBM traffic: 8n + 8*sum(K) bytes + the range table.
//  * scatter - one kernel per diff, one thread per record; for windows that
//              touch only a small part of w.
#include "ld_common.h"

namespace {

constexpr int kSub = 4096;     // elements per wave sub-tile (16 KB of LDS)
constexpr int kWaves = 4;      // waves per block
constexpr int kGroupMax = 128; // diffs per launch (pointer table travels as a kernel argument)
constexpr int kPrefetch = 8;   // diffs whose records are loaded before any is applied

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

// tab[t*(nsub+1) + b] = number of records of diff t with idx < min(n, b*kSub).
// A workgroup covers 256 consecutive boundaries of one diff: two threads bracket
// the whole run with full searches, then every thread bisects inside the bracket
// (a few KB of indices that the workgroup shares through the cache).
__global__ __launch_bounds__(256) void k_partition(DiffTable tb, int64_t n, int32_t nsub,
                                                   int32_t* __restrict__ tab) {
    __shared__ int32_t bracket[2];
    const int32_t b0 = blockIdx.x * 256;
    const int32_t b = b0 + threadIdx.x;
    const int t = blockIdx.y;
    const int32_t* __restrict__ idx = tb.idx[t];
    const int32_t K = tb.K[t];
    if (threadIdx.x < 2) {
        int32_t bb = threadIdx.x == 0 ? b0 : b0 + 255;
        if (bb > nsub) bb = nsub;
        int64_t target = static_cast<int64_t>(bb) * kSub;
        if (target > n) target = n;
        bracket[threadIdx.x] = lower_bound_idx(idx, 0, K, target);
    }
    __syncthreads();
    if (b > nsub) return;
    int64_t target = static_cast<int64_t>(b) * kSub;
    if (target > n) target = n;
    tab[static_cast<int64_t>(t) * (nsub + 1) + b] = lower_bound_idx(idx, bracket[0], bracket[1], target);
}

__device__ __forceinline__ void apply_record(float* tile, int32_t local, float val, float lr) {
    const float p = __fmul_rn(lr, val);        // rounded product: never fused
    tile[local] = __fsub_rn(tile[local], p);
}

__global__ __launch_bounds__(256) void k_merge_sweep(float* __restrict__ w, int64_t n, int32_t nsub,
                                                     DiffTable tb, int32_t W,
                                                     const int32_t* __restrict__ tab, float lr) {
    __shared__ float tile_all[kWaves][kSub];
    const int wv = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    const int64_t sub = static_cast<int64_t>(blockIdx.x) * kWaves + wv;
    if (sub >= nsub) return;  // waves are independent: no block barrier anywhere below
    float* tile = tile_all[wv];
    const int64_t lo = sub * kSub;
    const int32_t len = static_cast<int32_t>((n - lo) < kSub ? (n - lo) : kSub);
    const bool full = (len == kSub);

    if (full) {
        const ld_f32x4* src = reinterpret_cast<const ld_f32x4*>(w + lo);
#pragma unroll
        for (int j = 0; j < kSub / 4 / LD_WAVE; ++j) {
            const ld_f32x4 x = ld_nt_load(src + j * LD_WAVE + lane);
            reinterpret_cast<ld_f32x4*>(tile)[j * LD_WAVE + lane] = x;
        }
    } else {
        for (int32_t e = lane; e < len; e += LD_WAVE) tile[e] = w[lo + e];
    }

    const int64_t stride = static_cast<int64_t>(nsub) + 1;
    const int32_t base = static_cast<int32_t>(lo);
    for (int32_t t0 = 0; t0 < W; t0 += kPrefetch) {
        int32_t p0[kPrefetch], cnt[kPrefetch], ri[kPrefetch];
        float rv[kPrefetch];
#pragma unroll
        for (int g = 0; g < kPrefetch; ++g) {
            const int32_t t = t0 + g;
            if (t < W) {
                p0[g] = tab[t * stride + sub];
                cnt[g] = tab[t * stride + sub + 1] - p0[g];
            } else {
                p0[g] = 0;
                cnt[g] = 0;
            }
        }
#pragma unroll
        for (int g = 0; g < kPrefetch; ++g) {
            ri[g] = 0;
            rv[g] = 0.0f;
            if (lane < cnt[g]) {
                ri[g] = __builtin_nontemporal_load(tb.idx[t0 + g] + p0[g] + lane);
                rv[g] = __builtin_nontemporal_load(tb.val[t0 + g] + p0[g] + lane);
            }
        }
#pragma unroll
        for (int g = 0; g < kPrefetch; ++g) {
            if (lane < cnt[g]) apply_record(tile, ri[g] - base, rv[g], lr);
            // more than 64 records of this diff in the sub-tile (density > 1.5 %)
            for (int32_t j = lane + LD_WAVE; j < cnt[g]; j += LD_WAVE) {
                const int32_t i = tb.idx[t0 + g][p0[g] + j];
                const float v = tb.val[t0 + g][p0[g] + j];
                apply_record(tile, i - base, v, lr);
            }
            __builtin_amdgcn_wave_barrier();  // keep diff g's LDS traffic ahead of diff g+1's
        }
    }

    if (full) {
        ld_f32x4* dst = reinterpret_cast<ld_f32x4*>(w + lo);
#pragma unroll
        for (int j = 0; j < kSub / 4 / LD_WAVE; ++j)
            ld_nt_store(reinterpret_cast<const ld_f32x4*>(tile)[j * LD_WAVE + lane], dst + j * LD_WAVE + lane);
    } else {
        for (int32_t e = lane; e < len; e += LD_WAVE) w[lo + e] = tile[e];
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

ld_status check_args(float* w, int64_t n, const int32_t* const* idx, const float* const* val,
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

extern "C" size_t ld_merge_sparse_workspace(int64_t n, int32_t W, const int64_t* K) {
    (void)K;
    if (n <= 0 || W <= 0) return 256;
    const int64_t group = W < kGroupMax ? W : kGroupMax;
    return ld_round_up(static_cast<size_t>(group) * (static_cast<size_t>(sub_tiles(n)) + 1) * 4, 256);
}

extern "C" ld_status ld_merge_sparse_strategy(float* w, int64_t n, const int32_t* const* idx,
                                              const float* const* val, const int64_t* K, int32_t W,
                                              float lr, void* workspace, size_t workspace_bytes,
                                              ld_stream stream, int32_t strategy) {
    const ld_status st = check_args(w, n, idx, val, K, W);
    if (st != LD_OK) return st;
    if (strategy < LD_MERGE_AUTO || strategy > LD_MERGE_SCATTER) return LD_ERR_RANGE;
    if (W == 0 || n == 0) return LD_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);

    int64_t total = 0;
    for (int32_t t = 0; t < W; ++t) total += K[t];
    if (total == 0) return LD_OK;
    if (strategy == LD_MERGE_AUTO)
        strategy = (total * 16 >= n) ? LD_MERGE_SWEEP : LD_MERGE_SCATTER;

    if (strategy == LD_MERGE_SCATTER) {
        for (int32_t t = 0; t < W; ++t) {
            if (K[t] == 0) continue;
            const int32_t k = static_cast<int32_t>(K[t]);
            k_merge_scatter<<<dim3((k + 255) / 256), dim3(256), 0, s>>>(w, idx[t], val[t], k, lr);
            if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
        }
        return LD_OK;
    }

    if (!workspace || !ld_aligned(workspace, 256) ||
        workspace_bytes < ld_merge_sparse_workspace(n, W, K))
        return LD_ERR_WORKSPACE;
    const int32_t nsub = sub_tiles(n);
    int32_t* tab = static_cast<int32_t*>(workspace);
    for (int32_t g0 = 0; g0 < W; g0 += kGroupMax) {
        const int32_t gw = (W - g0) < kGroupMax ? (W - g0) : kGroupMax;
        DiffTable tb;
        for (int32_t t = 0; t < kGroupMax; ++t) {
            const bool live = t < gw;
            tb.idx[t] = live ? idx[g0 + t] : nullptr;
            tb.val[t] = live ? val[g0 + t] : nullptr;
            tb.K[t] = live ? static_cast<int32_t>(K[g0 + t]) : 0;
        }
        k_partition<<<dim3((nsub + 1 + 255) / 256, gw), dim3(256), 0, s>>>(tb, n, nsub, tab);
        if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
        k_merge_sweep<<<dim3((nsub + kWaves - 1) / kWaves), dim3(256), 0, s>>>(w, n, nsub, tb, gw,
                                                                                tab, lr);
        if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    }
    return LD_OK;
}

extern "C" ld_status ld_merge_sparse(float* w, int64_t n, const int32_t* const* idx,
                                     const float* const* val, const int64_t* K, int32_t W, float lr,
                                     void* workspace, size_t workspace_bytes, ld_stream stream) {
    return ld_merge_sparse_strategy(w, n, idx, val, K, W, lr, workspace, workspace_bytes, stream,
                                    LD_MERGE_AUTO);
}
