// LowDiff+ dense path: layer snapshot and incremental Adam merge.
//
// ld_snapshot_layer(s): Snapshot(G^n_t) of Algorithm 2 (Sec. VI-B) - as soon as a
//   layer's synchronized gradient exists it is copied, bit for bit, into a
//   checkpoint-owned buffer so the backward pass may go on.  Here the copy stays
//   in HBM (streaming 16-byte loads/stores); the multi-layer entry packs many
//   small layers into one launch (Sec. VI-C, "Snapshotting module").
// ld_merge_dense_adam: "Merge in CPU" of Algorithm 2, M <- M + Adam(o_t, G_t)
//   (Eq. (4)), with the replica kept in HBM and the W steps of a window fused
//   into one pass: (24 + 2W) bytes per parameter instead of 26 per step.
#include <math.h>

#include "ld_common.h"

namespace {

// ----------------------------------------------------------------- snapshot

constexpr int kCopyThreads = 256;
constexpr int kCopyUnroll = 4;                                    // 16-byte vectors per thread
constexpr int64_t kCopyBlockBytes = kCopyThreads * kCopyUnroll * 16;  // 16 KB per block
constexpr int kLayersPerLaunch = 128;

struct CopyJob {
    const unsigned char* src;
    unsigned char* dst;
    int64_t bytes;
};

struct CopyBatch {
    CopyJob job[kLayersPerLaunch];
    int32_t first_block[kLayersPerLaunch + 1];  // prefix of blocks per layer
    int32_t n;
};

__device__ __forceinline__ void copy_block(const unsigned char* __restrict__ src,
                                           unsigned char* __restrict__ dst, int64_t bytes,
                                           int64_t blk) {
    const int64_t b0 = blk * kCopyBlockBytes;
    const int64_t b1 = (b0 + kCopyBlockBytes < bytes) ? b0 + kCopyBlockBytes : bytes;
    const bool vec = ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) == 0;
    if (vec && b1 - b0 == kCopyBlockBytes) {
        const ld_u32x4* s = reinterpret_cast<const ld_u32x4*>(src + b0);
        ld_u32x4* d = reinterpret_cast<ld_u32x4*>(dst + b0);
        ld_u32x4 x[kCopyUnroll];
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u) x[u] = ld_nt_load(s + u * kCopyThreads + threadIdx.x);
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u) ld_nt_store(x[u], d + u * kCopyThreads + threadIdx.x);
    } else {
        // ragged tail or unaligned layer: 2-byte elements
        const uint16_t* s = reinterpret_cast<const uint16_t*>(src + b0);
        uint16_t* d = reinterpret_cast<uint16_t*>(dst + b0);
        const int32_t cnt = static_cast<int32_t>((b1 - b0) >> 1);
        for (int32_t e = threadIdx.x; e < cnt; e += kCopyThreads) d[e] = s[e];
    }
}

__global__ __launch_bounds__(kCopyThreads) void k_snapshot(const unsigned char* __restrict__ src,
                                                           unsigned char* __restrict__ dst,
                                                           int64_t bytes) {
    // consecutive workgroups go to different XCDs: each XCD copies one contiguous eighth
    const int64_t per = (static_cast<int64_t>(gridDim.x) + 7) / 8;
    const int64_t blk = static_cast<int64_t>(blockIdx.x % 8) * per + blockIdx.x / 8;
    if (blk * kCopyBlockBytes < bytes) copy_block(src, dst, bytes, blk);
}

__global__ __launch_bounds__(kCopyThreads) void k_snapshot_batch(CopyBatch cb) {
    // which layer does this block belong to: binary search in the block prefix
    // consecutive workgroups go to different XCDs: each XCD copies one contiguous eighth of the launch
    const int32_t per = (static_cast<int32_t>(gridDim.x) + 7) / 8;
    const int32_t blk = static_cast<int32_t>(blockIdx.x % 8) * per + static_cast<int32_t>(blockIdx.x / 8);
    if (blk >= cb.first_block[cb.n]) return;
    int lo = 0, hi = cb.n;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cb.first_block[mid] <= blk) lo = mid; else hi = mid;
    }
    copy_block(cb.job[lo].src, cb.job[lo].dst, cb.job[lo].bytes, blk - cb.first_block[lo]);
}

// --------------------------------------------------------------------- Adam

struct AdamArgs {
    const uint16_t* grad[LD_MAX_ADAM_WINDOW];
    LdAdamSteps s;
    int32_t W;
};

constexpr int kAdamThreads = 256;
constexpr int kAdamH = 4;                          // 16-byte fp32 vectors per thread and array
constexpr int kAdamBlockElems = kAdamThreads * 4 * kAdamH; // elements per workgroup

typedef uint32_t ld_u32x2 __attribute__((ext_vector_type(2)));

// Replays steps [t0, t0 + WT) of the window (those below a.W). One workgroup per
// kAdamBlockElems consecutive elements; every load instruction of a wave covers
// one contiguous run (16 bytes of fp32 state or 8 bytes of bf16 gradient per
// lane), and all loads are issued before the first value is used. Consecutive
// workgroups go to different XCDs, so each XCD is given one contiguous eighth of
// the arrays (its address translations and DRAM pages stay its own).
template <int WT, bool TINY_EPS>
__global__ __launch_bounds__(kAdamThreads) void k_adam(float* __restrict__ w, float* __restrict__ m,
                                                       float* __restrict__ v, int64_t n, AdamArgs a, int t0) {
    const int64_t per = (static_cast<int64_t>(gridDim.x) + 7) / 8;
    const int64_t blk = static_cast<int64_t>(blockIdx.x % 8) * per + blockIdx.x / 8;
    const int64_t b0 = blk * kAdamBlockElems;
    if (b0 >= n) return;
    if (b0 + kAdamBlockElems <= n) {
        const int64_t q0 = b0 / 4 + threadIdx.x;  // index of the thread's first 4-element vector
        ld_f32x4 wv[kAdamH], mv[kAdamH], vv[kAdamH];
        ld_u32x2 gq[WT][kAdamH];
#pragma unroll
        for (int t = 0; t < WT; ++t)
#pragma unroll
            for (int h = 0; h < kAdamH; ++h)
                gq[t][h] = (t0 + t < a.W) ? __builtin_nontemporal_load(reinterpret_cast<const ld_u32x2*>(a.grad[t0 + t]) +
                                                                       q0 + h * kAdamThreads)
                                          : ld_u32x2{0u, 0u};
        ld_f32x4* w4 = reinterpret_cast<ld_f32x4*>(w) + q0;
        ld_f32x4* m4 = reinterpret_cast<ld_f32x4*>(m) + q0;
        ld_f32x4* v4 = reinterpret_cast<ld_f32x4*>(v) + q0;
#pragma unroll
        for (int h = 0; h < kAdamH; ++h) {
            wv[h] = ld_nt_load(w4 + h * kAdamThreads);
            mv[h] = ld_nt_load(m4 + h * kAdamThreads);
            vv[h] = ld_nt_load(v4 + h * kAdamThreads);
        }
#pragma unroll
        for (int h = 0; h < kAdamH; ++h) {
            float ww[4] = {wv[h].x, wv[h].y, wv[h].z, wv[h].w};
            float mm[4] = {mv[h].x, mv[h].y, mv[h].z, mv[h].w};
            float v4_[4] = {vv[h].x, vv[h].y, vv[h].z, vv[h].w};
#pragma unroll
            for (int t = 0; t < WT; ++t) {
                if (t0 + t < a.W) {
                    const uint32_t gw[2] = {gq[t][h].x, gq[t][h].y};
                    const float lr_bc1 = a.s.lr_over_bc1[t0 + t], ibc2 = a.s.inv_bc2[t0 + t];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint32_t half = (e & 1) ? (gw[e >> 1] >> 16) : (gw[e >> 1] & 0xFFFFu);
                        ld_adam_step<TINY_EPS>(ww[e], mm[e], v4_[e], ld_bf16_widen(half), a.s.beta1, a.s.one_m_beta1, a.s.beta2,
                                  a.s.one_m_beta2, a.s.eps, lr_bc1, ibc2);
                    }
                }
            }
            ld_nt_store(ld_f32x4{ww[0], ww[1], ww[2], ww[3]}, w4 + h * kAdamThreads);
            ld_nt_store(ld_f32x4{mm[0], mm[1], mm[2], mm[3]}, m4 + h * kAdamThreads);
            ld_nt_store(ld_f32x4{v4_[0], v4_[1], v4_[2], v4_[3]}, v4 + h * kAdamThreads);
        }
    } else {
        // the last, ragged workgroup: element by element
        for (int64_t e = b0 + threadIdx.x; e < n; e += kAdamThreads) {
            float ww = w[e], mm = m[e], v1 = v[e];
            for (int t = t0; t < t0 + WT && t < a.W; ++t)
                ld_adam_step<TINY_EPS>(ww, mm, v1, ld_bf16_widen(a.grad[t][e]), a.s.beta1, a.s.one_m_beta1, a.s.beta2,
                          a.s.one_m_beta2, a.s.eps, a.s.lr_over_bc1[t], a.s.inv_bc2[t]);
            w[e] = ww;
            m[e] = mm;
            v[e] = v1;
        }
    }
}

}  // namespace

extern "C" ld_status ld_snapshot_layer(const void* grad_bf16, void* snap_bf16, int64_t n_elems,
                                       ld_stream stream) {
    if (n_elems < 0) return LD_ERR_RANGE;
    if (n_elems == 0) return LD_OK;
    if (!grad_bf16 || !snap_bf16) return LD_ERR_NULL;
    if (!ld_aligned(grad_bf16, 2) || !ld_aligned(snap_bf16, 2)) return LD_ERR_ALIGN;
    const int64_t bytes = n_elems * 2;
    const int64_t blocks = (bytes + kCopyBlockBytes - 1) / kCopyBlockBytes;
    if (blocks > INT32_MAX - 8) return LD_ERR_RANGE;
    ld_begin_call();
    k_snapshot<<<dim3(static_cast<uint32_t>((blocks + 7) / 8 * 8)), dim3(kCopyThreads), 0,
                 static_cast<hipStream_t>(stream)>>>(static_cast<const unsigned char*>(grad_bf16),
                                                     static_cast<unsigned char*>(snap_bf16), bytes);
    return ld_launch_status();
}

extern "C" ld_status ld_snapshot_layers(const void* const* src, void* const* dst,
                                        const int64_t* n_elems, int32_t n_layers, ld_stream stream) {
    if (n_layers < 0) return LD_ERR_RANGE;
    if (n_layers == 0) return LD_OK;
    if (!src || !dst || !n_elems) return LD_ERR_NULL;
    for (int32_t l = 0; l < n_layers; ++l) {
        if (n_elems[l] < 0) return LD_ERR_RANGE;
        if (n_elems[l] > 0 && (!src[l] || !dst[l])) return LD_ERR_NULL;
        if (!ld_aligned(src[l], 2) || !ld_aligned(dst[l], 2)) return LD_ERR_ALIGN;
        if ((n_elems[l] * 2 + kCopyBlockBytes - 1) / kCopyBlockBytes > (1 << 30)) return LD_ERR_RANGE;
    }
    ld_begin_call();
    int32_t l = 0;
    while (l < n_layers) {
        CopyBatch cb;
        cb.n = 0;
        int64_t blocks = 0;
        cb.first_block[0] = 0;
        while (l < n_layers && cb.n < kLayersPerLaunch) {
            const int64_t bytes = n_elems[l] * 2;
            const int64_t nb = (bytes + kCopyBlockBytes - 1) / kCopyBlockBytes;
            if (nb == 0) { ++l; continue; }
            if (blocks + nb > (1 << 30)) break;
            cb.job[cb.n] = CopyJob{static_cast<const unsigned char*>(src[l]),
                                   static_cast<unsigned char*>(dst[l]), bytes};
            blocks += nb;
            cb.first_block[++cb.n] = static_cast<int32_t>(blocks);
            ++l;
        }
        if (cb.n == 0) continue;
        for (int32_t j = cb.n; j < kLayersPerLaunch; ++j) {
            cb.job[j] = CopyJob{nullptr, nullptr, 0};
            cb.first_block[j + 1] = cb.first_block[cb.n];
        }
        k_snapshot_batch<<<dim3(static_cast<uint32_t>((blocks + 7) / 8 * 8)), dim3(kCopyThreads), 0,
                           static_cast<hipStream_t>(stream)>>>(cb);
        if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    }
    return LD_OK;
}

extern "C" ld_status ld_merge_dense_adam(float* w, float* m, float* v, int64_t n,
                                         const void* const* grads_bf16, int32_t W, int64_t step0,
                                         float lr, float beta1, float beta2, float eps,
                                         ld_stream stream) {
    if (n < 0 || W < 0 || W > LD_MAX_ADAM_WINDOW || step0 < 0) return LD_ERR_RANGE;
    if (!(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f)) return LD_ERR_RANGE;
    if (W == 0 || n == 0) return LD_OK;
    if (!w || !m || !v || !grads_bf16) return LD_ERR_NULL;
    if (!ld_aligned(w, 16) || !ld_aligned(m, 16) || !ld_aligned(v, 16)) return LD_ERR_ALIGN;
    static_assert(LD_MAX_ADAM_WINDOW <= LD_MAX_ADAM_STEPS, "step table too small");
    AdamArgs a;
    for (int32_t t = 0; t < LD_MAX_ADAM_WINDOW; ++t) a.grad[t] = nullptr;
    for (int32_t t = 0; t < W; ++t) {
        if (!grads_bf16[t]) return LD_ERR_NULL;
        if (!ld_aligned(grads_bf16[t], 16)) return LD_ERR_ALIGN;
        a.grad[t] = static_cast<const uint16_t*>(grads_bf16[t]);
    }
    ld_fill_adam_steps(a.s, W, step0, lr, beta1, beta2, eps);
    a.W = W;
    const int64_t blocks = (n + kAdamBlockElems - 1) / kAdamBlockElems;
    if (blocks > INT32_MAX - 8) return LD_ERR_RANGE;
    const dim3 grid(static_cast<uint32_t>((blocks + 7) / 8 * 8)), block(kAdamThreads);
    hipStream_t s = static_cast<hipStream_t>(stream);
    ld_begin_call();
    // steps are fused four (or eight) at a time; the state round-trips through fp32
    // memory between passes, which is exactly what it does between two calls
    const bool careful = ld_adam_careful(eps);
    int t0 = 0;
    while (t0 < W) {
        const int left = W - t0;
        if (careful) {
            if (left > 4) { k_adam<8, true><<<grid, block, 0, s>>>(w, m, v, n, a, t0); t0 += 8; }
            else if (left > 2) { k_adam<4, true><<<grid, block, 0, s>>>(w, m, v, n, a, t0); t0 += 4; }
            else if (left > 1) { k_adam<2, true><<<grid, block, 0, s>>>(w, m, v, n, a, t0); t0 += 2; }
            else { k_adam<1, true><<<grid, block, 0, s>>>(w, m, v, n, a, t0); t0 += 1; }
        } else {
            if (left > 4) { k_adam<8, false><<<grid, block, 0, s>>>(w, m, v, n, a, t0); t0 += 8; }
            else if (left > 2) { k_adam<4, false><<<grid, block, 0, s>>>(w, m, v, n, a, t0); t0 += 4; }
            else if (left > 1) { k_adam<2, false><<<grid, block, 0, s>>>(w, m, v, n, a, t0); t0 += 2; }
            else { k_adam<1, false><<<grid, block, 0, s>>>(w, m, v, n, a, t0); t0 += 1; }
        }
        if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    }
    return LD_OK;
}
