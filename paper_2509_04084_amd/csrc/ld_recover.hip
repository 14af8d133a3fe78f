// ld_merge_sparse_from_host: the recovery loop with its differentials still in host memory.
//
// Pipelined recovery module (Sec. VI-C) of the Recovery Process of Algorithm 1: while one
// differential checkpoint is being merged, the next ones are already being read. Here
// "read" is the copy of a group of diffs from page-locked host memory into a device
// staging buffer on one stream, "merge" is ld_merge_sparse of the previous group on
// another; two staging slots alternate. The diffs are applied in the order given, group
// after group, so the result is bit for bit that of one ld_merge_sparse call.
// No kernel of its own: stream and event orchestration around the merge.
#include "ld_common.h"

#define LD_HIP_OK(expr)                          \
    do {                                         \
        if ((expr) != hipSuccess) return LD_ERR_HIP; \
    } while (0)

namespace {

constexpr int kSlots = 2;
constexpr int kGroupLimit = 64;  // diffs per stage: their device addresses travel as one pointer table

// Bytes of one staging slot: the largest group's records (idx then val per diff, in 256-byte pieces).
size_t slot_bytes(const int64_t* K, int32_t W, int32_t group) {
    size_t most = 0;
    for (int32_t g0 = 0; g0 < W; g0 += group) {
        size_t need = 0;
        for (int32_t t = g0; t < W && t < g0 + group; ++t) need += 2 * ld_round_up(static_cast<size_t>(K[t]) * 4, 256);
        if (need > most) most = need;
    }
    return most;
}

struct Events {
    hipEvent_t copied[kSlots] = {nullptr, nullptr}, merged[kSlots] = {nullptr, nullptr};
    bool owned = false;
    // The caller's four events (copied[0], copied[1], merged[0], merged[1]), or events of the call's own.
    bool init(void* const* given) {
        if (given) {
            for (int i = 0; i < kSlots; ++i) {
                copied[i] = static_cast<hipEvent_t>(given[i]);
                merged[i] = static_cast<hipEvent_t>(given[kSlots + i]);
                if (!copied[i] || !merged[i]) return false;
            }
            return true;
        }
        owned = true;
        for (int i = 0; i < kSlots; ++i) {
            if (hipEventCreateWithFlags(&copied[i], hipEventDisableTiming) != hipSuccess) return false;
            if (hipEventCreateWithFlags(&merged[i], hipEventDisableTiming) != hipSuccess) return false;
        }
        return true;
    }
    ~Events() {  // an event that is still pending is released when it completes
        if (!owned) return;
        for (int i = 0; i < kSlots; ++i) {
            if (copied[i]) (void)hipEventDestroy(copied[i]);
            if (merged[i]) (void)hipEventDestroy(merged[i]);
        }
    }
};

}  // namespace

extern "C" size_t ld_merge_sparse_from_host_staging(const int64_t* K, int32_t W, int32_t group) {
    if (!K || W <= 0 || group <= 0 || group > kGroupLimit) return 0;
    for (int32_t t = 0; t < W; ++t)
        if (K[t] < 0) return 0;
    return kSlots * slot_bytes(K, W, group < W ? group : W);
}

extern "C" ld_status ld_merge_sparse_from_host_events(float* w, int64_t n, const int32_t* const* host_idx,
                                                      const float* const* host_val, const int64_t* K, int32_t W,
                                                      float lr, int32_t group, void* staging, size_t staging_bytes,
                                                      void* workspace, size_t workspace_bytes,
                                                      ld_stream copy_stream, ld_stream merge_stream,
                                                      void* const* events) {
    if (n < 0 || n > INT32_MAX || W < 0 || W > LD_MAX_WINDOW || group <= 0 || group > kGroupLimit)
        return LD_ERR_RANGE;
    if (W == 0 || n == 0) return LD_OK;
    if (!w || !host_idx || !host_val || !K) return LD_ERR_NULL;
    for (int32_t t = 0; t < W; ++t) {
        if (K[t] < 0 || K[t] > n) return LD_ERR_RANGE;
        if (K[t] > 0 && (!host_idx[t] || !host_val[t])) return LD_ERR_NULL;
    }
    if (group > W) group = W;
    const size_t slot = slot_bytes(K, W, group);
    if (slot == 0) return LD_OK;  // every diff is empty
    if (!staging || !ld_aligned(staging, 256) || staging_bytes < kSlots * slot) return LD_ERR_WORKSPACE;
    if (!workspace || !ld_aligned(workspace, 256) || workspace_bytes < ld_merge_sparse_workspace(n, group, K))
        return LD_ERR_WORKSPACE;
    hipStream_t cs = static_cast<hipStream_t>(copy_stream), ms = static_cast<hipStream_t>(merge_stream);
    Events ev;
    if (!ev.init(events)) return events ? LD_ERR_NULL : LD_ERR_HIP;

    int32_t stage = 0;
    for (int32_t g0 = 0; g0 < W; g0 += group, ++stage) {
        const int32_t gw = (W - g0) < group ? (W - g0) : group;
        const int s = stage % kSlots;
        char* base = static_cast<char*>(staging) + static_cast<size_t>(s) * slot;
        // the slot is free once the merge that read it two stages ago is done
        if (stage >= kSlots) LD_HIP_OK(hipStreamWaitEvent(cs, ev.merged[s], 0));
        const int32_t* di[kGroupLimit];
        const float* dv[kGroupLimit];
        size_t at = 0;
        for (int32_t j = 0; j < gw; ++j) {
            const int32_t t = g0 + j;
            const size_t bytes = static_cast<size_t>(K[t]) * 4;
            int32_t* pi = reinterpret_cast<int32_t*>(base + at);
            at += ld_round_up(bytes, 256);
            float* pv = reinterpret_cast<float*>(base + at);
            at += ld_round_up(bytes, 256);
            if (bytes) {
                LD_HIP_OK(hipMemcpyAsync(pi, host_idx[t], bytes, hipMemcpyHostToDevice, cs));
                LD_HIP_OK(hipMemcpyAsync(pv, host_val[t], bytes, hipMemcpyHostToDevice, cs));
            }
            di[j] = pi;
            dv[j] = pv;
        }
        LD_HIP_OK(hipEventRecord(ev.copied[s], cs));
        LD_HIP_OK(hipStreamWaitEvent(ms, ev.copied[s], 0));
        const ld_status st = ld_merge_sparse(w, n, di, dv, K + g0, gw, lr, workspace, workspace_bytes, ms);
        if (st != LD_OK) return st;
        LD_HIP_OK(hipEventRecord(ev.merged[s], ms));
    }
    return LD_OK;
}

extern "C" ld_status ld_merge_sparse_from_host(float* w, int64_t n, const int32_t* const* host_idx,
                                               const float* const* host_val, const int64_t* K, int32_t W,
                                               float lr, int32_t group, void* staging, size_t staging_bytes,
                                               void* workspace, size_t workspace_bytes, ld_stream copy_stream,
                                               ld_stream merge_stream) {
    return ld_merge_sparse_from_host_events(w, n, host_idx, host_val, K, W, lr, group, staging, staging_bytes,
                                            workspace, workspace_bytes, copy_stream, merge_stream, nullptr);
}
