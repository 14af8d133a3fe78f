// ld_check_diff: does a differential read back from storage meet what the merges assume?
//
// The Recovery loop of Algorithm 1 (Sec. IV-B) loads differential checkpoints from storage
// and merges them. The merge kernels take for granted that a diff's indices lie in [0, n) and
// ascend strictly, and that no value is a NaN; a damaged file breaks that silently (the sweep
// would skip records, the scatter would write outside w). This pass counts the violations so
// that a caller can refuse the file before merging it. One read of the records, 8 bytes each.
#include "ld_common.h"

namespace {

constexpr int kCheckThreads = 256;
constexpr int kCheckPer = 8;  // records per thread

__global__ void k_check_zero(unsigned long long* out) {
    if (threadIdx.x < 3) out[threadIdx.x] = 0;
}

__global__ __launch_bounds__(kCheckThreads) void k_check_diff(const int32_t* __restrict__ idx,
                                                              const float* __restrict__ val, int64_t K, int64_t n,
                                                              unsigned long long* __restrict__ out) {
    __shared__ uint32_t part[3][kCheckThreads / LD_WAVE];
    uint32_t range = 0, order = 0, nan = 0;
    const int64_t base = static_cast<int64_t>(blockIdx.x) * (kCheckThreads * kCheckPer);
#pragma unroll
    for (int u = 0; u < kCheckPer; ++u) {
        const int64_t j = base + u * kCheckThreads + threadIdx.x;
        if (j < K) {
            const int32_t i = idx[j];
            range += i < 0 || i >= n;
            if (j > 0) order += i <= idx[j - 1];
            if (val) {
                const float v = val[j];
                nan += v != v;
            }
        }
    }
    range = ld_wave_sum(range);
    order = ld_wave_sum(order);
    nan = ld_wave_sum(nan);
    const int w = threadIdx.x >> 6;
    if (ld_lane() == 0) {
        part[0][w] = range;
        part[1][w] = order;
        part[2][w] = nan;
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        uint32_t total = 0;
        for (int q = 0; q < kCheckThreads / LD_WAVE; ++q) total += part[threadIdx.x][q];
        if (total) atomicAdd(out + threadIdx.x, static_cast<unsigned long long>(total));
    }
}

}  // namespace

extern "C" ld_status ld_check_diff(const int32_t* idx, const float* val, int64_t K, int64_t n, int64_t* counts,
                                   ld_stream stream) {
    if (K < 0 || n < 0 || n > INT32_MAX) return LD_ERR_RANGE;
    if (!counts) return LD_ERR_NULL;
    if (K > 0 && !idx) return LD_ERR_NULL;
    if (!ld_aligned(idx, 4) || !ld_aligned(val, 4) || !ld_aligned(counts, 8)) return LD_ERR_ALIGN;
    const int64_t blocks = (K + kCheckThreads * kCheckPer - 1) / (kCheckThreads * kCheckPer);
    if (blocks > INT32_MAX) return LD_ERR_RANGE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    ld_begin_call();
    unsigned long long* out = reinterpret_cast<unsigned long long*>(counts);
    k_check_zero<<<dim3(1), dim3(LD_WAVE), 0, s>>>(out);
    if (ld_launch_status() != LD_OK) return LD_ERR_HIP;
    if (K == 0) return LD_OK;
    k_check_diff<<<dim3(static_cast<uint32_t>(blocks)), dim3(kCheckThreads), 0, s>>>(idx, val, K, n, out);
    return ld_launch_status();
}
