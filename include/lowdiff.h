/*
 * lowdiff.h - C ABI of the MI355X (gfx950) LowDiff hot-path library.
 *
 * The library turns each training iteration's gradient into a differential
 * checkpoint and merges a window of such differentials onto a dense base
 * checkpoint.  The operations, all executed by hand-written HIP kernels:
 *
 *   ld_compress_topk     Comp of Algorithm 1 (Sec. IV-B): the compressed
 *                        gradient that LowDiff reuses as the differential
 *                        checkpoint C^D_t; sparsification at ratio rho
 *                        (Sec. II-C, Sec. VII-A).
 *   ld_merge_sparse      Recovery loop of Algorithm 1 / Eq. (6): load, decompress
 *                        and merge the diffs of a window strictly in iteration
 *                        order (Sec. IV-C, "Batched write semantics").
 *   ld_snapshot_layer    Snapshot(G^n_t) of Algorithm 2 (Sec. VI-B): copy one
 *                        layer's synchronized gradient out of the training
 *                        buffer as soon as it exists.
 *   ld_merge_dense_adam  "Merge in CPU" of Algorithm 2, M <- M + Adam(o_t, G_t)
 *                        (Eq. (4)): incremental merge of dense diffs into the
 *                        resident replica (kept in HBM here).
 *   ld_combine_sparse    Sync of Algorithm 1 (Eq. (3)) on all-gathered compressed
 *                        gradients: per-worker record lists added into one.
 *   ld_merge_sparse_adam Recovery loop of Algorithm 1 with the paper's own update:
 *                        sparse diffs decompressed and merged through Adam into
 *                        model and optimizer state.
 * and two helpers of the recovery path: ld_merge_sparse_from_host (the merge fed
 * from page-locked host memory, copies and merges pipelined) and ld_check_diff
 * (counts what is wrong with a diff before it is merged).
 *
 * General conventions
 *   - Pointers marked "dev" are device (HBM) addresses of the current HIP
 *     device; pointers marked "host" are ordinary host memory that the call
 *     reads completely before it returns.
 *   - Ownership: every buffer, workspaces included, is allocated, owned and
 *     freed by the caller.  The library allocates nothing and keeps no state
 *     between calls.
 *   - Asynchrony: a call only enqueues kernels on `stream` (a hipStream_t
 *     passed as void*; NULL is the default stream) and returns.  Results are
 *     ready when the stream reaches that point.  Calls on one stream execute
 *     in call order; that order is the iteration order of the diffs.
 *   - Errors: argument errors are found on the host before anything is
 *     enqueued; the call then returns a negative ld_status and touches no
 *     buffer.  Data-dependent preconditions (indices in range and strictly
 *     ascending inside a diff, no NaN among the values) are the caller's
 *     contract and are not checked.
 *   - Alignment: dev pointers to fp32 / int32 arrays must be 16-byte aligned
 *     unless stated otherwise (LD_ERR_ALIGN).
 *   - Inputs declared const are never written.
 */
#ifndef LOWDIFF_H_
#define LOWDIFF_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t ld_status;
typedef void*   ld_stream; /* hipStream_t */

#define LD_OK             0
#define LD_ERR_NULL      -1 /* a required pointer is NULL                          */
#define LD_ERR_RANGE     -2 /* a size, count or table entry is out of range        */
#define LD_ERR_WORKSPACE -3 /* workspace missing, misaligned or too small          */
#define LD_ERR_HIP       -4 /* a HIP runtime call or kernel launch failed          */
#define LD_ERR_ALIGN     -5 /* a device pointer is not aligned as required         */

/* Largest window one ld_merge_* call accepts. */
#define LD_MAX_WINDOW 4096

/* Human-readable name of a status code; never NULL; static storage. */
const char* ld_status_string(ld_status s);

/* ------------------------------------------------------------------------
 * ld_compress_topk - per-segment top-k sparsification with error feedback.
 *
 * For every segment s = [seg_off[s], seg_off[s+1]) of the flat gradient:
 *   a_i   = fl32(residual_i + grad_i)                (one IEEE add, RNE)
 *   order : i before j  iff  |a_i| > |a_j|, or |a_i| == |a_j| and i < j
 *           (|.| compared on the binary32 bit pattern with the sign cleared,
 *            so +0 and -0 tie, and denormals are not flushed)
 *   S     = the first seg_k[s] positions of that order
 *   emit  : for i in S ascending: out_idx = i (global flat index),
 *           out_val = a_i bit for bit; segment s's records start at
 *           sum_{s'<s} seg_k[s']; the whole diff is strictly ascending in idx
 *   residual_i <- +0.0f for i in S, a_i otherwise
 * The result is unique (the order is total); it does not depend on launch
 * shape or timing.
 *
 *   grad       dev  [n] fp32, read only, n = seg_off[n_seg] <= 2^31-1
 *   residual   dev  [n] fp32, in/out
 *   seg_off    host [n_seg+1] int64, seg_off[0] = 0, non-decreasing
 *   seg_k      host [n_seg] int32, 0 <= seg_k[s] <= n_s
 *   out_idx    dev  [K] int32, K = sum seg_k
 *   out_val    dev  [K] fp32
 *   workspace  dev, 256-byte aligned, at least ld_compress_topk_workspace()
 *              bytes; contents on entry are irrelevant, contents on exit are
 *              unspecified. That minimum serves densities seg_k[s]/n_s up to
 *              about 1 % at full speed; the results are the same at any
 *              density, but denser calls run faster with the
 *              ld_compress_topk_workspace_for() size of their seg_k (the call
 *              uses as much of a larger workspace as its densities ask for)
 * Errors: LD_ERR_NULL, LD_ERR_RANGE (bad table, n > 2^31-1), LD_ERR_ALIGN,
 * LD_ERR_WORKSPACE, LD_ERR_HIP.
 */
size_t    ld_compress_topk_workspace(int32_t n_seg, const int64_t* seg_off /* host */);
size_t    ld_compress_topk_workspace_for(int32_t n_seg, const int64_t* seg_off /* host */,
                                         const int32_t* seg_k /* host */);
ld_status ld_compress_topk(const float* grad, float* residual,
                           const int64_t* seg_off, const int32_t* seg_k, int32_t n_seg,
                           int32_t* out_idx, float* out_val,
                           void* workspace, size_t workspace_bytes, ld_stream stream);

/* Same operation with the selection strategy chosen by the caller (a tuning and
 * test hook; the result is identical for every strategy):
 *   LD_COMPRESS_AUTO  one streaming pass; a per-segment candidate threshold is
 *                     estimated from a sample, the exact top-k is then resolved
 *                     among the candidates (segments whose estimate turns out
 *                     too high are redone by the FULL method)
 *   LD_COMPRESS_FULL  no estimate: multi-pass radix select over whole segments
 */
#define LD_COMPRESS_AUTO 0
#define LD_COMPRESS_FULL 1
ld_status ld_compress_topk_strategy(const float* grad, float* residual,
                                    const int64_t* seg_off, const int32_t* seg_k, int32_t n_seg,
                                    int32_t* out_idx, float* out_val,
                                    void* workspace, size_t workspace_bytes, ld_stream stream,
                                    int32_t strategy);

/* Which way the last ld_compress_topk call on `workspace` went, segment by segment (a test and
 * diagnosis hook: the result of a call never depends on it).  Enqueues one small kernel on
 * `stream`, after which
 *   paths[s] & 0xFF     LD_PATH_CANDIDATES: the top-k was resolved among the sampled-threshold
 *                       candidates; LD_PATH_TIES: same, the threshold being a massively repeated
 *                       key whose ties were taken in index order; LD_PATH_FULL: the segment was
 *                       redone by the radix select over all its elements
 *   paths[s] & 0x100    the sample of the segment held one key so often that the candidates were
 *                       taken above it
 *   paths[s] & 0x10000  the full-segment pass gave up waiting at its grid barrier (its workgroups
 *                       were never all resident: more compress calls in flight on one GPU than
 *                       it holds); the outputs of that call are not valid
 *   overflowed_tiles[s] 4096-element tiles of the segment with more candidates than a slot holds
 *                       (they were read back from the residual); may be NULL
 *
 *   workspace  dev, the workspace of that call, unchanged since
 *   n_seg, seg_off      the segment table of that call (host)
 *   paths, overflowed_tiles  dev [n_seg] int32
 * Errors: LD_ERR_NULL, LD_ERR_RANGE, LD_ERR_ALIGN, LD_ERR_WORKSPACE, LD_ERR_HIP.
 */
#define LD_PATH_CANDIDATES 0
#define LD_PATH_FULL       1
#define LD_PATH_TIES       2
ld_status ld_compress_topk_paths(const void* workspace, size_t workspace_bytes, int32_t n_seg,
                                 const int64_t* seg_off /* host */, int32_t* paths,
                                 int32_t* overflowed_tiles, ld_stream stream);

/* ------------------------------------------------------------------------
 * ld_snapshot_layer - bit-exact copy of one layer's bf16 gradient into a
 * checkpoint-owned buffer, so training may overwrite its gradient buffer.
 *
 *   grad_bf16  dev [n_elems] 16-bit elements, read only (2-byte aligned is enough)
 *   snap_bf16  dev [n_elems] destination; must not overlap the source
 *   n_elems    >= 0 (0 enqueues nothing)
 * Errors: LD_ERR_NULL, LD_ERR_RANGE (n_elems < 0), LD_ERR_ALIGN (odd address),
 * LD_ERR_HIP.
 */
ld_status ld_snapshot_layer(const void* grad_bf16, void* snap_bf16, int64_t n_elems,
                            ld_stream stream);

/* Same copy for many layers in one launch (small layers packed into one grid;
 * the chunking/packing remark of Sec. VI-C "Snapshotting module").
 *   src, dst  host arrays of n_layers dev pointers;  n_elems host [n_layers]
 */
ld_status ld_snapshot_layers(const void* const* src, void* const* dst, const int64_t* n_elems,
                             int32_t n_layers, ld_stream stream);

/* ------------------------------------------------------------------------
 * ld_merge_sparse - replay a window of W sparse diffs onto w, in order:
 *   for t = 0..W-1, for every record j of diff t:
 *       p = fl32(lr * val[t][j]);  w[idx[t][j]] = fl32(w[idx[t][j]] - p)
 * (two roundings, never a fused multiply-add).  One call with W diffs gives
 * bit for bit the result of W calls with one diff each.
 *
 *   w          dev  [n] fp32 in/out, n <= 2^31-1
 *   idx, val   host arrays of W dev pointers; idx[t] int32[K[t]] strictly
 *              ascending and in [0, n); val[t] fp32[K[t]]
 *   K          host [W] int64, 0 <= K[t] <= n
 *   W          0 <= W <= LD_MAX_WINDOW (0 enqueues nothing)
 *   workspace  dev, 256-byte aligned, ld_merge_sparse_workspace() bytes. With K = NULL
 *              the query gives the minimum (the call fails with less); with K it
 *              gives what the window's shape asks for, which is more for long windows
 *              of very sparse diffs (they then run a lane per diff instead of as
 *              ordinary sweeps; same result, less time)
 * Errors: LD_ERR_NULL, LD_ERR_RANGE, LD_ERR_ALIGN, LD_ERR_WORKSPACE, LD_ERR_HIP.
 */
size_t    ld_merge_sparse_workspace(int64_t n, int32_t W, const int64_t* K /* host, or NULL */);
ld_status ld_merge_sparse(float* w, int64_t n,
                          const int32_t* const* idx, const float* const* val,
                          const int64_t* K, int32_t W, float lr,
                          void* workspace, size_t workspace_bytes, ld_stream stream);

/* ------------------------------------------------------------------------
 * ld_merge_sparse_from_host - ld_merge_sparse for diffs that still lie in host
 * memory, pipelined (pipelined recovery module, Sec. VI-C: while one
 * differential checkpoint is merged the next ones are already being read).
 * The diffs are copied to the device in groups of `group` on copy_stream and
 * each group is merged on merge_stream while the next one is copied; two
 * staging slots alternate.  The result is bit for bit that of one
 * ld_merge_sparse call with the same diffs in the same order.
 *
 *   host_idx, host_val  host arrays of W HOST pointers (int32[K[t]], fp32[K[t]]);
 *              page-locked memory for the copies to overlap; they must stay
 *              valid and unchanged until copy_stream has passed the call
 *   group      1 <= group <= 64: diffs per stage (a larger group means fewer
 *              passes over w and a longer wait before the first merge)
 *   staging    dev, 256-byte aligned, ld_merge_sparse_from_host_staging() bytes
 *   workspace  dev, 256-byte aligned, ld_merge_sparse_workspace(n, group, K) bytes
 *   copy_stream, merge_stream  may be the same stream (then nothing overlaps).
 *              w is ready when merge_stream has passed the call.
 * The call creates and destroys four HIP events (it allocates no device memory), so
 * it cannot be recorded into a HIP graph; ld_merge_sparse_from_host_events takes the
 * four events from the caller instead and then only enqueues copies, kernels, event
 * records and stream waits:
 *   events     host array of 4 hipEvent_t the caller created (timing may be disabled)
 *              and does not use for anything else while the call's work is pending;
 *              NULL: as ld_merge_sparse_from_host
 * Unlike the other entry points, this one can fail part-way: argument errors are
 * found before anything is enqueued, but when a HIP call fails in the loop over the
 * groups (LD_ERR_HIP) the earlier groups have been enqueued and will be merged into
 * w; w then holds base + the first whole groups and must be rebuilt from the base
 * checkpoint.
 * Errors: LD_ERR_NULL, LD_ERR_RANGE, LD_ERR_ALIGN, LD_ERR_WORKSPACE, LD_ERR_HIP.
 */
size_t    ld_merge_sparse_from_host_staging(const int64_t* K /* host */, int32_t W, int32_t group);
ld_status ld_merge_sparse_from_host(float* w, int64_t n,
                                    const int32_t* const* host_idx, const float* const* host_val,
                                    const int64_t* K, int32_t W, float lr, int32_t group,
                                    void* staging, size_t staging_bytes,
                                    void* workspace, size_t workspace_bytes,
                                    ld_stream copy_stream, ld_stream merge_stream);
ld_status ld_merge_sparse_from_host_events(float* w, int64_t n,
                                           const int32_t* const* host_idx, const float* const* host_val,
                                           const int64_t* K, int32_t W, float lr, int32_t group,
                                           void* staging, size_t staging_bytes,
                                           void* workspace, size_t workspace_bytes,
                                           ld_stream copy_stream, ld_stream merge_stream,
                                           void* const* events /* host, 4 hipEvent_t, or NULL */);

/* ------------------------------------------------------------------------
 * ld_check_diff - does a differential that was read back from storage meet
 * what the merges take for granted?  (Recovery loop of Algorithm 1, Sec. IV-B:
 * differentials are loaded from storage and then merged.)  Counts, over the K
 * records of one diff,
 *   counts[0]  indices outside [0, n)
 *   counts[1]  records j >= 1 with idx[j] <= idx[j-1]   (not strictly ascending)
 *   counts[2]  values that are NaN                      (0 when val is NULL)
 * All zero: the diff may be passed to ld_merge_sparse / ld_merge_sparse_adam /
 * ld_combine_sparse.  Anything else: those calls would skip records or, with
 * the scatter strategy, write outside w.
 *
 *   idx     dev [K] int32, 4-byte aligned
 *   val     dev [K] fp32 or NULL, 4-byte aligned
 *   n       0 <= n <= 2^31-1
 *   counts  dev [3] int64, 8-byte aligned; overwritten (zeroed on the stream
 *           first, so the same buffer can be reused call after call)
 * Errors: LD_ERR_NULL, LD_ERR_RANGE, LD_ERR_ALIGN, LD_ERR_HIP.
 */
ld_status ld_check_diff(const int32_t* idx, const float* val, int64_t K, int64_t n,
                        int64_t* counts, ld_stream stream);

/* Same operation with the execution strategy chosen by the caller (a tuning and
 * test hook; the result is identical for every strategy):
 *   LD_MERGE_AUTO     library decides from n and sum K
 *   LD_MERGE_SWEEP    one streaming pass over w consuming all W diffs per tile
 *   LD_MERGE_SCATTER  W scatter kernels, one per diff, in order
 */
#define LD_MERGE_AUTO    0
#define LD_MERGE_SWEEP   1
#define LD_MERGE_SCATTER 2
ld_status ld_merge_sparse_strategy(float* w, int64_t n,
                                   const int32_t* const* idx, const float* const* val,
                                   const int64_t* K, int32_t W, float lr,
                                   void* workspace, size_t workspace_bytes, ld_stream stream,
                                   int32_t strategy);

/* ------------------------------------------------------------------------
 * ld_merge_sparse_static - ld_merge_sparse for callers that cannot allocate:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same operation, same results bit for bit, no workspace argument:
 * the chunk table (the merge's only scratch memory) lies in a device array that
 * is part of the library image, LD_MERGE_STATIC_SCRATCH bytes per GPU, held
 * until the process ends.  The call allocates and frees nothing and calls no
 * allocating routine; the first call on a device looks up that device's copy
 * of the array (hipGetSymbolAddress), later calls only enqueue kernels.
 *
 *   w, n, idx, val, K, W, lr   as for ld_merge_sparse
 * Limit: ld_merge_sparse_workspace(n, W, NULL) <= ld_merge_sparse_static_limit()
 * (= LD_MERGE_STATIC_SCRATCH; a window of up to 128 diffs over about 400 M
 * elements, or 20 diffs over the full 2^31-1); larger calls are refused with
 * LD_ERR_WORKSPACE before anything is enqueued.
 * Every call on a GPU shares that GPU's array: calls that overlap in time on one
 * GPU (different streams, or threads) race on it and must be serialized by the
 * caller.  Nothing in the array has to start at zero, and what a call leaves in
 * it is never read by a later one.
 * Errors: LD_ERR_NULL, LD_ERR_RANGE, LD_ERR_ALIGN, LD_ERR_WORKSPACE (over the
 * limit), LD_ERR_HIP.
 */
#define LD_MERGE_STATIC_SCRATCH (4u << 20)
size_t    ld_merge_sparse_static_limit(void);
ld_status ld_merge_sparse_static(float* w, int64_t n,
                                 const int32_t* const* idx, const float* const* val,
                                 const int64_t* K, int32_t W, float lr, ld_stream stream);

/* ------------------------------------------------------------------------
 * ld_merge_dense_adam - replay W dense bf16 gradients through Adam onto the
 * fp32 replica (w, m, v): for s = step0+1 .. step0+W with g = widen(grad_s),
 *   m <- beta1*m + (1-beta1)*g
 *   v <- beta2*v + (1-beta2)*g*g
 *   w <- w - lr * (m / (1-beta1^s)) / (sqrt(v / (1-beta2^s)) + eps)
 * in fp32 (bias-correction factors prepared on the host in double).  No weight
 * decay, no AMSGrad.  A call with W gradients gives bit for bit the result of
 * W calls with one gradient each.
 *
 *   w, m, v     dev  [n] fp32 in/out (n may exceed 2^32)
 *   grads_bf16  host array of W dev pointers to bf16[n], 16-byte aligned
 *   W           0 <= W <= 64
 *   step0       >= 0, optimizer steps already contained in (w, m, v)
 * Errors: LD_ERR_NULL, LD_ERR_RANGE, LD_ERR_ALIGN, LD_ERR_HIP.
 */
#define LD_MAX_ADAM_WINDOW 64
ld_status ld_merge_dense_adam(float* w, float* m, float* v, int64_t n,
                              const void* const* grads_bf16, int32_t W, int64_t step0,
                              float lr, float beta1, float beta2, float eps, ld_stream stream);

/* ------------------------------------------------------------------------
 * ld_merge_sparse_adam - replay a window of W sparse diffs through Adam onto
 * (w, m, v): the Recovery loop of Algorithm 1 (Sec. IV-B) with the update the
 * paper names there - decompress diff j (Comp^-1), then M_{j+1} = M_j + Adam(G_j)
 * (Eq. (4)) on the model and the optimizer state.  For t = 0..W-1, step
 * s = step0+1+t, with g_i = val[t][j] where idx[t][j] = i and g_i = 0 elsewhere:
 *   m <- beta1*m + (1-beta1)*g
 *   v <- beta2*v + (1-beta2)*g*g
 *   w <- w - lr * (m / (1-beta1^s)) / (sqrt(v / (1-beta2^s)) + eps)
 * for EVERY element i (a zero gradient still decays m and v and moves w), in
 * fp32, the same arithmetic as ld_merge_dense_adam.  One call with W diffs gives
 * bit for bit the result of W calls with one diff each.
 *
 *   w, m, v    dev  [n] fp32 in/out, n <= 2^31-1
 *   idx, val   host arrays of W dev pointers; idx[t] int32[K[t]] strictly
 *              ascending and in [0, n); val[t] fp32[K[t]]
 *   K          host [W] int64, 0 <= K[t] <= n
 *   W          0 <= W <= LD_MAX_WINDOW (0 enqueues nothing)
 *   step0      >= 0, optimizer steps already contained in (w, m, v)
 *   workspace  dev, 256-byte aligned, ld_merge_sparse_adam_workspace() bytes
 * Errors: LD_ERR_NULL, LD_ERR_RANGE, LD_ERR_ALIGN, LD_ERR_WORKSPACE, LD_ERR_HIP.
 */
size_t    ld_merge_sparse_adam_workspace(int64_t n, int32_t W, const int64_t* K /* host */);
ld_status ld_merge_sparse_adam(float* w, float* m, float* v, int64_t n,
                               const int32_t* const* idx, const float* const* val,
                               const int64_t* K, int32_t W, int64_t step0,
                               float lr, float beta1, float beta2, float eps,
                               void* workspace, size_t workspace_bytes, ld_stream stream);

/* ------------------------------------------------------------------------
 * ld_combine_sparse - N per-worker record lists combined into one: Sync of
 * Algorithm 1 (Sec. IV-B; Eq. (3)) applied to compressed gradients as an
 * all-gather leaves them on every rank.  The output holds, ascending in index,
 * every index recorded by at least one worker, with
 *     out_val = fl32(scale * (((+0 + v_r1) + v_r2) + ...))
 * over the workers r1 < r2 < ... that recorded it - one fp32 add each, in worker
 * order (scale = 1: sum; 1/N: mean; the paper does not say which).  An index whose
 * values cancel to zero is still emitted.
 *
 *   idx, val   host arrays of N dev pointers; idx[r] int32[K[r]] strictly
 *              ascending and in [0, n); val[r] fp32[K[r]]
 *   K          host [N] int64, 0 <= K[r] <= n
 *   N          0 <= N <= LD_MAX_WORKERS
 *   n          size of the index space, <= 2^31-1
 *   out_idx, out_val  dev [out_cap]; records beyond out_cap are not written
 *              (sum K always suffices)
 *   out_count  dev int64, 8-byte aligned: the number of distinct indices (compare
 *              with out_cap to detect a truncated output)
 *   workspace  dev, 256-byte aligned, ld_combine_sparse_workspace() bytes (about
 *              n / 8: a bit per index, plus small tables)
 * Errors: LD_ERR_NULL, LD_ERR_RANGE, LD_ERR_ALIGN, LD_ERR_WORKSPACE, LD_ERR_HIP.
 */
#define LD_MAX_WORKERS 64
size_t    ld_combine_sparse_workspace(int64_t n, int32_t N);
ld_status ld_combine_sparse(const int32_t* const* idx, const float* const* val, const int64_t* K,
                            int32_t N, int64_t n, float scale,
                            int32_t* out_idx, float* out_val, int64_t out_cap, int64_t* out_count,
                            void* workspace, size_t workspace_bytes, ld_stream stream);

/* ------------------------------------------------------------------------
 * Checkpointing configuration model (Sec. V-C).  Host arithmetic only; nothing is
 * enqueued.  f = full-checkpoint interval in iterations, b = differentials per
 * batched checkpoint, 1 <= b <= f.
 *
 *   ld_config_wasted_time        T_w(f, b), Eq. (10):
 *       (N T / M) [ b tau / 2 + R_F + (R_B / 2)(f/b - 1) ] + (N T / (f tau)) [ C_F + C_B (f/b - 1) ]
 *   ld_config_critical_interval  f_c(b) = sqrt( 2 M b (C_F - C_B) / (tau R_B) ), Eq. (11)
 *   ld_config_select             Eq. (12): index of the candidate (f[i], b[i]) with the smallest
 *                                T_w, R_B[i] and C_B[i] being the costs measured for b[i];
 *                                wasted (optional, [n_cand]) receives every T_w
 * R_B: recovery time of one batched differential (read + decompress + replay of b diffs),
 * C_B: its write cost (Eqs. (8), (9)); all times in one unit (seconds).
 * Invalid arguments give NaN (the first two) or -1 (select); candidates whose T_w is NaN
 * are skipped.
 */
typedef struct ld_config_params {
    double N;    /* GPUs                                   */
    double T;    /* failure-free training duration         */
    double M;    /* mean time between failures             */
    double tau;  /* average iteration time                 */
    double R_F;  /* time to restore one full checkpoint    */
    double C_F;  /* time to write one full checkpoint      */
} ld_config_params;
double  ld_config_wasted_time(const ld_config_params* p, double f, double b, double R_B, double C_B);
double  ld_config_critical_interval(const ld_config_params* p, double b, double R_B, double C_B);
int32_t ld_config_select(const ld_config_params* p, int32_t n_cand, const int32_t* f, const int32_t* b,
                         const double* R_B, const double* C_B, double* wasted /* may be NULL */);

#ifdef __cplusplus
}
#endif
#endif /* LOWDIFF_H_ */
