// LowDiff / LowDiff+ CPU oracle.  TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, obviously-correct statement of what the differential-checkpoint
// hot path computes.  It exists so that tests, the smoke check and the
// benchmark's cpu_baseline leg have something independent to compare the GPU
// library against.  Nothing in the product path may include, link or call it,
// and it shares no code, header, table or helper with the HIP sources.
//
// Build: g++ -O2 -std=c++17 -ffp-contract=off -fPIC -shared  (no -ffast-math:
// every float operation below is one IEEE-754 binary32 operation, round to
// nearest even, and denormals are kept).
//
// What each function follows:
//   oracle_topk_ef / oracle_topk_select : the Comp step of Algorithm 1 (Sec. IV-B,
//       "Compress"), read as exact per-segment top-k by magnitude with an
//       error-feedback residual.  The paper only says "sparsification ... selects
//       a subset of the elements" (Sec. II-C) at ratio rho (Sec. VII-A); the
//       precise rule (accumulate r+g, order by |a| then lower index, emit
//       ascending (idx,val), zero the selected residuals) is the reading fixed
//       for this build.
//   oracle_merge_sparse : the Recovery loop of Algorithm 1 (load diff j,
//       decompress, merge, for j in iteration order) and Eq. (6), with the
//       update rule w[idx] -= lr*val.  Batched diffs are replayed one after
//       another, never summed first (Sec. IV-C "Batched write semantics").
//   oracle_snapshot : Snapshot(G^n_t) of Algorithm 2 - a bit copy of one layer.
//   oracle_adam_replay : "Merge in CPU" of Algorithm 2, M <- M + Adam(o_t, G_t)
//       (Eq. (4)), with the textbook bias-corrected Adam of Kingma & Ba.
//   oracle_wasted_time / oracle_critical_interval : the configuration model of
//       Sec. V-C, Eqs. (8)-(12), written term by term.
//   oracle_combine_sparse : Sync of Algorithm 1 / Eq. (3) on the all-gathered
//       per-worker record lists: values at equal indices added in worker order.
//   oracle_check_diff : what the Recovery loop of Algorithm 1 takes for granted about a
//       differential it has loaded from storage (indices in range, strictly ascending,
//       values that are numbers), counted record by record.
//   oracle_sparse_adam_replay : the Recovery loop of Algorithm 1 with the update
//       the paper itself names there (decompress, then Adam on model and optimizer
//       state), for diffs that are sparse.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

inline uint32_t abs_bits(float a) {
    uint32_t u;
    std::memcpy(&u, &a, sizeof u);
    return u & 0x7FFFFFFFu;  // |a| as an integer: monotone in |a| for non-NaN
}

struct KeyPos {
    uint32_t key;
    int64_t pos;  // position inside the segment
};

// The total order of the selection: larger magnitude first, then lower index.
inline bool precedes(const KeyPos& x, const KeyPos& y) {
    if (x.key != y.key) return x.key > y.key;
    return x.pos < y.pos;
}

// Steps shared by the two top-k variants (they differ only in how the first k
// elements of the total order are found: full sort, or nth_element).
template <bool kFullSort>
int topk_ef(const float* g, float* r, const int64_t* seg_off, const int32_t* seg_k,
            int32_t n_seg, int32_t* out_idx, float* out_val) {
    int64_t out_base = 0;
    for (int32_t s = 0; s < n_seg; ++s) {
        const int64_t o = seg_off[s];
        const int64_t ns = seg_off[s + 1] - o;
        const int64_t k = seg_k[s];
        if (ns < 0 || k < 0 || k > ns) return -1;
        // 1. accumulate: a_i = fl32(r_i + g_i), kept in r.
        for (int64_t i = 0; i < ns; ++i) r[o + i] = r[o + i] + g[o + i];
        // 2.-4. the k first positions under the total order.
        std::vector<KeyPos> e(static_cast<size_t>(ns));
        for (int64_t i = 0; i < ns; ++i) e[i] = KeyPos{abs_bits(r[o + i]), i};
        if (kFullSort) {
            std::sort(e.begin(), e.end(), precedes);
        } else if (k > 0 && k < ns) {
            std::nth_element(e.begin(), e.begin() + (k - 1), e.end(), precedes);
        }
        // 5. emit the selected set in ascending index order.
        std::vector<int64_t> sel(static_cast<size_t>(k));
        for (int64_t j = 0; j < k; ++j) sel[j] = e[j].pos;
        std::sort(sel.begin(), sel.end());
        for (int64_t j = 0; j < k; ++j) {
            const int64_t gi = o + sel[j];
            if (gi > INT32_MAX) return -2;
            out_idx[out_base + j] = static_cast<int32_t>(gi);
            out_val[out_base + j] = r[gi];  // a_i bit for bit
        }
        // 6. selected positions leave nothing behind.
        for (int64_t j = 0; j < k; ++j) r[o + sel[j]] = 0.0f;
        out_base += k;
    }
    return 0;
}

inline float bf16_to_f32(uint16_t h) {
    uint32_t u = static_cast<uint32_t>(h) << 16;  // exact widening
    float f;
    std::memcpy(&f, &u, sizeof f);
    return f;
}

}  // namespace

extern "C" {

// Per-segment top-k with error feedback, by full sort (the definition).
//   g        [n]  gradient, read only
//   r        [n]  residual, in/out
//   seg_off  [n_seg+1] segment boundaries, seg_off[0]=0
//   seg_k    [n_seg]   records to keep per segment, 0 <= k_s <= n_s
//   out_idx  [sum k_s] global flat index, ascending
//   out_val  [sum k_s] accumulated value at that index
// Returns 0, or <0 on a malformed segment table.
int oracle_topk_ef(const float* g, float* r, const int64_t* seg_off, const int32_t* seg_k,
                   int32_t n_seg, int32_t* out_idx, float* out_val) {
    return topk_ef<true>(g, r, seg_off, seg_k, n_seg, out_idx, out_val);
}

// Same result through std::nth_element with the identical comparator; used
// where a full sort of >1e8 elements would take minutes.
int oracle_topk_select(const float* g, float* r, const int64_t* seg_off, const int32_t* seg_k,
                       int32_t n_seg, int32_t* out_idx, float* out_val) {
    return topk_ef<false>(g, r, seg_off, seg_k, n_seg, out_idx, out_val);
}

// Replay W sparse diffs onto w in iteration order: for every record,
// p = fl32(lr*val); w[idx] = fl32(w[idx] - p).  Two roundings, no fused
// multiply-add (the build forbids contraction).
int oracle_merge_sparse(float* w, int64_t n, const int32_t* const* idx, const float* const* val,
                        const int64_t* K, int32_t W, float lr) {
    for (int32_t t = 0; t < W; ++t) {
        for (int64_t j = 0; j < K[t]; ++j) {
            const int64_t i = idx[t][j];
            if (i < 0 || i >= n) return -1;
            const float p = lr * val[t][j];
            w[i] = w[i] - p;
        }
    }
    return 0;
}

// Layer snapshot: bit copy of n bf16 elements.
void oracle_snapshot(const uint16_t* src, uint16_t* dst, int64_t n) {
    std::memcpy(dst, src, static_cast<size_t>(n) * sizeof(uint16_t));
}

// Replay W dense bf16 gradients through Adam onto fp32 (w, m, v).
// Steps step0+1 .. step0+W.  Arithmetic in double; each stored quantity is
// rounded to fp32 once per step, and the parameter update of a step uses the
// moments as stored by that step.  No weight decay, no AMSGrad; eps is added
// to the square root of the bias-corrected second moment.
void oracle_adam_replay(float* w, float* m, float* v, int64_t n, const uint16_t* const* grads,
                        int32_t W, int64_t step0, float lr, float beta1, float beta2, float eps) {
    const double b1 = beta1, b2 = beta2, lrd = lr, epsd = eps;
    for (int32_t t = 0; t < W; ++t) {
        const double s = static_cast<double>(step0 + 1 + t);
        const double bc1 = 1.0 - std::pow(b1, s);
        const double bc2 = 1.0 - std::pow(b2, s);
        const uint16_t* gt = grads[t];
        for (int64_t i = 0; i < n; ++i) {
            const double g = bf16_to_f32(gt[i]);
            const float mf = static_cast<float>(b1 * m[i] + (1.0 - b1) * g);
            const float vf = static_cast<float>(b2 * v[i] + (1.0 - b2) * g * g);
            m[i] = mf;
            v[i] = vf;
            const double mhat = static_cast<double>(mf) / bc1;
            const double vhat = static_cast<double>(vf) / bc2;
            w[i] = static_cast<float>(static_cast<double>(w[i]) - lrd * mhat / (std::sqrt(vhat) + epsd));
        }
    }
}

// Replay W sparse diffs through Adam onto fp32 (w, m, v): the recovery loop of
// Algorithm 1 as the paper states it, M_{j+1} = M_j + Adam(G_j), where G_j is the
// decompressed diff j - a dense gradient that is val at the recorded positions and
// zero everywhere else.  Every element takes every step (a zero gradient still
// decays m and v and moves w while m is non-zero).  Steps step0+1 .. step0+W;
// arithmetic as in oracle_adam_replay.  Returns 0, or -1 on an index out of range.
int oracle_sparse_adam_replay(float* w, float* m, float* v, int64_t n, const int32_t* const* idx,
                              const float* const* val, const int64_t* K, int32_t W, int64_t step0,
                              float lr, float beta1, float beta2, float eps) {
    const double b1 = beta1, b2 = beta2, lrd = lr, epsd = eps;
    std::vector<float> g(static_cast<size_t>(n));
    for (int32_t t = 0; t < W; ++t) {
        // Comp^-1: decompress diff t into a dense gradient
        std::fill(g.begin(), g.end(), 0.0f);
        for (int64_t j = 0; j < K[t]; ++j) {
            const int64_t i = idx[t][j];
            if (i < 0 || i >= n) return -1;
            g[static_cast<size_t>(i)] = val[t][j];
        }
        const double s = static_cast<double>(step0 + 1 + t);
        const double bc1 = 1.0 - std::pow(b1, s);
        const double bc2 = 1.0 - std::pow(b2, s);
        for (int64_t i = 0; i < n; ++i) {
            const double gi = g[static_cast<size_t>(i)];
            const float mf = static_cast<float>(b1 * m[i] + (1.0 - b1) * gi);
            const float vf = static_cast<float>(b2 * v[i] + (1.0 - b2) * gi * gi);
            m[i] = mf;
            v[i] = vf;
            const double mhat = static_cast<double>(mf) / bc1;
            const double vhat = static_cast<double>(vf) / bc2;
            w[i] = static_cast<float>(static_cast<double>(w[i]) - lrd * mhat / (std::sqrt(vhat) + epsd));
        }
    }
    return 0;
}

// Sync of Algorithm 1 (Eq. (3)) for compressed gradients that arrive as N per-worker
// record lists (what an all-gather leaves on every rank): one list, ascending in
// index, holding for every index recorded by at least one worker
//     scale * (((+0 + v_{r1}) + v_{r2}) + ...)      r1 < r2 < ... the workers that recorded it
// - each + one fp32 add, in worker order; scale = 1 for a sum, 1/N for a mean.  The paper
// does not say which; the caller chooses.  Returns the number of records written
// (out_idx / out_val must hold sum K), or -1 on an index out of range or not ascending.
int64_t oracle_combine_sparse(const int32_t* const* idx, const float* const* val, const int64_t* K,
                              int32_t N, int64_t n, float scale, int32_t* out_idx, float* out_val) {
    std::vector<int64_t> head(static_cast<size_t>(N), 0);
    int64_t out = 0;
    for (;;) {
        // smallest index not yet consumed
        int64_t cur = -1;
        for (int32_t r = 0; r < N; ++r) {
            if (head[r] < K[r]) {
                const int64_t i = idx[r][head[r]];
                if (i < 0 || i >= n) return -1;
                if (head[r] > 0 && idx[r][head[r] - 1] >= i) return -1;
                if (cur < 0 || i < cur) cur = i;
            }
        }
        if (cur < 0) break;
        float sum = 0.0f;
        for (int32_t r = 0; r < N; ++r) {
            if (head[r] < K[r] && idx[r][head[r]] == cur) {
                sum = sum + val[r][head[r]];
                ++head[r];
            }
        }
        out_idx[out] = static_cast<int32_t>(cur);
        out_val[out] = scale * sum;
        ++out;
    }
    return out;
}

// The Recovery loop of Algorithm 1 merges differentials it has just read back from storage.
// The merges assume of such a differential that every index lies in [0, n), that the indices
// ascend strictly, and that no value is a NaN. Counts, record by record, how often each
// assumption is broken: out[0] indices out of range, out[1] records whose index does not
// exceed its predecessor's, out[2] NaN values (val may be null: then 0).
void oracle_check_diff(const int32_t* idx, const float* val, int64_t K, int64_t n, int64_t* out) {
    out[0] = out[1] = out[2] = 0;
    for (int64_t j = 0; j < K; ++j) {
        if (idx[j] < 0 || idx[j] >= n) ++out[0];
        if (j > 0 && idx[j] <= idx[j - 1]) ++out[1];
        if (val && std::isnan(val[j])) ++out[2];
    }
}

// Expected wasted GPU time of a run, Eq. (10) of Sec. V-C, for a full-checkpoint interval of f
// iterations and b differentials per batched checkpoint (1 <= b <= f):
//   failures  N*T/M  times  [ half a batching interval of lost work, b*tau/2
//                             + one full-checkpoint restore, R_F
//                             + half of the (f/b - 1) batched differentials replayed, R_B each ]
//   + the writes: T/(f*tau) full checkpoints at C_F each and (f/b - 1) times as many batched
//     differentials at C_B each, on all N GPUs.
double oracle_wasted_time(double N, double T, double M, double tau, double f, double b, double R_F,
                          double R_B, double C_F, double C_B) {
    const double n_failures = T / M;
    const double per_failure = b * tau / 2.0 + R_F + (R_B / 2.0) * (f / b - 1.0);
    const double n_full = T / (f * tau);
    const double n_diff = n_full * (f / b - 1.0);
    return N * n_failures * per_failure + N * n_full * C_F + N * n_diff * C_B;
}

// The interval at which dT_w/df = 0 for a given b, Eq. (11).
double oracle_critical_interval(double M, double tau, double b, double R_B, double C_F, double C_B) {
    return std::sqrt(2.0 * M * b * (C_F - C_B) / (tau * R_B));
}

}  // extern "C"
