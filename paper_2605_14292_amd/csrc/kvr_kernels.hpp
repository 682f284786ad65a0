// Launch interface between the host entry points and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvr {

struct Layout {
  int heads, n, d, dtype;
  long long stride_head, stride_tok;
};

// Compute units of the current device (256 on an MI355X), looked up on first use.  The value only
// sizes grids (persistent workgroups, one-head-per-CU dispatch), so the device of the first call
// stands for every device of the process.
inline int cu_count() {
  static const int cus = [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      return v;
    return 256;
  }();
  return cus;
}

hipError_t launch_score(const void* K, const void* Q, int G, const Layout& lay,
                        float* s_out, hipStream_t st);
// lambda = 0 for heads of more than 256 tokens: top-b of the scores (any dtype: V is not read), and
// the compaction of the kept rows when K_out / V_out are given (bf16 layouts only).
bool topb_supported(const Layout& lay, int b, float lambda);
hipError_t launch_select_topb(const void* K, const void* V, const float* s, const Layout& lay, int b,
                              int32_t* idx_sorted, int32_t* pick_order, float* pick_gain, void* K_out,
                              void* V_out, hipStream_t st, const int32_t* b_h = nullptr);
// bf16 scores for up to 256 queries per head and any n: two passes over K on the matrix cores.
bool score_wide_supported(const Layout& lay, int G);
hipError_t launch_score_wide(const void* K, const void* Q, int G, const Layout& lay, float* s_out,
                             hipStream_t st);
hipError_t launch_select_generic(const void* V, const float* s, const Layout& lay, int b,
                                 float lambda, float eps, int32_t* idx_sorted,
                                 int32_t* pick_order, float* pick_gain, hipStream_t st);
// idx_group consecutive heads share one row of idx (1: every head has its own).
hipError_t launch_compact(const void* K, const void* V, const Layout& lay, const int32_t* idx,
                          int b, void* K_out, void* V_out, hipStream_t st, int idx_group = 1);
// The same move inside K and V themselves (rows 0..b-1 of each head receive the kept rows);
// pos: dense int32 [heads, n] moved alike, or null.  Index rows must be strictly ascending.
hipError_t launch_compact_inplace(void* K, void* V, const Layout& lay, const int32_t* idx, int idx_group,
                                  int b, int32_t* pos, hipStream_t st);

// Pooling of each score row over a centred window of `kernel` (odd) tokens: maximum, or mean if `mean`.
hipError_t launch_score_pool(const float* s_in, int heads, int n, int kernel, int mean, float* s_out,
                             hipStream_t st);
// s_out = s_in + lambda_p * cos(V_i, mean_j V_j) per head; s_out may be s_in.
hipError_t launch_score_prior(const void* V, const Layout& lay, const float* s_in, float lambda_p, float eps,
                              float* s_out, hipStream_t st);

// Mean of V over each run of `group` consecutive heads: u_out is dense fp32 [heads/group, n, d].
hipError_t launch_signature_flat(const void* V, const Layout& lay, int group, float* u_out, hipStream_t st,
                                 const float* s = nullptr, int b = 0, float lambda = 0.f, float* thr = nullptr,
                                 int thr_stride = 0);
// With s (one score vector per sequence): the rows of tokens with s_j < s_(b) - lambda, which Algorithm 1 never
// selects, are not computed (zero rows); thr[seq * thr_stride] receives the per-sequence threshold.

// Selection for heads with fp32 rows and n <= 256 (no compaction).
bool dense_f32_supported(const Layout& lay, int b);
hipError_t launch_select_dense_f32(const void* V, const float* s, const Layout& lay, int b, float lambda,
                                   float eps, int32_t* idx_sorted, int32_t* pick_order, float* pick_gain,
                                   hipStream_t st);
// The same kernel with the base scores computed inside (Q given, G <= 16) and the kept rows written.
constexpr int kDenseF32MaxG = 16;
hipError_t launch_retain_dense_f32(const void* K, const void* V, const void* Q, int G, const float* s,
                                   const Layout& lay, int b, float lambda, float eps, float* s_out,
                                   int32_t* idx_sorted, int32_t* pick_order, float* pick_gain, void* K_out,
                                   void* V_out, hipStream_t st);

// Fused path for bf16 heads with n <= 256 (any of K/Q/K_out/V_out may be null
// to skip scoring or compaction).
bool dense_supported(const Layout& lay, int b, int G, bool has_q);
hipError_t launch_retain_dense(const void* K, const void* V, const void* Q, int G, const float* s_in,
                               const Layout& lay, int b, float lambda, float eps, float* s_out,
                               int32_t* idx_sorted, int32_t* pick_order, float* pick_gain,
                               void* K_out, void* V_out, hipStream_t st, bool only_marked = false,
                               const int32_t* b_h = nullptr);

// The same event for calls with at most one head per CU (heads <= cus) and 128 < n <= 256: sixteen
// waves per head for the parallel phases.
bool dense16_supported(const Layout& lay, int b, int G, bool has_q, int cus);
hipError_t launch_retain_dense16(const void* K, const void* V, const void* Q, int G, const float* s_in,
                                 const Layout& lay, int b, float lambda, float eps, float* s_out,
                                 int32_t* idx_sorted, int32_t* pick_order, float* pick_gain, void* K_out,
                                 void* V_out, hipStream_t st, const int32_t* b_h = nullptr);

// Fused path for bf16 heads with 128 < n <= 256 and given scores: tokens that the score bound
// s_j < s_(b) - lambda excludes from every pick are dropped first; heads left with at most 128
// candidates are finished, the others get idx_sorted[h*b] = -1 and must be passed to
// launch_retain_dense(..., only_marked = true) afterwards.
bool pruned_supported(const Layout& lay, int b, float lambda, bool has_q);
hipError_t launch_retain_pruned(const void* K, const void* V, const float* s, const Layout& lay, int b,
                                float lambda, float eps, int32_t* idx_sorted, int32_t* pick_order,
                                float* pick_gain, void* K_out, void* V_out, hipStream_t st,
                                const int32_t* b_h = nullptr);

// Budget allocator frame (per-head candidate counts, budgets, protected tokens): score masking
// and offsets before the selection, prefix cut, ascending read-out and row copy after it.
hipError_t launch_budget_prepare(const float* s_src, const Layout& lay, const int32_t* n_h,
                                 const uint8_t* keep, const float* lambda_h, float lambda, float* s_work,
                                 hipStream_t st);
hipError_t launch_budget_fixup(const Layout& lay, int b_max, const uint8_t* keep, const float* lambda_h,
                               float lambda, const int32_t* pos_in, const int32_t* idx_sorted,
                               const int32_t* pick_order, float* pick_gain, int32_t* pos_out, hipStream_t st);
hipError_t launch_budget_finalize(const void* K, const void* V, const Layout& lay, const int32_t* b_h,
                                  int b_max, const uint8_t* keep, const float* lambda_h, float lambda,
                                  const int32_t* pos_in, int32_t* idx_sorted, int32_t* pick_order,
                                  float* pick_gain, void* K_out, void* V_out, int32_t* pos_out,
                                  hipStream_t st);

// Pool-based exact greedy for bf16 heads with 256 < n <= 8192 and b <= 1024 (selection plus
// optional compaction; scores come in through s).
bool pool_supported(const Layout& lay, int b);
hipError_t launch_select_pool(const void* K, const void* V, const float* s, const Layout& lay, int b,
                              float lambda, float eps, int32_t* idx_sorted, int32_t* pick_order,
                              float* pick_gain, void* K_out, void* V_out, hipStream_t st,
                              const int32_t* b_h = nullptr, bool prune = false);
// prune: take the variant that first drops the tokens the score bound rules out (s_j < s_(b) - lambda)
// and skips their rows.  Worth it for scores the caller supplies; mean-of-softmax scores over hundreds
// of tokens lie far below any lambda in use, nothing can be dropped, and the variant only costs.


// The same selection with lazily refreshed penalties for bf16 heads with 256 < n <= 4096, b <= 128 and
// lambda > 0: after the first epoch only the tokens whose gain bounds can matter soon are brought up to
// date (against the rows of all picks, kept in LDS), so a head's rows are read about 2.7 times instead of
// once per epoch.  Always applies the score bound first.
bool lazy_supported(const Layout& lay, int b, float lambda);
hipError_t launch_select_lazy(const void* K, const void* V, const float* s, const Layout& lay, int b,
                              float lambda, float eps, int32_t* idx_sorted, int32_t* pick_order,
                              float* pick_gain, void* K_out, void* V_out, hipStream_t st,
                              const int32_t* b_h = nullptr, bool only_marked = false);
// only_marked: only the heads whose idx_sorted[h*b] is -1 are processed (launch_retain_sparse has finished the others).

// Fused path for the same heads (b >= 2) when their scores are handed in: the tokens that the score bound
// s_j < s_(b) - lambda excludes from every pick are dropped first; heads left with at most 128 (b <= 64) or 192
// candidates are finished as short heads are (rows gathered into LDS, cosine triangle, pick chain, kept rows),
// the others get idx_sorted[h*b] = -1 and must be passed to launch_select_lazy(..., only_marked = true) afterwards.
bool sparse_supported(const Layout& lay, int b, float lambda);
hipError_t launch_retain_sparse(const void* K, const void* V, const float* s, const Layout& lay, int b, float lambda,
                                float eps, int32_t* idx_sorted, int32_t* pick_order, float* pick_gain, void* K_out,
                                void* V_out, hipStream_t st, const int32_t* b_h = nullptr);
// The same for fp32 rows (the mean rows of the flat-signature mode, fp32 caches), selection only: the
// Gram and the passes run on the fp32 MFMAs, the rows of a pass are loaded straight into operand layout.
bool lazy_f32_supported(const Layout& lay, int b, float lambda);
hipError_t launch_select_lazy_f32(const void* V, const float* s, const Layout& lay, int b, float lambda,
                                  float eps, int32_t* idx_sorted, int32_t* pick_order, float* pick_gain,
                                  hipStream_t st);

// Debug validator: found = 1 when K, V ([heads, n, d] in lay; either may be null), Q ([heads, G, d] dense, may
// be null) or s ([heads, n], may be null) hold a NaN or an infinity.  Synchronises the stream.
hipError_t validate_finite(const void* K, const void* V, const void* Q, int G, const float* s, const Layout& lay,
                           hipStream_t st, int* found);

// Debug build only (-DKVR_BOUNDS): the largest id of a failed bounds check in the kernels of the source file since
// the last call (0: none; the product build always returns 0).  Synchronises the device.
unsigned int bounds_bad_lazy();
unsigned int bounds_bad_pool();
unsigned int bounds_bad_sparse();
// One thread range-checks the index 5 against the limit 3 (id 199) and stores what the check returned (2 in the
// debug build, 5 in the product build) in out[0]; no memory is accessed through the index.
hipError_t launch_bounds_selftest(int32_t* out, hipStream_t st);

}  // namespace kvr
