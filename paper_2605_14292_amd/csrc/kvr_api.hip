// C-ABI entry points: argument validation on the host, then kernel launches on
// the caller's stream.  Nothing here allocates, synchronises or keeps state.
#include "../../include/kvr.h"

#include <cmath>
#include <mutex>

#include "kvr_kernels.hpp"

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_layout(const kvr_layout* lay) {
  if (!lay) return KVR_ERR_ARG;
  if (lay->heads < 1 || lay->n < 1) return KVR_ERR_ARG;
  if (lay->dtype != KVR_F32 && lay->dtype != KVR_BF16) return KVR_ERR_UNSUPPORTED;
  if (lay->d != 128) return KVR_ERR_UNSUPPORTED;
  if (lay->n > KVR_MAX_N) return KVR_ERR_UNSUPPORTED;
  if (lay->stride_tok < lay->d || (lay->stride_tok & 7)) return KVR_ERR_ARG;
  if (lay->stride_head < static_cast<int64_t>(lay->n) * lay->stride_tok || (lay->stride_head & 7))
    return KVR_ERR_ARG;
  if (lay->heads > 65535 * 1024) return KVR_ERR_UNSUPPORTED;
  return KVR_OK;
}

kvr::Layout to_dev(const kvr_layout* lay) {
  kvr::Layout l;
  l.heads = lay->heads; l.n = lay->n; l.d = lay->d; l.dtype = lay->dtype;
  l.stride_head = lay->stride_head; l.stride_tok = lay->stride_tok;
  return l;
}

int check_select(const kvr_layout* lay, int b, float lambda, float eps) {
  const int rc = check_layout(lay);
  if (rc) return rc;
  if (b < 1 || b > lay->n) return KVR_ERR_ARG;
  if (!(lambda >= 0.0f) || std::isinf(lambda)) return KVR_ERR_ARG;
  if (!(eps >= 0.0f) || std::isinf(eps)) return KVR_ERR_ARG;
  return KVR_OK;
}

using kvr::cu_count;

// The fused kernel for bf16 heads of up to 256 tokens: sixteen waves per head when every head gets
// a CU to itself, four otherwise.
hipError_t retain_dense_any(const void* K, const void* V, const void* Q, int G, const float* s_in,
                            const kvr::Layout& l, int b, float lambda, float eps, float* s_out,
                            int32_t* idx_sorted, int32_t* pick_order, float* pick_gain, void* K_out, void* V_out,
                            hipStream_t st, const int32_t* b_h = nullptr) {
  if (kvr::dense16_supported(l, b, G, Q != nullptr, cu_count()))
    return kvr::launch_retain_dense16(K, V, Q, G, s_in, l, b, lambda, eps, s_out, idx_sorted, pick_order,
                                      pick_gain, K_out, V_out, st, b_h);
  return kvr::launch_retain_dense(K, V, Q, G, s_in, l, b, lambda, eps, s_out, idx_sorted, pick_order, pick_gain,
                                  K_out, V_out, st, false, b_h);
}

// Selection without compaction: the kernel is chosen by shape only.
hipError_t select_only(const void* V, const float* s, const kvr::Layout& l, int b, float lambda, float eps,
                       int32_t* idx_sorted, int32_t* pick_order, float* pick_gain, hipStream_t st) {
  // (a call with at most one head per CU is a latency problem: the sixteen-wave kernel takes it)
  if (kvr::pruned_supported(l, b, lambda, false) && !kvr::dense16_supported(l, b, 0, false, cu_count())) {
    const hipError_t e = kvr::launch_retain_pruned(nullptr, V, s, l, b, lambda, eps, idx_sorted, pick_order,
                                                   pick_gain, nullptr, nullptr, st);
    if (e != hipSuccess) return e;
    return kvr::launch_retain_dense(nullptr, V, nullptr, 0, s, l, b, lambda, eps, nullptr, idx_sorted,
                                    pick_order, pick_gain, nullptr, nullptr, st, true);
  }
  if (kvr::dense_supported(l, b, 0, false))
    return retain_dense_any(nullptr, V, nullptr, 0, s, l, b, lambda, eps, nullptr, idx_sorted, pick_order,
                            pick_gain, nullptr, nullptr, st);
  if (kvr::dense_f32_supported(l, b))
    return kvr::launch_select_dense_f32(V, s, l, b, lambda, eps, idx_sorted, pick_order, pick_gain, st);
  if (kvr::topb_supported(l, b, lambda))
    return kvr::launch_select_topb(nullptr, nullptr, s, l, b, idx_sorted, pick_order, pick_gain, nullptr,
                                   nullptr, st);
  if (kvr::lazy_supported(l, b, lambda)) {
    const bool sparse = kvr::sparse_supported(l, b, lambda);   // heads that the score bound shrinks to a short head first
    if (sparse) {
      const hipError_t e = kvr::launch_retain_sparse(nullptr, V, s, l, b, lambda, eps, idx_sorted, pick_order,
                                                     pick_gain, nullptr, nullptr, st);
      if (e != hipSuccess) return e;
    }
    return kvr::launch_select_lazy(nullptr, V, s, l, b, lambda, eps, idx_sorted, pick_order, pick_gain,
                                   nullptr, nullptr, st, nullptr, sparse);
  }
  if (kvr::lazy_f32_supported(l, b, lambda))
    return kvr::launch_select_lazy_f32(V, s, l, b, lambda, eps, idx_sorted, pick_order, pick_gain, st);
  if (kvr::pool_supported(l, b))
    return kvr::launch_select_pool(nullptr, V, s, l, b, lambda, eps, idx_sorted, pick_order, pick_gain,
                                   nullptr, nullptr, st, nullptr, true);
  return kvr::launch_select_generic(V, s, l, b, lambda, eps, idx_sorted, pick_order, pick_gain, st);
}

int retain_budgeted(const void* K, const void* V, const void* Q, int G, const float* s_in,
                    const kvr_layout* lay, const int32_t* n_h, const int32_t* b_h, int b_max,
                    const uint8_t* keep, const int32_t* pos_in, const float* lambda_h, float lambda,
                    float eps, float* s_work, int32_t* idx_sorted, int32_t* pick_order, float* pick_gain,
                    void* K_out, void* V_out, int32_t* pos_out, void* stream);

// Scratch of kvr_retain_budgeted_static: the adjusted scores [heads, n] of a call, in device memory that
// the library's code object brings along (every GPU the library runs on holds its own copy of the array at
// its own address until the process ends).  In host code the array's name is only a handle: the device
// address is asked for once per device, with that device current, and kept.
static __device__ __align__(256) float scratch[KVR_STATIC_SCRATCH_FLOATS];

constexpr int kMaxDevices = 64;
std::mutex scratch_mu;
float* scratch_ptr[kMaxDevices] = {};

int static_scratch(float** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return KVR_ERR_HIP;
  std::lock_guard<std::mutex> lock(scratch_mu);
  if (!scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return KVR_ERR_HIP;
    scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = scratch_ptr[dev];
  return KVR_OK;
}

}  // namespace

extern "C" {

int kvr_version(void) { return 1; }

int kvr_debug_validate_finite(const void* K, const void* V, const void* Q, int G, const float* s,
                              const kvr_layout* lay, void* stream) {
  const int rc = check_layout(lay);
  if (rc) return rc;
  if (!K && !V && !Q && !s) return KVR_ERR_ARG;
  if (Q && G < 1) return KVR_ERR_ARG;
  if (Q && G > KVR_MAX_G) return KVR_ERR_UNSUPPORTED;
  if (!aligned16(K) || !aligned16(V) || !aligned16(Q) || !aligned16(s)) return KVR_ERR_ARG;
  int found = 0;
  if (kvr::validate_finite(K, V, Q, G, s, to_dev(lay), static_cast<hipStream_t>(stream), &found) != hipSuccess)
    return KVR_ERR_HIP;
  return found ? KVR_ERR_NONFINITE : KVR_OK;
}

int kvr_debug_bounds_selftest(int32_t* out, void* stream) {
  if (!out) return KVR_ERR_ARG;
  return kvr::launch_bounds_selftest(out, static_cast<hipStream_t>(stream)) == hipSuccess ? KVR_OK : KVR_ERR_HIP;
}

int kvr_debug_bounds_violation(uint32_t* worst_id) {
  if (!worst_id) return KVR_ERR_ARG;
  const unsigned int a = kvr::bounds_bad_lazy(), b = kvr::bounds_bad_pool(), c = kvr::bounds_bad_sparse();
  if (a == 0xffffffffu || b == 0xffffffffu || c == 0xffffffffu) return KVR_ERR_HIP;
  *worst_id = a > b ? (a > c ? a : c) : (b > c ? b : c);
  return KVR_OK;
}

const char* kvr_strerror(int status) {
  switch (status) {
    case KVR_OK: return "ok";
    case KVR_ERR_ARG: return "invalid argument";
    case KVR_ERR_UNSUPPORTED: return "unsupported shape or dtype";
    case KVR_ERR_WORKSPACE: return "workspace too small";
    case KVR_ERR_HIP: return "HIP launch failed";
    case KVR_ERR_NONFINITE: return "non-finite value in the inputs";
    default: return "unknown kvr status";
  }
}

int kvr_workspace_bytes(const kvr_layout* lay, int b, int G, size_t* bytes_out) {
  if (!bytes_out) return KVR_ERR_ARG;
  const int rc = check_layout(lay);
  if (rc) return rc;
  if (b < 1 || b > lay->n || G < 0 || G > KVR_MAX_G) return KVR_ERR_ARG;
  *bytes_out = 0;
  return KVR_OK;
}

int kvr_score(const void* K, const void* Q, int G, const kvr_layout* lay, float* s_out,
              void* stream) {
  const int rc = check_layout(lay);
  if (rc) return rc;
  if (!K || !Q || !s_out) return KVR_ERR_ARG;
  if (G < 1) return KVR_ERR_ARG;
  if (G > KVR_MAX_G) return KVR_ERR_UNSUPPORTED;
  if (!aligned16(K) || !aligned16(Q) || !aligned16(s_out)) return KVR_ERR_ARG;
  const hipError_t e = kvr::launch_score(K, Q, G, to_dev(lay), s_out, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? KVR_OK : KVR_ERR_HIP;
}

int kvr_select_greedy(const void* V, const float* s, const kvr_layout* lay, int b, float lambda,
                      float eps, int32_t* idx_sorted, int32_t* pick_order, float* pick_gain,
                      void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace; (void)workspace_bytes;
  const int rc = check_select(lay, b, lambda, eps);
  if (rc) return rc;
  if (!s || !idx_sorted) return KVR_ERR_ARG;
  if (lambda != 0.0f && !V) return KVR_ERR_ARG;
  if ((V && !aligned16(V)) || !aligned16(s)) return KVR_ERR_ARG;
  const hipError_t e = select_only(V, s, to_dev(lay), b, lambda, eps, idx_sorted, pick_order, pick_gain,
                                   static_cast<hipStream_t>(stream));
  return e == hipSuccess ? KVR_OK : KVR_ERR_HIP;
}

int kvr_compact(const void* K, const void* V, const kvr_layout* lay, const int32_t* idx, int b,
                void* K_out, void* V_out, void* stream) {
  const int rc = check_layout(lay);
  if (rc) return rc;
  if (b < 1 || b > lay->n || !idx) return KVR_ERR_ARG;
  if ((K == nullptr) != (K_out == nullptr) || (V == nullptr) != (V_out == nullptr)) return KVR_ERR_ARG;
  if (!K && !V) return KVR_ERR_ARG;
  if ((K && (!aligned16(K) || !aligned16(K_out))) || (V && (!aligned16(V) || !aligned16(V_out))))
    return KVR_ERR_ARG;
  const hipError_t e = kvr::launch_compact(K, V, to_dev(lay), idx, b, K_out, V_out,
                                           static_cast<hipStream_t>(stream));
  return e == hipSuccess ? KVR_OK : KVR_ERR_HIP;
}

int kvr_retain(const void* K, const void* V, const void* Q, int G, const float* s_in,
               const kvr_layout* lay, int b, float lambda, float eps, float* s_out,
               int32_t* idx_sorted, int32_t* pick_order, float* pick_gain, void* K_out,
               void* V_out, void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace; (void)workspace_bytes;
  const int rc = check_select(lay, b, lambda, eps);
  if (rc) return rc;
  if (!K || !V || !idx_sorted || !K_out || !V_out) return KVR_ERR_ARG;
  if ((Q == nullptr) == (s_in == nullptr)) return KVR_ERR_ARG;
  if (Q && (G < 1)) return KVR_ERR_ARG;
  if (Q && G > KVR_MAX_G) return KVR_ERR_UNSUPPORTED;
  if (Q && !s_out) return KVR_ERR_ARG;  // the computed scores need somewhere to live
  if (!aligned16(K) || !aligned16(V) || !aligned16(K_out) || !aligned16(V_out) ||
      (Q && !aligned16(Q)) || (s_in && !aligned16(s_in)) || (s_out && !aligned16(s_out)))
    return KVR_ERR_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const kvr::Layout l = to_dev(lay);
  const float* s = s_in;
  if (Q && kvr::dense_supported(l, b, G, true)) {       // short heads, few queries: scoring is fused too
    const hipError_t e = retain_dense_any(K, V, Q, G, nullptr, l, b, lambda, eps, s_out, idx_sorted, pick_order,
                                          pick_gain, K_out, V_out, st);
    return e == hipSuccess ? KVR_OK : KVR_ERR_HIP;
  }
  if (kvr::dense_f32_supported(l, b) && (!Q || G <= kvr::kDenseF32MaxG)) {   // short fp32 heads: one launch
    const hipError_t e = kvr::launch_retain_dense_f32(K, V, Q, G, s_in, l, b, lambda, eps, s_out, idx_sorted,
                                                      pick_order, pick_gain, K_out, V_out, st);
    return e == hipSuccess ? KVR_OK : KVR_ERR_HIP;
  }
  if (Q) {
    if (kvr::launch_score(K, Q, G, l, s_out, st) != hipSuccess) return KVR_ERR_HIP;
    s = s_out;
  }
  // scores computed here are softmax means, far tighter than lambda: the score bound removes nothing;
  // and a call with at most one head per CU is a latency problem, which the sixteen-wave kernel takes
  if (!Q && kvr::pruned_supported(l, b, lambda, false) && !kvr::dense16_supported(l, b, 0, false, cu_count())) {
    hipError_t e = kvr::launch_retain_pruned(K, V, s, l, b, lambda, eps, idx_sorted, pick_order,
                                             pick_gain, K_out, V_out, st);
    if (e == hipSuccess)
      e = kvr::launch_retain_dense(K, V, nullptr, 0, s, l, b, lambda, eps, nullptr, idx_sorted,
                                   pick_order, pick_gain, K_out, V_out, st, true);
    return e == hipSuccess ? KVR_OK : KVR_ERR_HIP;
  }
  if (kvr::dense_supported(l, b, 0, false)) {
    const hipError_t e = retain_dense_any(K, V, nullptr, 0, s, l, b, lambda, eps, nullptr, idx_sorted, pick_order,
                                          pick_gain, K_out, V_out, st);
    return e == hipSuccess ? KVR_OK : KVR_ERR_HIP;
  }
  if (kvr::topb_supported(l, b, lambda) && l.dtype == KVR_BF16) {
    const hipError_t e = kvr::launch_select_topb(K, V, s, l, b, idx_sorted, pick_order, pick_gain, K_out,
                                                 V_out, st);
    return e == hipSuccess ? KVR_OK : KVR_ERR_HIP;
  }
  if (kvr::lazy_supported(l, b, lambda)) {
    // scores handed in may spread by more than lambda: the heads that the score bound shrinks to a short head are
    // finished first (scores computed here are softmax means, far tighter than lambda: nothing to drop)
    const bool sparse = !Q && kvr::sparse_supported(l, b, lambda);
    hipError_t e = hipSuccess;
    if (sparse)
      e = kvr::launch_retain_sparse(K, V, s, l, b, lambda, eps, idx_sorted, pick_order, pick_gain, K_out, V_out, st);
    if (e == hipSuccess)
      e = kvr::launch_select_lazy(K, V, s, l, b, lambda, eps, idx_sorted, pick_order, pick_gain, K_out, V_out, st,
                                  nullptr, sparse);
    return e == hipSuccess ? KVR_OK : KVR_ERR_HIP;
  }
  if (kvr::pool_supported(l, b)) {
    const hipError_t e = kvr::launch_select_pool(K, V, s, l, b, lambda, eps, idx_sorted, pick_order,
                                                 pick_gain, K_out, V_out, st, nullptr, Q == nullptr);
    return e == hipSuccess ? KVR_OK : KVR_ERR_HIP;
  }
  if (select_only(V, s, l, b, lambda, eps, idx_sorted, pick_order, pick_gain, st) != hipSuccess)
    return KVR_ERR_HIP;
  if (kvr::launch_compact(K, V, l, idx_sorted, b, K_out, V_out, st) != hipSuccess)
    return KVR_ERR_HIP;
  return KVR_OK;
}

int kvr_retain_budgeted(const void* K, const void* V, const void* Q, int G, const float* s_in,
                        const kvr_layout* lay, const int32_t* n_h, const int32_t* b_h, int b_max,
                        const uint8_t* keep, const int32_t* pos_in, const float* lambda_h, float lambda,
                        float eps, float* s_work, int32_t* idx_sorted, int32_t* pick_order, float* pick_gain,
                        void* K_out, void* V_out, int32_t* pos_out, void* stream) {
  return retain_budgeted(K, V, Q, G, s_in, lay, n_h, b_h, b_max, keep, pos_in, lambda_h, lambda, eps, s_work,
                         idx_sorted, pick_order, pick_gain, K_out, V_out, pos_out, stream);
}

int kvr_retain_budgeted_static(const void* K, const void* V, const void* Q, int G, const float* s_in,
                               const kvr_layout* lay, const int32_t* n_h, const int32_t* b_h, int b_max,
                               const uint8_t* keep, const int32_t* pos_in, const float* lambda_h, float lambda,
                               float eps, int32_t* idx_sorted, int32_t* pick_order, float* pick_gain,
                               void* K_out, void* V_out, int32_t* pos_out, void* stream) {
  const int rc = check_select(lay, b_max, lambda, eps);
  if (rc) return rc;
  if (static_cast<unsigned long long>(lay->heads) * static_cast<unsigned long long>(lay->n) > KVR_STATIC_SCRATCH_FLOATS)
    return KVR_ERR_WORKSPACE;                 // the adjusted scores of this call do not fit the static array
  float* s_work = nullptr;
  const int rs = static_scratch(&s_work);
  if (rs) return rs;
  return retain_budgeted(K, V, Q, G, s_in, lay, n_h, b_h, b_max, keep, pos_in, lambda_h, lambda, eps, s_work,
                         idx_sorted, pick_order, pick_gain, K_out, V_out, pos_out, stream);
}

}  // extern "C"

namespace {

int retain_budgeted(const void* K, const void* V, const void* Q, int G, const float* s_in,
                    const kvr_layout* lay, const int32_t* n_h, const int32_t* b_h, int b_max,
                    const uint8_t* keep, const int32_t* pos_in, const float* lambda_h, float lambda,
                    float eps, float* s_work, int32_t* idx_sorted, int32_t* pick_order, float* pick_gain,
                    void* K_out, void* V_out, int32_t* pos_out, void* stream) {
  const int rc = check_select(lay, b_max, lambda, eps);
  if (rc) return rc;
  if (!V || !s_work || !idx_sorted || !pick_order) return KVR_ERR_ARG;
  if ((Q == nullptr) == (s_in == nullptr)) return KVR_ERR_ARG;
  if (Q && (G < 1 || !K)) return KVR_ERR_ARG;
  if (Q && G > KVR_MAX_G) return KVR_ERR_UNSUPPORTED;
  if ((K_out && !K) || (pos_out && !pos_in)) return KVR_ERR_ARG;
  if (lambda_h && !(lambda > 0.0f)) return KVR_ERR_ARG;   // per-head values rescale a positive launch lambda
  if (!aligned16(V) || !aligned16(s_work) || (K && !aligned16(K)) || (Q && !aligned16(Q)) ||
      (s_in && !aligned16(s_in)) || (K_out && !aligned16(K_out)) || (V_out && !aligned16(V_out)))
    return KVR_ERR_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const kvr::Layout l = to_dev(lay);
  const float* src = s_in;
  if (Q) {
    if (kvr::launch_score(K, Q, G, l, s_work, st) != hipSuccess) return KVR_ERR_HIP;
    src = s_work;
  }
  if (kvr::launch_budget_prepare(src, l, n_h, keep, lambda_h, lambda, s_work, st) != hipSuccess)
    return KVR_ERR_HIP;
  // bf16 heads of up to 4096 tokens: the fused kernels take the per-head budgets themselves (the chain of a head
  // stops at its own budget; lists, padding and kept rows are written by the kernel that selected
  // them); what is left is elementwise: the gains of protected tokens, per-head lambdas, position ids.
  const bool long_heads = lambda > 0.0f && kvr::pool_supported(l, b_max);
  const bool long_topb = kvr::topb_supported(l, b_max, lambda) && l.dtype == KVR_BF16;
  const bool fused = (K_out == nullptr) == (V_out == nullptr) && (!K_out || K) &&
                     (kvr::pruned_supported(l, b_max, lambda, false) || kvr::dense_supported(l, b_max, 0, false) ||
                      long_heads || long_topb);
  if (fused) {
    hipError_t e;
    if (long_topb) {
      e = kvr::launch_select_topb(K, V, s_work, l, b_max, idx_sorted, pick_order, pick_gain, K_out, V_out, st, b_h);
    } else if (long_heads && kvr::lazy_supported(l, b_max, lambda)) {
      // scores handed in may spread by more than lambda: the heads that the score bound shrinks to a short head are
      // finished first (computed scores are tighter than lambda, and the offsets of protected tokens would only
      // make the kernel search every head in vain)
      const bool sparse = !Q && kvr::sparse_supported(l, b_max, lambda);
      e = hipSuccess;
      if (sparse)
        e = kvr::launch_retain_sparse(K, V, s_work, l, b_max, lambda, eps, idx_sorted, pick_order, pick_gain, K_out,
                                      V_out, st, b_h);
      if (e == hipSuccess)
        e = kvr::launch_select_lazy(K, V, s_work, l, b_max, lambda, eps, idx_sorted, pick_order, pick_gain, K_out,
                                    V_out, st, b_h, sparse);
    } else if (long_heads) {
      e = kvr::launch_select_pool(K, V, s_work, l, b_max, lambda, eps, idx_sorted, pick_order, pick_gain, K_out,
                                  V_out, st, b_h, Q == nullptr);
    } else if (kvr::pruned_supported(l, b_max, lambda, false) &&
               !kvr::dense16_supported(l, b_max, 0, false, cu_count())) {
      e = kvr::launch_retain_pruned(K, V, s_work, l, b_max, lambda, eps, idx_sorted, pick_order, pick_gain, K_out,
                                    V_out, st, b_h);
      if (e == hipSuccess)
        e = kvr::launch_retain_dense(K, V, nullptr, 0, s_work, l, b_max, lambda, eps, nullptr, idx_sorted,
                                     pick_order, pick_gain, K_out, V_out, st, true, b_h);
    } else {
      e = retain_dense_any(K, V, nullptr, 0, s_work, l, b_max, lambda, eps, nullptr, idx_sorted, pick_order,
                           pick_gain, K_out, V_out, st, b_h);
    }
    if (e != hipSuccess) return KVR_ERR_HIP;
    if (kvr::launch_budget_fixup(l, b_max, keep, lambda_h, lambda, pos_in, idx_sorted, pick_order, pick_gain,
                                 pos_out, st) != hipSuccess)
      return KVR_ERR_HIP;
    return KVR_OK;
  }
  if (select_only(V, s_work, l, b_max, lambda, eps, idx_sorted, pick_order, pick_gain, st) != hipSuccess)
    return KVR_ERR_HIP;
  if (kvr::launch_budget_finalize(K, V, l, b_h, b_max, keep, lambda_h, lambda, pos_in, idx_sorted, pick_order, pick_gain,
                                  K_out, V_out, pos_out, st) != hipSuccess)
    return KVR_ERR_HIP;
  return KVR_OK;
}

}  // namespace

extern "C" {

int kvr_signature_flat(const void* V, const kvr_layout* lay, int group, float* u_out, void* stream) {
  const int rc = check_layout(lay);
  if (rc) return rc;
  if (!V || !u_out || group < 1 || lay->heads % group != 0) return KVR_ERR_ARG;
  if (!aligned16(V) || !aligned16(u_out)) return KVR_ERR_ARG;
  const hipError_t e = kvr::launch_signature_flat(V, to_dev(lay), group, u_out, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? KVR_OK : KVR_ERR_HIP;
}

int kvr_compact_shared(const void* K, const void* V, const kvr_layout* lay, int group, const int32_t* idx,
                       int b, void* K_out, void* V_out, void* stream) {
  const int rc = check_layout(lay);
  if (rc) return rc;
  if (b < 1 || b > lay->n || !idx || group < 1 || lay->heads % group != 0) return KVR_ERR_ARG;
  if ((K == nullptr) != (K_out == nullptr) || (V == nullptr) != (V_out == nullptr)) return KVR_ERR_ARG;
  if (!K && !V) return KVR_ERR_ARG;
  if ((K && (!aligned16(K) || !aligned16(K_out))) || (V && (!aligned16(V) || !aligned16(V_out))))
    return KVR_ERR_ARG;
  const hipError_t e = kvr::launch_compact(K, V, to_dev(lay), idx, b, K_out, V_out,
                                           static_cast<hipStream_t>(stream), group);
  return e == hipSuccess ? KVR_OK : KVR_ERR_HIP;
}

int kvr_score_pool(const float* s_in, int heads, int n, int kernel, int mode, float* s_out, void* stream) {
  if (!s_in || !s_out || s_in == s_out) return KVR_ERR_ARG;
  if (heads < 1 || heads > 65535 || n < 1 || n > KVR_MAX_N) return KVR_ERR_ARG;
  if (kernel < 1 || kernel > KVR_MAX_POOL || (kernel & 1) == 0) return KVR_ERR_ARG;
  if (mode != KVR_POOL_MAX && mode != KVR_POOL_MEAN) return KVR_ERR_ARG;
  const hipError_t e = kvr::launch_score_pool(s_in, heads, n, kernel, mode == KVR_POOL_MEAN, s_out,
                                              static_cast<hipStream_t>(stream));
  return e == hipSuccess ? KVR_OK : KVR_ERR_HIP;
}

int kvr_score_prior(const void* V, const kvr_layout* lay, const float* s_in, float lambda_p, float eps,
                    float* s_out, void* stream) {
  const int rc = check_layout(lay);
  if (rc) return rc;
  if (!V || !s_in || !s_out || !aligned16(V)) return KVR_ERR_ARG;
  if (std::isnan(lambda_p) || std::isinf(lambda_p) || !(eps >= 0.0f) || std::isinf(eps)) return KVR_ERR_ARG;
  const hipError_t e = kvr::launch_score_prior(V, to_dev(lay), s_in, lambda_p, eps, s_out,
                                               static_cast<hipStream_t>(stream));
  return e == hipSuccess ? KVR_OK : KVR_ERR_HIP;
}

int kvr_compact_inplace(void* K, void* V, const kvr_layout* lay, int group, const int32_t* idx, int b,
                        int32_t* pos, void* stream) {
  const int rc = check_layout(lay);
  if (rc) return rc;
  if (b < 1 || b > lay->n || !idx || group < 1 || lay->heads % group != 0) return KVR_ERR_ARG;
  if (!K && !V && !pos) return KVR_ERR_ARG;
  if ((K && !aligned16(K)) || (V && !aligned16(V))) return KVR_ERR_ARG;
  const hipError_t e = kvr::launch_compact_inplace(K, V, to_dev(lay), idx, group, b, pos,
                                                   static_cast<hipStream_t>(stream));
  return e == hipSuccess ? KVR_OK : KVR_ERR_HIP;
}

int kvr_retain_flat(const void* K, const void* V, const float* s, const kvr_layout* lay, int group, int b,
                    float lambda, float eps, float* u_out, int32_t* idx_sorted, int32_t* pick_order,
                    float* pick_gain, void* K_out, void* V_out, void* stream) {
  const int rc = check_select(lay, b, lambda, eps);
  if (rc) return rc;
  if (!K || !V || !s || !idx_sorted || !K_out || !V_out) return KVR_ERR_ARG;
  if (group < 1 || lay->heads % group != 0) return KVR_ERR_ARG;
  if (lambda != 0.0f && !u_out) return KVR_ERR_ARG;    // the signature rows need somewhere to live
  if (!aligned16(K) || !aligned16(V) || !aligned16(s) || !aligned16(K_out) || !aligned16(V_out) ||
      (u_out && !aligned16(u_out)))
    return KVR_ERR_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const kvr::Layout l = to_dev(lay);
  kvr::Layout lu = l;                                   // the per-sequence problems: fp32 rows, dense
  lu.heads = l.heads / group; lu.dtype = KVR_F32;
  lu.stride_tok = l.d; lu.stride_head = static_cast<long long>(l.n) * l.d;
  // (the per-sequence thresholds of the signature kernel park in idx_sorted[q * b], which the selection overwrites)
  if (lambda != 0.0f && kvr::launch_signature_flat(V, l, group, u_out, st, s, b, lambda,
                                                   reinterpret_cast<float*>(idx_sorted), b) != hipSuccess)
    return KVR_ERR_HIP;
  if (select_only(u_out, s, lu, b, lambda, eps, idx_sorted, pick_order, pick_gain, st) != hipSuccess)
    return KVR_ERR_HIP;
  if (kvr::launch_compact(K, V, l, idx_sorted, b, K_out, V_out, st, group) != hipSuccess)
    return KVR_ERR_HIP;
  return KVR_OK;
}

}  // extern "C"
