// lambda = 0 for heads of more than 256 tokens: Algorithm 1's explicit top-b branch
// (paper Sec. 4.1: at lambda = 0 the selector is the baseline's modular top-k, ties to
// the lower index), followed by the compaction of the kept rows.  V is never read for
// the selection, so the kernel needs a few KB of LDS and many heads share a CU, which
// is what hides the latency of its short dependent steps:
//   1. the b-th largest score key by a bitwise search (one workgroup-wide count per bit);
//   2. the selected tokens in token order (keys above the threshold, then the lowest-
//      indexed of the equal ones) -- that list is sort(S);
//   3. each selected token's rank among the selected gives the pick order and gains;
//   4. the kept K/V rows are copied (bf16 rows; other layouts are compacted by the caller).
// Token j = 256 * k + thread: score loads are coalesced.
#include "kvr_dense_common.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

constexpr int kTopbThreads = 256;
constexpr int kTopbMaxB = 1024;

struct TopbArgs {
  const char* K; const char* V; const float* s_in;
  int32_t* idx_sorted; int32_t* pick_order; float* pick_gain;
  char* K_out; char* V_out;
  long long stride_head, stride_tok;   // elements (bf16 when K_out / V_out are given)
  int n, b;
  const int32_t* b_h;                  // per-head budgets <= b (output rows stay b apart), or null
};

template <int S>
__global__ __launch_bounds__(kTopbThreads) void select_topb_kernel(TopbArgs a) {
  constexpr int NT = kTopbThreads, W = NT / 64;
  extern __shared__ __align__(16) int32_t smem_i[];
  int32_t* cnt_l = smem_i;                       // [2][W] counts of a search round
  int32_t* tab_a = smem_i + 16;                  // [S][W] per (slot, wave) counts
  int32_t* tab_b = tab_a + S * W;                // [S][W]
  uint32_t* sel_key = reinterpret_cast<uint32_t*>(tab_b + S * W);   // [b]
  int32_t* sel_tok = reinterpret_cast<int32_t*>(sel_key) + a.b;    // [b] = sort(S)
  int32_t* order_l = sel_tok + a.b;                                 // [b]
  float* gain_l = reinterpret_cast<float*>(order_l + a.b);          // [b]
  const int bs = a.b;                                               // rows of the outputs per head

  const int h = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = a.n;
  const int b = a.b_h ? min(max(a.b_h[h], 0), bs) : bs;             // the head's own budget
  uint32_t key[S];
#pragma unroll
  for (int k = 0; k < S; ++k) {
    const int j = k * NT + tid;
    key[k] = j < n ? ordered_key(a.s_in[static_cast<long long>(h) * n + j] + 0.0f) : 0u;   // -0 counts as +0
  }
  // ---- 1. tau = the largest key value with at least b keys >= it
  int par = 0;
  uint32_t tau = 0;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = tau | (1u << bit);
    int c_w = 0;
#pragma unroll
    for (int k = 0; k < S; ++k) c_w += __popcll(__ballot(key[k] >= cand));
    if (lane == 0) cnt_l[par * W + w] = c_w;
    lds_barrier();
    int c = 0;
#pragma unroll
    for (int u = 0; u < W; ++u) c += cnt_l[par * W + u];
    par ^= 1;
    if (c >= b) tau = cand;
  }
  // ---- 2. selected tokens in token order: token order is slot-major, then wave, then lane
  unsigned long long above[S], equal[S];
#pragma unroll
  for (int k = 0; k < S; ++k) {
    above[k] = __ballot(key[k] > tau);
    equal[k] = __ballot(key[k] == tau);
    if (lane == 0) { tab_a[k * W + w] = __popcll(above[k]); tab_b[k * W + w] = __popcll(equal[k]); }
  }
  lds_barrier();
  int above_all = 0;
  for (int u = 0; u < S * W; ++u) above_all += tab_a[u];
  const int need_eq = b - above_all;               // >= 1 by the choice of tau
  // position of this lane's tokens: selected tokens before them
  const unsigned long long below = (1ull << lane) - 1ull;
  int before_above = 0, before_equal = 0;          // counts over the (slot, wave) cells before cell (k, w)
  int cell = 0;
#pragma unroll
  for (int k = 0; k < S; ++k) {
    for (; cell < k * W + w; ++cell) { before_above += tab_a[cell]; before_equal += tab_b[cell]; }
    const int eq_rank = before_equal + __popcll(equal[k] & below);       // this token's rank among the equal ones
    const bool is_above = (above[k] >> lane) & 1ull, is_equal = (equal[k] >> lane) & 1ull;
    if (is_above || (is_equal && eq_rank < need_eq)) {
      const int eq_taken = eq_rank < need_eq ? eq_rank : need_eq;        // equal tokens before it that are selected
      const int p = before_above + __popcll(above[k] & below) + eq_taken;
      sel_key[p] = key[k];
      sel_tok[p] = k * NT + tid;
    }
  }
  lds_barrier();
  // ---- 3. rank among the selected: (score descending, index ascending); the list is in index order
  for (int e = tid; e < b; e += NT) {
    const uint32_t ke = sel_key[e];
    int rank = 0;
    for (int f = 0; f < b; ++f) {
      const uint32_t kf = sel_key[f];
      rank += (kf > ke || (kf == ke && f < e)) ? 1 : 0;
    }
    order_l[rank] = sel_tok[e];
    gain_l[rank] = key_to_float(ke);
  }
  lds_barrier();
  // ---- 4. outputs
  const long long ob = static_cast<long long>(h) * bs;
  for (int u = tid; u < bs; u += NT) {                              // entries past the head's budget are padding
    a.idx_sorted[ob + u] = u < b ? sel_tok[u] : -1;
    if (a.pick_order) a.pick_order[ob + u] = u < b ? order_l[u] : -1;
    if (a.pick_gain) a.pick_gain[ob + u] = u < b ? gain_l[u] : -INFINITY;
  }
  if ((a.K_out || a.V_out) && b > 0)
    compact_rows<4>(a.K, a.V, a.K_out, a.V_out, h * a.stride_head * 2, a.stride_tok, sel_tok, n, b, ob, tid, NT);
}

bool topb_supported(const Layout& lay, int b, float lambda) {
  return lambda == 0.0f && lay.n > 256 && lay.n <= 32 * kTopbThreads && b <= kTopbMaxB;
}

hipError_t launch_select_topb(const void* K, const void* V, const float* s, const Layout& lay, int b,
                              int32_t* idx_sorted, int32_t* pick_order, float* pick_gain, void* K_out,
                              void* V_out, hipStream_t st, const int32_t* b_h) {
  TopbArgs a;
  a.b_h = b_h;
  a.K = static_cast<const char*>(K); a.V = static_cast<const char*>(V); a.s_in = s;
  a.idx_sorted = idx_sorted; a.pick_order = pick_order; a.pick_gain = pick_gain;
  a.K_out = static_cast<char*>(K_out); a.V_out = static_cast<char*>(V_out);
  a.stride_head = lay.stride_head; a.stride_tok = lay.stride_tok;
  a.n = lay.n; a.b = b;
  if ((K_out || V_out) && lay.dtype != DT_BF16) return hipErrorInvalidValue;   // rows are copied as bf16 rows
  auto go = [&](auto kern, int slots) -> hipError_t {
    const int smem = (16 + 2 * slots * (kTopbThreads / 64) + 4 * b) * 4;
    hipLaunchKernelGGL(kern, dim3(lay.heads), dim3(kTopbThreads), smem, st, a);
    return hipGetLastError();
  };
  if (lay.n <= 4 * kTopbThreads) return go(&select_topb_kernel<4>, 4);
  if (lay.n <= 8 * kTopbThreads) return go(&select_topb_kernel<8>, 8);
  if (lay.n <= 16 * kTopbThreads) return go(&select_topb_kernel<16>, 16);
  return go(&select_topb_kernel<32>, 32);
}

}  // namespace kvr
