// Fused retention step for long bf16 heads (256 < n <= 4096, 2 <= b <= 128, lambda > 0) whose scores
// are handed in and spread by more than lambda: the head shrinks to the tokens that can ever be picked
// before a single row of V is read.
//
// While fewer than b tokens are selected, one of the b best-scored tokens is still free and gains at
// least s_(b) - lambda (a cosine is at most 1, Eq. 2), and a token gains at most its score, so a token
// with s_j < s_(b) - lambda never wins Eq. 3 (paper Sec. 4.1).  With scores of the paper's regime (of the
// order of lambda or larger; log-normal scores leave 4-16 % of a long head) the survivors fit the fused
// kernel for short heads: their rows are gathered into LDS, the lower-triangular 32x32 tiles of their Gram
// matrix go through the bf16 MFMA into a packed fp32 cosine triangle, one wave runs Algorithm 1's pick
// chain, and the kept rows of K and V are copied out.  Survivors keep their token order, so every tie
// still goes to the lowest token index.
//
// A head with more survivors than the kernel's capacity (128 or 192 tokens) keeps the best-scored of them and
// remembers the best score left out; the run is valid iff that score stays below the gain of the last pick
// (gains never increase, and a token gains at most its score), which is checked when the chain is done.  A head
// that fails the check, or whose cut could not be verified anyway, or with fewer than b candidates (non-finite
// scores), gets idx_sorted[h*b] = -1 and is left to the kernel for long heads, which is launched afterwards on
// the marked heads only.
//
// Layout: persistent workgroups of four wave64s, one head at a time; token j = 256*k + thread in slot k of
// its thread while the scores are searched (coalesced score loads), compacted to positions 0..ns-1 for
// everything after.  The scores of the workgroup's next head travel during the pick chain.
#define KVR_BOUNDS_FILE 3   // ids 3xx of the debug build's bounds checks (kvr_bounds.hpp)
#include "kvr_dense_common.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

struct SparseArgs {
  const char* K; const char* V; const float* s_in;
  int32_t* idx_sorted; int32_t* pick_order; float* pick_gain;
  char* K_out; char* V_out;
  long long stride_head, stride_tok;   // elements
  int n, b, heads;
  float lambda, eps;
  const int32_t* b_h;                  // per-head budgets <= b (output rows stay b apart), or null
};

constexpr int kSpMaxB = 128;
__host__ __device__ constexpr int sparse_smem_bytes(int NT) {
  // region A | s_l[N32] | rinv[N32] | tok_c[N32] | redf[16] redi[16] cnt[64] off[64] meta[32] | idx_l, order_l, gain_l [128]
  return dense_region_a(NT) + NT * 32 * 4 * 3 + 192 * 4 + kSpMaxB * 4 * 3;
}

// NT: capacity 32*NT survivors.  S: score slots per thread, n <= 256*S.
template <int NT, int S>
__global__ __launch_bounds__(kDenseThreads, (NT <= 4 ? 4 : 2)) void retain_sparse_kernel(SparseArgs a) {
  constexpr int N32 = NT * 32;
  constexpr int NQ = NT / 2;                         // tokens per lane in the greedy wave
  constexpr int NTILES = NT * (NT + 1) / 2;          // lower-triangular 32x32 tiles of the survivors' Gram matrix
  constexpr int TPWV = (NTILES + 3) / 4;             // ... per wave
  constexpr int kIters = NT * 32 * 16 / kDenseThreads;
  extern __shared__ __align__(16) char smem[];
  char* stage = smem;                                // gathered rows ...
  float* tri = reinterpret_cast<float*>(smem);       // ... later the packed cosine triangle
  float* s_l = reinterpret_cast<float*>(smem + dense_region_a(NT));
  float* rinv = s_l + N32;
  int32_t* tok_c = reinterpret_cast<int32_t*>(rinv + N32);        // token of a compacted position
  float* redf = reinterpret_cast<float*>(tok_c + N32);           // [2][4] hi | [2][4] lo
  int32_t* redi = reinterpret_cast<int32_t*>(redf + 16);         // [2][4] counts (+ 8 spare)
  int32_t* cnt = redi + 16;                                      // [S][4] survivors per slot and wave
  int32_t* off = cnt + 64;                                       // [S][4] their exclusive prefix
  int32_t* idx_l = off + 64 + 32;
  int32_t* order_l = idx_l + kSpMaxB;
  float* gain_l = reinterpret_cast<float*>(order_l + kSpMaxB);

  const int tid0 = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid0 >> 6);
  const int n = a.n, b = a.b;
  int par = 0;

  float spre[S];                                     // scores of the head about to be processed
  auto prefetch_scores = [&](int hh, int tid) {
    const float* sp = a.s_in + static_cast<long long>(hh) * n;
#pragma unroll
    for (int k = 0; k < S; ++k) spre[k] = k * 256 + tid < n ? sp[k * 256 + tid] : -INFINITY;
  };
  int h = blockIdx.x;
  if (h < a.heads) prefetch_scores(h, tid0);

  for (; h < a.heads; h += gridDim.x) {
    const int h_next = h + gridDim.x;
    const long long head_off = h * a.stride_head * 2;  // bytes
    int tid = tid0;
    asm volatile("" : "+v"(tid));                    // (per-lane LDS addresses are recomputed per head, not kept in registers)
    const int lane = tid & 63, hf = lane >> 5;
    const unsigned long long below = (1ull << lane) - 1ull;
    float sv[S];
#pragma unroll
    for (int k = 0; k < S; ++k) sv[k] = spre[k];
    // the head's own budget: its picks are the first bt picks of a run for b (the rows of the outputs per head); a head
    // with budget 0 still runs one pick, nothing of which is written
    const int bt = a.b_h ? __builtin_amdgcn_readfirstlane(min(max(a.b_h[h], 0), b)) : b;
    const int bq = bt < 1 ? 1 : bt;

    // ------------------------------------------------ the tokens that can ever be picked
    // Nothing can go when the finite scores spread by at most lambda: one min/max settles that.
    bool marked = false;
    {
      float hi = -INFINITY, lo = INFINITY;
#pragma unroll
      for (int k = 0; k < S; ++k)
        if (sv[k] > -INFINITY && sv[k] < INFINITY) { hi = hw_max(hi, sv[k]); lo = fminf(lo, sv[k]); }
      hi = wave_max_uniform(hi);
      lo = -wave_max_uniform(-lo);
      if (lane == 0) { redf[par * 4 + wave] = hi; redf[8 + par * 4 + wave] = lo; }
      lds_barrier();
      float ghi = -INFINITY, glo = INFINITY;
#pragma unroll
      for (int u = 0; u < 4; ++u) { ghi = hw_max(ghi, redf[par * 4 + u]); glo = fminf(glo, redf[8 + par * 4 + u]); }
      par ^= 1;
      marked = __builtin_amdgcn_readfirstlane(ghi - glo > a.lambda ? 0 : 1) != 0;   // also when no score is finite
    }
    int ns = 0;
    unsigned long long km[S];
    float excl = -INFINITY;                          // best score among the candidates left out (none: -inf)
    if (!marked) {
      uint32_t key[S];
#pragma unroll
      for (int k = 0; k < S; ++k) key[k] = k * 256 + tid < n ? ordered_key(sv[k] + 0.0f) : 0u;
      // largest value of the leading 16 key bits that at least `want` keys reach (0 when fewer keys exist)
      auto kth_key16 = [&](int want) -> uint32_t {
        uint32_t T = 0;
        for (int bit = 31; bit >= 16; --bit) {
          const uint32_t cand = T | (1u << bit);
          int c = 0;
#pragma unroll
          for (int k = 0; k < S; ++k) c += __popcll(__ballot(key[k] >= cand));
          if (lane == 0) redi[par * 4 + wave] = c;
          lds_barrier();
          const int tot = redi[par * 4] + redi[par * 4 + 1] + redi[par * 4 + 2] + redi[par * 4 + 3];
          par ^= 1;
          if (tot >= want) T = cand;
        }
        return T;
      };
      // survivors per slot and wave into cnt[], their number over the workgroup returned
      auto count_kept = [&]() -> int {
        int c = 0;
#pragma unroll
        for (int k = 0; k < S; ++k) {
          c += __popcll(km[k]);
          if (lane == 0) cnt[k * 4 + wave] = __popcll(km[k]);
        }
        if (lane == 0) redi[par * 4 + wave] = c;
        lds_barrier();
        const int tot = redi[par * 4] + redi[par * 4 + 1] + redi[par * 4 + 2] + redi[par * 4 + 3];
        par ^= 1;
        return tot;
      };
      // s_(b) from the leading 16 bits of the ordered keys: at most s_(b), so the bound only loosens
      const float sb = key_to_float(kth_key16(bq));
      const float thr = sb - a.lambda * 1.00001f - 1e-5f * fabsf(sb);   // fp32 cosines may exceed 1 by a few ulp
#pragma unroll
      for (int k = 0; k < S; ++k) km[k] = __ballot(k * 256 + tid < n && !(sv[k] < thr));   // (a NaN threshold or score keeps the token)
      ns = count_kept();
      if (ns > N32) {
        // (first the cheap half of the test below: when more than N32 tokens score within a quarter of lambda of
        // s_(b), the best one left out does too, and the second search is not worth running)
        int c = 0;
#pragma unroll
        for (int k = 0; k < S; ++k) c += __popcll(__ballot(k * 256 + tid < n && !(sv[k] < sb - 0.25f * a.lambda)));
        if (lane == 0) redi[par * 4 + wave] = c;
        lds_barrier();
        const int near = redi[par * 4] + redi[par * 4 + 1] + redi[par * 4 + 2] + redi[par * 4 + 3];
        par ^= 1;
        if (near > N32) ns = -1;                       // handed on
      }
      if (ns > N32) {
        // More candidates than fit: the best-scored are kept, cut where the leading 16 key bits change (at most N32
        // of them), and the best score left out is remembered.  Pick gains never increase and a token gains at most
        // its score, so the run is valid iff that score stays below the last pick's gain, which is checked when the
        // chain is done.  That gain is at most s_(b) and in practice a good part of lambda below it: when the score
        // left out lies within a quarter of lambda of s_(b) the chain would be run in vain, and the head is handed
        // on at once (a guess about speed only: either way the picks are exact).
        const uint32_t T2 = kth_key16(N32 + 1);       // > 0: more than N32 keys exist
        const uint32_t cut = T2 + 0x10000u;            // (wraps to 0 only for all-ones keys, NaNs: every token then passes and the head is handed on)
        float ob = -INFINITY;
#pragma unroll
        for (int k = 0; k < S; ++k) {
          const bool in = k * 256 + tid < n && key[k] >= cut;
          if (k * 256 + tid < n && !in) ob = hw_max(ob, sv[k]);
          km[k] = __ballot(in);
        }
        ob = wave_max_uniform(ob);
        if (lane == 0) redf[par * 4 + wave] = ob;      // (exchanged by the barrier inside count_kept, read right after it)
        const int pf = par;
        ns = count_kept();
        excl = hw_max(hw_max(redf[pf * 4], redf[pf * 4 + 1]), hw_max(redf[pf * 4 + 2], redf[pf * 4 + 3]));
        if (!(excl < sb - 0.25f * a.lambda)) ns = N32 + 1;              // hopeless: handed on
      }
      marked = ns > N32 || ns < bq;
    }
    if (marked) {                                    // uniform: every wave takes the same branch
      if (tid == 0) a.idx_sorted[static_cast<long long>(h) * b] = -1;
      if (h_next < a.heads) prefetch_scores(h_next, tid);
      continue;
    }
    // positions in token order: slot k before slot k + 1, wave w before wave w + 1, lane by lane
    if (wave == 0) {
      int v = lane < 4 * S ? cnt[lane] : 0;
      const int own = v;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(v, d, kWave);
        if (lane >= d) v += o;
      }
      off[lane] = v - own;
    }
    lds_barrier();
#pragma unroll
    for (int k = 0; k < S; ++k) {
      if ((km[k] >> lane) & 1ull) {
        const int pos = min(kvr_ix(off[k * 4 + wave] + __popcll(km[k] & below), N32, 301), N32 - 1);   // 301: a survivor's position
        tok_c[pos] = k * 256 + tid;
        s_l[pos] = sv[k];
      }
    }
    if (tid >= ns && tid < N32) { tok_c[tid] = 0; s_l[tid] = -INFINITY; }   // padding never competes
    lds_barrier();

    // ------------------------------------------------ rows of the survivors -> LDS
    {
      uint4 vreg[kIters];
      const int chunk = tid & 15, r0 = tid >> 4;
      const char* vb = a.V + head_off + chunk * 16;
      int trow[kIters];
#pragma unroll
      for (int k = 0; k < kIters; ++k) trow[k] = min(max(kvr_ix(tok_c[r0 + 16 * k], n, 302), 0), n - 1);   // 302: token of a survivor
#pragma unroll
      for (int k = 0; k < kIters; ++k) {
        vreg[k] = make_uint4(0u, 0u, 0u, 0u);        // rows past the survivors read as zero: zero Gram entries
        if (r0 + 16 * k < ns) vreg[k] = *reinterpret_cast<const uint4*>(vb + trow[k] * a.stride_tok * 2);
      }
      store_rows<NT>(stage, tid, vreg);
    }
    lds_barrier();

    // ------------------------------------------------ Gram -> packed cosines
    // The lower-triangular 32x32 tiles are dealt to the four waves in turn (tile t to wave t % 4): a wave keeps
    // at most TPWV accumulators, which is what lets four workgroups of the 128-survivor instance share a CU.
    {
      f32x16 acc[TPWV];
#pragma unroll
      for (int q = 0; q < TPWV; ++q) {
        const int tile = wave + 4 * q;
        acc[q] = f32x16{0};
        if (tile < NTILES) {
          int I = 0;
          while ((I + 1) * (I + 2) / 2 <= tile) ++I;
          const int J = tile - I * (I + 1) / 2;
          __builtin_amdgcn_sched_barrier(0);          // keep one tile's fragment loads in flight, not all of them
#pragma unroll
          for (int ks = 0; ks < 8; ++ks)
            acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_at(stage, I, ks, lane), frag_at(stage, J, ks, lane),
                                                             acc[q], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          if (I == J) {                               // squared norms sit on the diagonal
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int il = (r >> 2) * 8 + hf * 4 + (r & 3);
              if (il == (lane & 31)) rinv[I * 32 + il] = acc[q][r];
            }
          }
        }
      }
      lds_barrier();                                // staged rows are dead from here on
      for (int j = tid; j < N32; j += kDenseThreads) rinv[j] = 1.0f / (sqrtf(rinv[j]) + a.eps);
      lds_barrier();
#pragma unroll
      for (int q = 0; q < TPWV; ++q) {
        const int tile = wave + 4 * q;
        if (tile < NTILES) {
          int I = 0;
          while ((I + 1) * (I + 2) / 2 <= tile) ++I;
          const int J = tile - I * (I + 1) / 2;
          write_cos_tile(tri, rinv, acc[q], I, J, lane);
        }
      }
    }
    lds_barrier();
    if (h_next < a.heads) prefetch_scores(h_next, tid);

    // ------------------------------------------------ greedy on the survivors, then back to token numbers
    if (wave == 0) {
      __builtin_amdgcn_s_setprio(3);                 // the chain goes first when it shares a SIMD with other workgroups' waves
      const float last_g = pick_chain<NQ>(s_l, tri, order_l, gain_l, ns, bq, a.lambda, true, lane);
      __builtin_amdgcn_s_setprio(0);
      sort_picks<NQ>(order_l, idx_l, reinterpret_cast<int32_t*>(rinv), bq, lane, tok_c);   // rinv is dead by now
      // the cut, if there was one, holds when every token left out scores below the last pick's gain
      const bool ok = excl == -INFINITY || excl < last_g - 1e-5f * (fabsf(last_g) + a.lambda);
      if (lane == 0) redi[8] = ok ? 0 : 1;
    }
    lds_barrier();
    const bool redo = redi[8] != 0;                  // the head is left to the kernel for long heads

    // ------------------------------------------------ outputs and compaction
    const long long ob = static_cast<long long>(h) * b;
    for (int t = tid; t < b; t += kDenseThreads) {             // entries past the head's budget are padding
      a.idx_sorted[ob + t] = ((redo && t == 0) || t >= bt) ? -1 : idx_l[t];
      if (a.pick_order) a.pick_order[ob + t] = t < bt ? order_l[t] : -1;
      if (a.pick_gain) a.pick_gain[ob + t] = t < bt ? gain_l[t] : -INFINITY;
    }
    if ((a.K_out || a.V_out) && !redo && bt > 0)
      compact_rows<4>(a.K, a.V, a.K_out, a.V_out, head_off, a.stride_tok, idx_l, n, bt, ob, tid, kDenseThreads);
    lds_barrier();                                   // the lists and tables are reused by the next head
  }
}

KVR_BOUNDS_TU(sparse)

bool sparse_supported(const Layout& lay, int b, float lambda) {
  // (the heads this kernel marks go to the kernel for long heads: its shapes bound this one's)
  return lazy_supported(lay, b, lambda) && b >= 2 && b <= kSpMaxB;
}

hipError_t launch_retain_sparse(const void* K, const void* V, const float* s, const Layout& lay, int b, float lambda,
                                float eps, int32_t* idx_sorted, int32_t* pick_order, float* pick_gain, void* K_out,
                                void* V_out, hipStream_t st, const int32_t* b_h) {
  SparseArgs a;
  a.b_h = b_h;
  a.K = static_cast<const char*>(K); a.V = static_cast<const char*>(V); a.s_in = s;
  a.idx_sorted = idx_sorted; a.pick_order = pick_order; a.pick_gain = pick_gain;
  a.K_out = static_cast<char*>(K_out); a.V_out = static_cast<char*>(V_out);
  a.stride_head = lay.stride_head; a.stride_tok = lay.stride_tok;
  a.n = lay.n; a.b = b; a.heads = lay.heads; a.lambda = lambda; a.eps = eps;
  const int cus = cu_count();
  auto go = [&](auto kern, int smem, int per_cu) -> hipError_t {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    const int blocks = lay.heads < cus * per_cu ? lay.heads : cus * per_cu;   // persistent workgroups
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(kDenseThreads), smem, st, a);
    return hipGetLastError();
  };
  // Capacity by budget: the survivors are the b best-scored tokens and those within lambda below them; 128
  // hold them for budgets up to 64 on scores that spread like the benchmark's, 192 for budgets up to 128.
  const bool small = b <= 64;
  auto by_n = [&](auto nt) -> hipError_t {
    constexpr int NT = decltype(nt)::value;
    constexpr int smem = sparse_smem_bytes(NT);
    constexpr int per_cu = NT <= 4 ? 4 : 2;
    if (lay.n <= 1024) return go(&retain_sparse_kernel<NT, 4>, smem, per_cu);
    if (lay.n <= 2048) return go(&retain_sparse_kernel<NT, 8>, smem, per_cu);
    return go(&retain_sparse_kernel<NT, 16>, smem, per_cu);
  };
  return small ? by_n(std::integral_constant<int, 4>{}) : by_n(std::integral_constant<int, 6>{});
}

}  // namespace kvr
