// Algorithm 1 of paper Sec. 4.1, one workgroup per head, for any n up to
// KVR_MAX_N: the similarity row of each pick is computed when the pick is made
// (only the b rows Algorithm 1 reads of its n x n cosine matrix), the running
// maximum m and the scores live in LDS, and each pick is a workgroup-wide
// argmax of a 64-bit (gain, ~index) key.  This is the shape-agnostic path; the
// shapes of the benchmark configurations have faster kernels of their own.
//
// Before anything of V is read the candidates are reduced, exactly: while fewer than b
// tokens are selected one of the b best-scored is free and gains at least s_(b) - lambda
// (Eq. 2, a cosine is at most 1), and a token gains at most its score, so a token with
// s_j < s_(b) - lambda never wins Eq. 3.  Only the others (in token order, so ties break as
// before) take part in the argmax and have their cosines computed.  With scores that spread
// by more than lambda this leaves a small part of a long head; with scores far below lambda
// it leaves everything.
#include "kvr_device.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelRows = kSelThreads / 16;   // rows per step of a pass: 16 lanes per row
constexpr int kSelBatch = 4;                 // steps whose loads are issued together

template <int DT>
__global__ __launch_bounds__(kSelThreads) void select_generic_kernel(
    const void* __restrict__ V, const float* __restrict__ s, Layout lay, int b, float lambda,
    float eps, int32_t* __restrict__ idx_sorted, int32_t* __restrict__ pick_order,
    float* __restrict__ pick_gain) {
  extern __shared__ float smem[];
  const int n = lay.n;
  const int nwords = (n + 31) >> 5;
  unsigned long long* red = reinterpret_cast<unsigned long long*>(smem);   // [16] wave maxima
  int32_t* cnt_l = reinterpret_cast<int32_t*>(smem + 32);                  // [2][16] wave counts, [32] the number of candidates
  float* sc = smem + 72;                    // [n] scores
  float* m = sc + n;                        // [n] running max cosine (floored at 0)
  float* r = m + n;                         // [n] 1/(||V_j|| + eps)
  float* vi = r + n;                        // [128] current pick's row times r_i
  uint32_t* selw = reinterpret_cast<uint32_t*>(vi + kD);          // [nwords] selected bits
  uint32_t* woff = selw + nwords;                                  // [nwords] prefix counts
  int32_t* live = reinterpret_cast<int32_t*>(woff + nwords);      // [n] the candidates, ascending

  const int h = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 15, rsub = tid >> 4;
  const char* Vh = static_cast<const char*>(V) + h * lay.stride_head * elem_bytes<DT>();
  const float* sh = s + static_cast<long long>(h) * n;
  const bool diverse = lambda != 0.0f;      // lambda == 0: explicit top-b branch, V untouched

  for (int j = tid; j < n; j += kSelThreads) { sc[j] = sh[j]; m[j] = 0.f; }
  for (int w = tid; w < nwords; w += kSelThreads) selw[w] = 0u;
  __syncthreads();
  // ---- s_(b) from the leading 16 bits of the ordered keys (at most s_(b): the bound only loosens)
  uint32_t T = 0;
  {
    int par = 0;
    for (int bit = 31; bit >= 16; --bit) {
      const uint32_t cand = T | (1u << bit);
      int cnt = 0;
      for (int j = tid; j < n; j += kSelThreads) cnt += ordered_key(sc[j] + 0.0f) >= cand ? 1 : 0;
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) cnt += __shfl_xor(cnt, off, kWave);
      if (lane == 0) cnt_l[par * 16 + wave] = cnt;
      __syncthreads();
      int tot = 0;
#pragma unroll
      for (int w = 0; w < kSelWaves; ++w) tot += cnt_l[par * 16 + w];
      par ^= 1;
      if (tot >= b) T = cand;
    }
  }
  const float sb = key_to_float(T);
  const float thr = sb - lambda * 1.00001f - 1e-5f * fabsf(sb);   // fp32 cosines may exceed 1 by a few ulp
  // ---- the candidates in token order (one wave: ballots and prefix counts, 64 tokens a step)
  if (wave == 0) {
    int base = 0;
    for (int j0 = 0; j0 < n; j0 += kWave) {
      const int j = j0 + lane;
      const bool keep = j < n && !(sc[j] < thr);       // a NaN threshold or score keeps the token
      const unsigned long long mask = __ballot(keep);
      if (keep) live[base + __popcll(mask & ((1ull << lane) - 1ull))] = j;
      base += __popcll(mask);
    }
    if (lane == 0) cnt_l[32] = base;
  }
  __syncthreads();
  const int nl = cnt_l[32];                  // >= b: the b best-scored tokens are among them
  if (diverse) {
    for (int u0 = 0; u0 < nl; u0 += kSelRows) {
      const int u = u0 + rsub;
      if (u < nl) {
        const int j = live[u];
        float x[8];
        load8<DT>(Vh + (static_cast<long long>(j) * lay.stride_tok + c * 8) * elem_bytes<DT>(), x);
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = fmaf(x[e], x[e], ss);
        ss = group16_sum(ss);
        if (c == 0) r[j] = 1.0f / (sqrtf(ss) + eps);
      }
    }
  }
  __syncthreads();

  for (int t = 0; t < b; ++t) {
    unsigned long long best = 0ull;
    for (int u = tid; u < nl; u += kSelThreads) {
      const int j = live[u];
      if (!((selw[j >> 5] >> (j & 31)) & 1u)) {
        const float a = diverse ? fmaf(-lambda, m[j], sc[j]) : sc[j];
        const unsigned long long k = pack_key(a, j);
        best = k > best ? k : best;
      }
    }
    best = wave_max_u64(best);
    if (lane == 0) red[wave] = best;
    __syncthreads();
    best = red[0];
#pragma unroll
    for (int w = 1; w < kSelWaves; ++w) best = red[w] > best ? red[w] : best;
    const int i = key_index(best);
    if (tid == 0) {
      selw[i >> 5] |= 1u << (i & 31);
      if (pick_order) pick_order[static_cast<long long>(h) * b + t] = i;
      if (pick_gain) pick_gain[static_cast<long long>(h) * b + t] = key_gain(best);
    }
    if (t + 1 == b || !diverse) { __syncthreads(); continue; }
    // row of the pick: cos(v_i, v_j) for every candidate j, folded into m
    if (tid < 16) {
      float x[8];
      load8<DT>(Vh + (static_cast<long long>(i) * lay.stride_tok + tid * 8) * elem_bytes<DT>(), x);
      const float ri = r[i];
#pragma unroll
      for (int e = 0; e < 8; ++e) vi[tid * 8 + e] = x[e] * ri;
    }
    __syncthreads();
    float y[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) y[e] = vi[c * 8 + e];
    for (int u0 = 0; u0 < nl; u0 += kSelRows * kSelBatch) {
      float x[kSelBatch][8];                      // the loads of a batch are issued before the first is used
      int jq[kSelBatch];
#pragma unroll
      for (int q = 0; q < kSelBatch; ++q) {
        const int u = u0 + q * kSelRows + rsub;
        jq[q] = u < nl ? live[u] : -1;
        load8<DT>(Vh + (static_cast<long long>(jq[q] < 0 ? 0 : jq[q]) * lay.stride_tok + c * 8) * elem_bytes<DT>(), x[q]);
      }
#pragma unroll
      for (int q = 0; q < kSelBatch; ++q) {
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) dot = fmaf(x[q][e], y[e], dot);
        dot = group16_sum(dot);
        if (c == 0 && jq[q] >= 0) m[jq[q]] = fmaxf(m[jq[q]], dot * r[jq[q]]);
      }
    }
    __syncthreads();
  }

  // sort(S): ascending indices from the selected bits (prefix popcount)
  if (tid == 0) {
    uint32_t run = 0;
    for (int w = 0; w < nwords; ++w) { woff[w] = run; run += __popc(selw[w]); }
  }
  __syncthreads();
  int32_t* out = idx_sorted + static_cast<long long>(h) * b;
  for (int w = tid; w < nwords; w += kSelThreads) {
    uint32_t bits = selw[w];
    uint32_t o = woff[w];
    while (bits) {
      const int bit = __ffs(bits) - 1;
      bits &= bits - 1;
      if (o < static_cast<uint32_t>(b)) out[o] = w * 32 + bit;
      ++o;
    }
  }
}

hipError_t launch_select_generic(const void* V, const float* s, const Layout& lay, int b,
                                 float lambda, float eps, int32_t* idx_sorted,
                                 int32_t* pick_order, float* pick_gain, hipStream_t st) {
  const int nwords = (lay.n + 31) >> 5;
  const size_t smem = (72 + 4 * static_cast<size_t>(lay.n) + kD + 2 * static_cast<size_t>(nwords)) * 4;
  dim3 grid(lay.heads), block(kSelThreads);
  hipError_t e;
  if (lay.dtype == DT_BF16) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&select_generic_kernel<DT_BF16>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(smem));
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((select_generic_kernel<DT_BF16>), grid, block, smem, st, V, s, lay, b,
                       lambda, eps, idx_sorted, pick_order, pick_gain);
  } else {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&select_generic_kernel<DT_F32>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(smem));
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((select_generic_kernel<DT_F32>), grid, block, smem, st, V, s, lay, b,
                       lambda, eps, idx_sorted, pick_order, pick_gain);
  }
  return hipGetLastError();
}

}  // namespace kvr
