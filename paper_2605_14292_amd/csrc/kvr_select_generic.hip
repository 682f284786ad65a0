// Algorithm 1 of paper Sec. 4.1, one workgroup per head, for any n up to
// KVR_MAX_N: the similarity row of each pick is computed when the pick is made
// (only the b rows Algorithm 1 reads of its n x n cosine matrix), the running
// maximum m and the scores live in LDS, and each pick is a workgroup-wide
// argmax of a 64-bit (gain, ~index) key.  This is the shape-agnostic path; the
// shapes of the benchmark configurations have faster kernels of their own.
#include "kvr_device.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

constexpr int kSelThreads = 256;

template <int DT>
__global__ __launch_bounds__(kSelThreads) void select_generic_kernel(
    const void* __restrict__ V, const float* __restrict__ s, Layout lay, int b, float lambda,
    float eps, int32_t* __restrict__ idx_sorted, int32_t* __restrict__ pick_order,
    float* __restrict__ pick_gain) {
  extern __shared__ float smem[];
  const int n = lay.n;
  const int nwords = (n + 31) >> 5;
  unsigned long long* red = reinterpret_cast<unsigned long long*>(smem);   // [4] wave maxima
  float* sc = smem + 8;                     // [n] scores
  float* m = sc + n;                        // [n] running max cosine (floored at 0)
  float* r = m + n;                         // [n] 1/(||V_j|| + eps)
  float* vi = r + n;                        // [128] current pick's row times r_i
  uint32_t* selw = reinterpret_cast<uint32_t*>(vi + kD);          // [nwords] selected bits
  uint32_t* woff = selw + nwords;                                  // [nwords] prefix counts

  const int h = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 15, rsub = tid >> 4;
  const char* Vh = static_cast<const char*>(V) + h * lay.stride_head * elem_bytes<DT>();
  const float* sh = s + static_cast<long long>(h) * n;
  const bool diverse = lambda != 0.0f;      // lambda == 0: explicit top-b branch, V untouched

  for (int j = tid; j < n; j += kSelThreads) { sc[j] = sh[j]; m[j] = 0.f; }
  for (int w = tid; w < nwords; w += kSelThreads) selw[w] = 0u;
  if (diverse) {
    for (int j0 = 0; j0 < n; j0 += kSelThreads / 16) {
      const int j = j0 + rsub;
      if (j < n) {
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
    for (int j = tid; j < n; j += kSelThreads) {
      if (!((selw[j >> 5] >> (j & 31)) & 1u)) {
        const float a = diverse ? fmaf(-lambda, m[j], sc[j]) : sc[j];
        const unsigned long long k = pack_key(a, j);
        best = k > best ? k : best;
      }
    }
    best = wave_max_u64(best);
    if (lane == 0) red[wave] = best;
    __syncthreads();
    {
      const unsigned long long k01 = red[0] > red[1] ? red[0] : red[1];
      const unsigned long long k23 = red[2] > red[3] ? red[2] : red[3];
      best = k01 > k23 ? k01 : k23;
    }
    const int i = key_index(best);
    if (tid == 0) {
      selw[i >> 5] |= 1u << (i & 31);
      if (pick_order) pick_order[static_cast<long long>(h) * b + t] = i;
      if (pick_gain) pick_gain[static_cast<long long>(h) * b + t] = key_gain(best);
    }
    if (t + 1 == b || !diverse) { __syncthreads(); continue; }
    // row of the pick: cos(v_i, v_j) for every j, folded into m
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
    for (int j0 = 0; j0 < n; j0 += kSelThreads / 16) {
      const int j = j0 + rsub;
      if (j < n) {
        float x[8];
        load8<DT>(Vh + (static_cast<long long>(j) * lay.stride_tok + c * 8) * elem_bytes<DT>(), x);
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) dot = fmaf(x[e], y[e], dot);
        dot = group16_sum(dot);
        if (c == 0) m[j] = fmaxf(m[j], dot * r[j]);
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
  const size_t smem = (8 + 3 * static_cast<size_t>(lay.n) + kD + 2 * static_cast<size_t>(nwords)) * 4;
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
