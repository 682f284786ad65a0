// Token-axis pooling of the base scores: the smoothing step of observation-window
// scorers (the scorer family of paper Sec. 2; Sec. 4.1 takes s as given and the paper
// does not restate the step).  s_out[i] = max, or mean, of s_in over the window of
// `kernel` tokens centred on i.  Window positions outside the head are skipped by the
// maximum and count as zeros in the mean, whose divisor is always `kernel`.
// One lane per token; the window is read straight from global memory (L1 serves it).
#include "kvr_device.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

constexpr int kPoolThreads = 256;

__global__ __launch_bounds__(kPoolThreads) void score_pool_kernel(const float* __restrict__ s_in, int n,
                                                                  int half, int mean, float* __restrict__ s_out) {
  const int i = blockIdx.x * kPoolThreads + threadIdx.x;
  if (i >= n) return;
  const float* sh = s_in + static_cast<long long>(blockIdx.y) * n;
  const int lo = max(i - half, 0), hi = min(i + half, n - 1);
  float v;
  if (mean) {
    v = 0.f;
    for (int j = lo; j <= hi; ++j) v += sh[j];
    v /= static_cast<float>(2 * half + 1);
  } else {
    v = sh[lo];
    for (int j = lo + 1; j <= hi; ++j) v = fmaxf(v, sh[j]);
  }
  s_out[static_cast<long long>(blockIdx.y) * n + i] = v;
}

hipError_t launch_score_pool(const float* s_in, int heads, int n, int kernel, int mean, float* s_out,
                             hipStream_t st) {
  hipLaunchKernelGGL(score_pool_kernel, dim3((n + kPoolThreads - 1) / kPoolThreads, heads), dim3(kPoolThreads),
                     0, st, s_in, n, kernel / 2, mean, s_out);
  return hipGetLastError();
}

}  // namespace kvr
