// Algorithm 1 (paper Sec. 4.1) inside a budget allocator's frame: per-head candidate counts
// n_h, per-head budgets b_h and protected tokens (attention sinks, a recent window) that are
// members of S from the start.  Two small kernels wrap the ordinary selection kernels:
//
//   prepare   s'_j = -inf for j >= n_h (not a candidate); s'_j = s_j + C for protected tokens,
//             with C larger than the spread of the head's scores plus lambda.  Under Eq. 2-3 every
//             protected token then wins before any other one, so after |protected| picks S is the
//             protected set and m holds its penalties, whatever the order they went in; from
//             there the picks are exactly Algorithm 1's continuation.
//             A per-head lambda_h is folded in here too: the argmax of s - lambda_h m is the
//             argmax of (lambda/lambda_h) s - lambda m, so the head's scores are scaled and the
//             kernels run with the one lambda of the launch; finalize scales the gains back.
//   finalize  Algorithm 1's picks for budget b_h are the first b_h picks of the run for
//             b_max >= b_h (each pick depends on the earlier ones only): the first b_h picks are
//             flagged in a bitmap, read out ascending, and the rows (and position ids) at those
//             indices are copied.
#include "kvr_device.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

constexpr int kBudThreads = 256;

// One wave per head (four heads per workgroup): no LDS, no barrier.
__global__ __launch_bounds__(kBudThreads) void budget_prepare_kernel(
    const float* s_src, int heads, int n, const int32_t* __restrict__ n_h,
    const uint8_t* __restrict__ keep, const float* __restrict__ lambda_h, float lambda,
    float* s_work) {                             // s_work may be s_src (scores computed in place)
  const int lane = threadIdx.x & 63;
  const int h = blockIdx.x * (kBudThreads / 64) + (threadIdx.x >> 6);
  if (h >= heads) return;
  const long long base = static_cast<long long>(h) * n;
  const int nh = n_h ? min(max(n_h[h], 0), n) : n;
  const float sc = lambda_h ? lambda / lambda_h[h] : 1.0f;     // lambda_h > 0 by contract
  float lo = INFINITY, hi = -INFINITY;
  for (int j = lane; j < nh; j += kWave) {
    const float v = s_src[base + j] * sc;
    if (v > -INFINITY && v < INFINITY) { lo = fminf(lo, v); hi = fmaxf(hi, v); }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    lo = fminf(lo, __shfl_xor(lo, off, kWave));
    hi = fmaxf(hi, __shfl_xor(hi, off, kWave));
  }
  // no finite score: any offset will do (the picks are unspecified then)
  const float C = hi >= lo ? ((hi - lo) + lambda + 1.0f) * 1.001f : 1.0f;
  for (int j = lane; j < n; j += kWave) {
    float v = -INFINITY;
    if (j < nh) {
      v = s_src[base + j] * sc;
      if (keep && keep[base + j]) v += C;
    }
    s_work[base + j] = v;
  }
}

__global__ __launch_bounds__(kBudThreads) void budget_finalize_kernel(
    const char* __restrict__ K, const char* __restrict__ V, Layout lay, int ebytes,
    const int32_t* __restrict__ b_h, int b_max, const uint8_t* __restrict__ keep,
    const float* __restrict__ lambda_h, float lambda, const int32_t* __restrict__ pos_in, int32_t* __restrict__ idx_sorted,
    int32_t* __restrict__ pick_order, float* __restrict__ pick_gain, char* __restrict__ K_out,
    char* __restrict__ V_out, int32_t* __restrict__ pos_out) {
  extern __shared__ __align__(16) int32_t sm[];
  const int n = lay.n, words = (n + 31) >> 5;
  uint32_t* bits = reinterpret_cast<uint32_t*>(sm);            // [words] picked-token bitmap
  int32_t* wbase = sm + words;                                 // [words] tokens picked before each word
  int32_t* il = wbase + words;                                 // [b_max] ascending kept indices
  const int h = blockIdx.x, tid = threadIdx.x;
  const long long ob = static_cast<long long>(h) * b_max;
  const int bh = b_h ? min(max(b_h[h], 0), b_max) : b_max;
  const float unscale = lambda_h ? lambda_h[h] / lambda : 1.0f;
  for (int w = tid; w < words; w += kBudThreads) bits[w] = 0u;
  for (int t = tid; t < b_max; t += kBudThreads) il[t] = -1;
  __syncthreads();
  for (int t = tid; t < b_max; t += kBudThreads) {
    const int i = pick_order[ob + t];
    if (t < bh) {
      if (i >= 0 && i < n) atomicOr(&bits[i >> 5], 1u << (i & 31));
      if (pick_gain) {
        if (keep && i >= 0 && i < n && keep[static_cast<long long>(h) * n + i])
          pick_gain[ob + t] = INFINITY;                        // kept unconditionally, not by its gain
        else if (lambda_h)
          pick_gain[ob + t] *= unscale;                        // back to s - lambda_h m
      }
    } else {
      pick_order[ob + t] = -1;
      if (pick_gain) pick_gain[ob + t] = -INFINITY;
    }
  }
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int w = 0; w < words; ++w) { wbase[w] = run; run += __popc(bits[w]); }
  }
  __syncthreads();
  for (int w = tid; w < words; w += kBudThreads) {
    uint32_t m = bits[w];
    int r = wbase[w];
    while (m) {
      const int bit = __ffs(static_cast<int>(m)) - 1;
      m &= m - 1;
      if (r < b_max) il[r] = w * 32 + bit;
      ++r;
    }
  }
  __syncthreads();
  for (int t = tid; t < b_max; t += kBudThreads) {
    const int i = t < bh ? il[t] : -1;
    idx_sorted[ob + t] = i;
    if (pos_out) pos_out[ob + t] = (i >= 0 && pos_in) ? pos_in[static_cast<long long>(h) * n + i] : -1;
  }
  // rows of the kept tokens: 16 threads per row, two rows per thread in flight
  const int row_bytes = lay.d * ebytes;
  const int chunk = tid & 15, g = tid >> 4, G = kBudThreads / 16;
  const long long hoff = h * lay.stride_head * ebytes;
  for (int first = 0; first < bh; first += 2 * G) {
    for (int o = chunk * 16; o < row_bytes; o += 256) {
      uint4 kr[2], vr[2];
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int t = min(first + g + k * G, bh - 1);
        const long long src = hoff + min(max(il[t], 0), n - 1) * lay.stride_tok * ebytes + o;   // never outside the head
        kr[k] = vr[k] = make_uint4(0u, 0u, 0u, 0u);
        if (K_out) kr[k] = *reinterpret_cast<const uint4*>(K + src);
        if (V_out) vr[k] = *reinterpret_cast<const uint4*>(V + src);
      }
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int t = first + g + k * G;
        if (t < bh) {
          const long long dst = (ob + t) * row_bytes + o;
          if (K_out) *reinterpret_cast<uint4*>(K_out + dst) = kr[k];
          if (V_out) *reinterpret_cast<uint4*>(V_out + dst) = vr[k];
        }
      }
    }
  }
}

// After the kernels that take the per-head budgets themselves (they write the ascending index
// lists, the padding and the kept rows): what is left is elementwise -- a protected token's gain
// reads +inf, gains computed at the launch lambda go back to the head's own, position ids follow
// the kept indices.
__global__ __launch_bounds__(kBudThreads) void budget_fixup_kernel(
    int n, int b_max, long long total, const uint8_t* __restrict__ keep, const float* __restrict__ lambda_h,
    float lambda, const int32_t* __restrict__ pos_in, const int32_t* __restrict__ idx_sorted,
    const int32_t* __restrict__ pick_order, float* __restrict__ pick_gain, int32_t* __restrict__ pos_out) {
  const long long e = static_cast<long long>(blockIdx.x) * kBudThreads + threadIdx.x;
  if (e >= total) return;
  const long long h = e / b_max;
  if (pick_gain && (keep || lambda_h)) {
    const int i = pick_order[e];
    if (i >= 0 && i < n) {
      if (keep && keep[h * n + i]) pick_gain[e] = INFINITY;
      else if (lambda_h) pick_gain[e] *= lambda_h[h] / lambda;
    }
  }
  if (pos_out) {
    const int i = idx_sorted[e];
    pos_out[e] = (i >= 0 && i < n && pos_in) ? pos_in[h * n + i] : -1;
  }
}

hipError_t launch_budget_fixup(const Layout& lay, int b_max, const uint8_t* keep, const float* lambda_h,
                               float lambda, const int32_t* pos_in, const int32_t* idx_sorted,
                               const int32_t* pick_order, float* pick_gain, int32_t* pos_out, hipStream_t st) {
  if (!(pick_gain && (keep || lambda_h)) && !pos_out) return hipSuccess;     // nothing to fix up
  const long long total = static_cast<long long>(lay.heads) * b_max;
  hipLaunchKernelGGL(budget_fixup_kernel, dim3(static_cast<unsigned>((total + kBudThreads - 1) / kBudThreads)),
                     dim3(kBudThreads), 0, st, lay.n, b_max, total, keep, lambda_h, lambda, pos_in, idx_sorted,
                     pick_order, pick_gain, pos_out);
  return hipGetLastError();
}

hipError_t launch_budget_prepare(const float* s_src, const Layout& lay, const int32_t* n_h,
                                 const uint8_t* keep, const float* lambda_h, float lambda, float* s_work,
                                 hipStream_t st) {
  hipLaunchKernelGGL(budget_prepare_kernel, dim3((lay.heads + kBudThreads / 64 - 1) / (kBudThreads / 64)),
                     dim3(kBudThreads), 0, st, s_src, lay.heads, lay.n, n_h, keep, lambda_h, lambda, s_work);
  return hipGetLastError();
}

hipError_t launch_budget_finalize(const void* K, const void* V, const Layout& lay, const int32_t* b_h,
                                  int b_max, const uint8_t* keep, const float* lambda_h, float lambda,
                                  const int32_t* pos_in, int32_t* idx_sorted, int32_t* pick_order,
                                  float* pick_gain, void* K_out, void* V_out, int32_t* pos_out,
                                  hipStream_t st) {
  const int words = (lay.n + 31) >> 5;
  const size_t smem = (2 * static_cast<size_t>(words) + b_max) * 4;
  const int ebytes = lay.dtype == DT_BF16 ? 2 : 4;
  hipLaunchKernelGGL(budget_finalize_kernel, dim3(lay.heads), dim3(kBudThreads), smem, st,
                     static_cast<const char*>(K), static_cast<const char*>(V), lay, ebytes, b_h, b_max, keep,
                     lambda_h, lambda, pos_in, idx_sorted, pick_order, pick_gain, static_cast<char*>(K_out),
                     static_cast<char*>(V_out), pos_out);
  return hipGetLastError();
}

}  // namespace kvr
