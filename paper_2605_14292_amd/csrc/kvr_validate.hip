// Optional debug validator: scans the inputs of a retention event (rows of K and V, queries,
// scores) for NaN and +-inf.  Algorithm 1 (paper Sec. 4.1) is defined on finite scores and
// rows; the selection kernels promise only distinct, in-range indices for anything else, so a
// caller that wants to know asks here first.  Not on the hot path: the entry point
// synchronises the stream and reads one flag back.
#include "kvr_device.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

static __device__ unsigned int g_nonfinite = 0;

__global__ void nonfinite_clear_kernel() { g_nonfinite = 0u; }

// rows [heads][rows_per_head][128] of bf16 (DT_BF16) or fp32: 16-byte pieces, one per thread and step
__global__ __launch_bounds__(256) void nonfinite_rows_kernel(const char* __restrict__ p, int dtype, int rows_per_head,
                                                             long long stride_head_b, long long stride_row_b) {
  const int pieces = dtype == DT_BF16 ? 16 : 32;                 // per row
  const long long total = static_cast<long long>(rows_per_head) * pieces;
  const char* ph = p + blockIdx.y * stride_head_b;
  bool bad = false;
  for (long long u = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x; u < total;
       u += static_cast<long long>(gridDim.x) * 256) {
    const long long row = u / pieces;
    const int piece = static_cast<int>(u % pieces);
    const uint4 x = *reinterpret_cast<const uint4*>(ph + row * stride_row_b + piece * 16);
    const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (dtype == DT_BF16) {
        bad = bad || ((w[q] & 0x7f80u) == 0x7f80u) || ((w[q] & 0x7f800000u) == 0x7f800000u);
      } else {
        bad = bad || ((w[q] & 0x7f800000u) == 0x7f800000u);
      }
    }
  }
  if (bad) g_nonfinite = 1u;                                     // (a plain vector store: every writer writes the same value)
}

__global__ __launch_bounds__(256) void nonfinite_f32_kernel(const float* __restrict__ p, long long count) {
  bool bad = false;
  for (long long u = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x; u < count;
       u += static_cast<long long>(gridDim.x) * 256)
    bad = bad || ((__float_as_uint(p[u]) & 0x7f800000u) == 0x7f800000u);
  if (bad) g_nonfinite = 1u;
}

// found: 1 when any scanned value is NaN or +-inf.  Synchronises `st`.
hipError_t validate_finite(const void* K, const void* V, const void* Q, int G, const float* s, const Layout& lay,
                           hipStream_t st, int* found) {
  hipLaunchKernelGGL(nonfinite_clear_kernel, dim3(1), dim3(1), 0, st);
  const int eb = lay.dtype == DT_BF16 ? 2 : 4;
  const long long per_head = static_cast<long long>(lay.n) * (lay.dtype == DT_BF16 ? 16 : 32);
  const int gx = static_cast<int>(per_head / 256 < 1 ? 1 : (per_head / 256 > 64 ? 64 : per_head / 256));
  for (const void* rows : {K, V})
    if (rows)
      hipLaunchKernelGGL(nonfinite_rows_kernel, dim3(gx, lay.heads), dim3(256), 0, st, static_cast<const char*>(rows),
                         lay.dtype, lay.n, lay.stride_head * eb, lay.stride_tok * eb);
  if (Q)
    hipLaunchKernelGGL(nonfinite_rows_kernel, dim3(1, lay.heads), dim3(256), 0, st, static_cast<const char*>(Q),
                       lay.dtype, G, static_cast<long long>(G) * lay.d * eb, static_cast<long long>(lay.d) * eb);
  if (s) {
    const long long count = static_cast<long long>(lay.heads) * lay.n;
    const int g = static_cast<int>(count / 1024 < 1 ? 1 : (count / 1024 > 2048 ? 2048 : count / 1024));
    hipLaunchKernelGGL(nonfinite_f32_kernel, dim3(g), dim3(256), 0, st, s, count);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  e = hipStreamSynchronize(st);
  if (e != hipSuccess) return e;
  unsigned int v = 0;
  e = hipMemcpyFromSymbol(&v, HIP_SYMBOL(g_nonfinite), sizeof(v));
  *found = v != 0;
  return e;
}

}  // namespace kvr
