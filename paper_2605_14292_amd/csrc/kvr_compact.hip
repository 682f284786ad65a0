// Cache update of paper Sec. 4.1 / Algorithm 1's return value: keep the rows
// at the ascending selected indices, bit for bit.  A group of 16 lanes moves
// one row (16-byte chunks), so a wave moves four whole rows per request and
// the dense output is written fully coalesced.
#include "kvr_device.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

constexpr int kCompactThreads = 256;

__global__ __launch_bounds__(kCompactThreads) void compact_kernel(
    const char* __restrict__ K, const char* __restrict__ V, Layout lay, int ebytes,
    const int32_t* __restrict__ idx, int idx_group, int b, char* __restrict__ K_out,
    char* __restrict__ V_out) {
  const int h = blockIdx.x;
  const int c = threadIdx.x & 15;
  const int t = blockIdx.y * (kCompactThreads / 16) + (threadIdx.x >> 4);
  if (t >= b) return;
  int i = idx[static_cast<long long>(h / idx_group) * b + t];   // idx_group heads share one index row
  i = min(max(i, 0), lay.n - 1);
  const int row_bytes = lay.d * ebytes;
  const long long src = (h * lay.stride_head + i * lay.stride_tok) * ebytes;
  const long long dst = (static_cast<long long>(h) * b + t) * row_bytes;
  for (int o = c * 16; o < row_bytes; o += 256) {
    if (K) *reinterpret_cast<uint4*>(K_out + dst + o) = *reinterpret_cast<const uint4*>(K + src + o);
    if (V) *reinterpret_cast<uint4*>(V_out + dst + o) = *reinterpret_cast<const uint4*>(V + src + o);
  }
}

hipError_t launch_compact(const void* K, const void* V, const Layout& lay, const int32_t* idx,
                          int b, void* K_out, void* V_out, hipStream_t st, int idx_group) {
  const int ebytes = lay.dtype == DT_BF16 ? 2 : 4;
  dim3 grid(lay.heads, (b + kCompactThreads / 16 - 1) / (kCompactThreads / 16));
  hipLaunchKernelGGL(compact_kernel, grid, dim3(kCompactThreads), 0, st,
                     static_cast<const char*>(K), static_cast<const char*>(V), lay, ebytes, idx, idx_group, b,
                     static_cast<char*>(K_out), static_cast<char*>(V_out));
  return hipGetLastError();
}

}  // namespace kvr
