// Cache update of paper Sec. 4.1 / Algorithm 1's return value: keep the rows
// at the ascending selected indices, bit for bit.  A group of 16 (bf16) or 32 (fp32)
// lanes moves one row in 16-byte units, so a wave moves whole rows per request and
// the dense output is written fully coalesced.
#include "kvr_device.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

constexpr int kCompactThreads = 256;

constexpr int kCompactUnits = 4;   // 16-byte units per thread, tensor and batch

__global__ __launch_bounds__(kCompactThreads) void compact_kernel(
    const char* __restrict__ K, const char* __restrict__ V, Layout lay, int ebytes,
    const int32_t* __restrict__ idx, int idx_group, int b, char* __restrict__ K_out,
    char* __restrict__ V_out) {
  const int h = blockIdx.x;
  const int tid = threadIdx.x;
  const int32_t* il = idx + static_cast<long long>(h / idx_group) * b;   // idx_group heads share one index row
  const int cpr_shift = ebytes == 2 ? 4 : 5;               // 16-byte units per row: d = 128
  const int total = b << cpr_shift;
  const long long head_off = h * lay.stride_head * ebytes;
  const long long tok_bytes = lay.stride_tok * ebytes;
  const long long out_off = static_cast<long long>(h) * total * 16;
  // one workgroup per head; every thread has its batch of loads in flight before the first store
  for (int u0 = 0; u0 < total; u0 += kCompactThreads * kCompactUnits) {
    uint4 xk[kCompactUnits], xv[kCompactUnits];
#pragma unroll
    for (int k = 0; k < kCompactUnits; ++k) {
      const int u = min(u0 + k * kCompactThreads + tid, total - 1);
      const int i = min(max(il[u >> cpr_shift], 0), lay.n - 1);
      const long long src = head_off + i * tok_bytes + (u & ((1 << cpr_shift) - 1)) * 16;
      xk[k] = xv[k] = make_uint4(0u, 0u, 0u, 0u);
      if (K) xk[k] = *reinterpret_cast<const uint4*>(K + src);
      if (V) xv[k] = *reinterpret_cast<const uint4*>(V + src);
    }
#pragma unroll
    for (int k = 0; k < kCompactUnits; ++k) {
      const int u = u0 + k * kCompactThreads + tid;
      if (u < total) {
        if (K) *reinterpret_cast<uint4*>(K_out + out_off + u * 16ll) = xk[k];
        if (V) *reinterpret_cast<uint4*>(V_out + out_off + u * 16ll) = xv[k];
      }
    }
  }
}

hipError_t launch_compact(const void* K, const void* V, const Layout& lay, const int32_t* idx,
                          int b, void* K_out, void* V_out, hipStream_t st, int idx_group) {
  const int ebytes = lay.dtype == DT_BF16 ? 2 : 4;
  hipLaunchKernelGGL(compact_kernel, dim3(lay.heads), dim3(kCompactThreads), 0, st,
                     static_cast<const char*>(K), static_cast<const char*>(V), lay, ebytes, idx, idx_group, b,
                     static_cast<char*>(K_out), static_cast<char*>(V_out));
  return hipGetLastError();
}

// The same update done inside the cache's own storage.  The index list of a head is
// strictly ascending (it is sort(S)), so idx[t] >= t: the destination of row t is
// never the source of a later row, and it can only be the source of an earlier
// row of the same batch or of a batch already finished.  One workgroup owns a
// head and moves it in batches of 16-byte units, lowest rows first; inside a
// batch every load has landed in registers, in every wave, before the first
// store is issued.  Entries < 0 (the padding past a head's own budget) move nothing.
constexpr int kInplaceUnits = 4;   // 16-byte units per thread, tensor and batch

__global__ __launch_bounds__(kCompactThreads) void compact_inplace_kernel(
    char* __restrict__ K, char* __restrict__ V, Layout lay, int ebytes, const int32_t* __restrict__ idx,
    int idx_group, int b, int32_t* __restrict__ pos) {
  const int h = blockIdx.x;
  const int tid = threadIdx.x;
  const int32_t* il = idx + static_cast<long long>(h / idx_group) * b;
  const int cpr_shift = ebytes == 2 ? 4 : 5;               // 16-byte units per row: d = 128
  const int total = b << cpr_shift;
  const long long head_off = h * lay.stride_head * ebytes;
  const long long tok_bytes = lay.stride_tok * ebytes;
  if (K || V) {
    for (int u0 = 0; u0 < total; u0 += kCompactThreads * kInplaceUnits) {
      uint4 xk[kInplaceUnits], xv[kInplaceUnits];
      long long dst[kInplaceUnits];
      bool move[kInplaceUnits];
#pragma unroll
      for (int k = 0; k < kInplaceUnits; ++k) {
        const int u = u0 + k * kCompactThreads + tid;
        const int t = min(u, total - 1) >> cpr_shift;
        const int c = u & ((1 << cpr_shift) - 1);
        const int i = il[t];
        move[k] = u < total && i >= 0 && i != t;
        const long long src = head_off + min(max(i, 0), lay.n - 1) * tok_bytes + c * 16;
        dst[k] = head_off + t * tok_bytes + c * 16;
        xk[k] = xv[k] = make_uint4(0u, 0u, 0u, 0u);
        if (K) xk[k] = *reinterpret_cast<const uint4*>(K + src);
        if (V) xv[k] = *reinterpret_cast<const uint4*>(V + src);
      }
      __syncthreads();                                     // waits for the loads, then for every wave
#pragma unroll
      for (int k = 0; k < kInplaceUnits; ++k) {
        if (move[k]) {
          if (K) *reinterpret_cast<uint4*>(K + dst[k]) = xk[k];
          if (V) *reinterpret_cast<uint4*>(V + dst[k]) = xv[k];
        }
      }
    }
  }
  if (pos) {
    int32_t* pl = pos + static_cast<long long>(h) * lay.n;
    for (int t0 = 0; t0 < b; t0 += kCompactThreads) {
      const int t = t0 + tid;
      const int i = t < b ? il[t] : -1;
      const int32_t p = pl[min(max(i, 0), lay.n - 1)];
      __syncthreads();
      if (i >= 0 && i != t) pl[t] = p;
    }
  }
}

hipError_t launch_compact_inplace(void* K, void* V, const Layout& lay, const int32_t* idx, int idx_group,
                                  int b, int32_t* pos, hipStream_t st) {
  const int ebytes = lay.dtype == DT_BF16 ? 2 : 4;
  hipLaunchKernelGGL(compact_inplace_kernel, dim3(lay.heads), dim3(kCompactThreads), 0, st,
                     static_cast<char*>(K), static_cast<char*>(V), lay, ebytes, idx, idx_group, b, pos);
  return hipGetLastError();
}

}  // namespace kvr
