// Flat V-signature of paper Eq. 1: u_i = (1/(L*H)) sum over layers and heads of V_i, one [n, d]
// matrix per sequence (the normalisation to v_i = u_i/(||u_i|| + eps) happens inside the
// selection kernel, which takes u as its rows).  The L*H heads of a sequence are `group`
// consecutive heads of the [heads, n, d] tensor.
//
// HBM-bound streaming reduction: a workgroup owns four tokens of one sequence; its 256 threads
// are 4 tokens x 16 column chunks (eight elements each) x 4 slices of the group, every thread
// sums its slice in fp32 with eight loads in flight, the four slices meet in LDS.
#include "kvr_device.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

constexpr int kSigThreads = 256;
constexpr int kSigTok = 4;                     // tokens per workgroup
constexpr int kSigSlices = 4;                  // slices of the group per token

template <int DT>
__global__ __launch_bounds__(kSigThreads) void signature_flat_kernel(const char* __restrict__ V, Layout lay,
                                                                     int group, float* __restrict__ u_out) {
  __shared__ float part[kSigSlices][kSigTok * 16][8];
  const int seq = blockIdx.y;
  const int tid = threadIdx.x;
  const int chunk = tid & 15, tk = (tid >> 4) & (kSigTok - 1), slice = tid >> 6;
  const int tok = blockIdx.x * kSigTok + tk;
  constexpr int eb = DT == DT_BF16 ? 2 : 4;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (tok < lay.n) {
    const char* p = V + ((static_cast<long long>(seq) * group) * lay.stride_head +
                         static_cast<long long>(tok) * lay.stride_tok + chunk * 8) * eb;
    const long long hstep = lay.stride_head * eb;
    int g = slice;
    for (; g + 7 * kSigSlices < group; g += 8 * kSigSlices) {
      float x[8][8];
#pragma unroll
      for (int u = 0; u < 8; ++u) load8<DT>(p + (g + u * kSigSlices) * hstep, x[u]);
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += x[u][e];
    }
    for (; g < group; g += kSigSlices) {
      float x[8];
      load8<DT>(p + g * hstep, x);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += x[e];
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[slice][tid & 63][e] = acc[e];
  __syncthreads();
  if (slice == 0 && tok < lay.n) {
    const float inv = 1.0f / static_cast<float>(group);
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e)
      o[e] = ((part[0][tid][e] + part[1][tid][e]) + (part[2][tid][e] + part[3][tid][e])) * inv;
    float* dst = u_out + (static_cast<long long>(seq) * lay.n + tok) * kD + chunk * 8;
    *reinterpret_cast<float4*>(dst) = make_float4(o[0], o[1], o[2], o[3]);
    *reinterpret_cast<float4*>(dst + 4) = make_float4(o[4], o[5], o[6], o[7]);
  }
}

hipError_t launch_signature_flat(const void* V, const Layout& lay, int group, float* u_out, hipStream_t st) {
  const int seqs = lay.heads / group;
  dim3 grid((lay.n + kSigTok - 1) / kSigTok, seqs);
  if (lay.dtype == DT_BF16)
    hipLaunchKernelGGL((signature_flat_kernel<DT_BF16>), grid, dim3(kSigThreads), 0, st,
                       static_cast<const char*>(V), lay, group, u_out);
  else
    hipLaunchKernelGGL((signature_flat_kernel<DT_F32>), grid, dim3(kSigThreads), 0, st,
                       static_cast<const char*>(V), lay, group, u_out);
  return hipGetLastError();
}

}  // namespace kvr
