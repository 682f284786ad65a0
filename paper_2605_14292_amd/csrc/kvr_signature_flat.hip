// Flat V-signature of paper Eq. 1: u_i = (1/(L*H)) sum over layers and heads of V_i, one [n, d]
// matrix per sequence (the normalisation to v_i = u_i/(||u_i|| + eps) happens inside the
// selection kernel, which takes u as its rows).  The L*H heads of a sequence are `group`
// consecutive heads of the [heads, n, d] tensor.
//
// HBM-bound streaming reduction: a workgroup owns four tokens of one sequence (1 KB contiguous
// per head, one wave's request); its 512 threads are 4 tokens x 16 column chunks (eight elements
// each) x 8 slices of the group, every thread sums its slice in fp32 with sixteen loads in flight,
// the slices meet in LDS.  Four tokens rather than eight per workgroup: 1536 workgroups fill the
// resident slots of 256 CUs in whole rounds on the benchmark shape (66-68 us against 76 us).
#include "kvr_device.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

constexpr int kSigThreads = 512;
constexpr int kSigTok = 4;                     // tokens per workgroup
constexpr int kSigSlices = kSigThreads / (16 * kSigTok);   // slices of the group per token

template <int DT>
__global__ __launch_bounds__(kSigThreads) void signature_flat_kernel(const char* __restrict__ V, Layout lay,
                                                                     int group, float* __restrict__ u_out) {
  __shared__ float part[kSigSlices][kSigTok * 16][8];
  const int seq = blockIdx.y;
  const int tid = threadIdx.x;
  const int chunk = tid & 15, tk = (tid >> 4) & (kSigTok - 1), slice = tid / (kSigTok * 16);
  const int tok = blockIdx.x * kSigTok + tk;
  constexpr int eb = DT == DT_BF16 ? 2 : 4;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (tok < lay.n) {
    const char* p = V + ((static_cast<long long>(seq) * group) * lay.stride_head +
                         static_cast<long long>(tok) * lay.stride_tok + chunk * 8) * eb;
    const long long hstep = lay.stride_head * eb;
    // slice k sums heads [k*per, (k+1)*per): neighbouring loads of a thread are one head apart
    const int per = (group + kSigSlices - 1) / kSigSlices;
    int g = slice * per;
    const int gend = min(group, g + per);
    for (; g + 15 < gend; g += 16) {
      uint4 w[16];                                // sixteen loads in flight per thread
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        if constexpr (DT == DT_BF16) w[u] = *reinterpret_cast<const uint4*>(p + (g + u) * hstep);
      }
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        float x[8];
        if constexpr (DT == DT_BF16) {
          x[0] = bf16_lo(w[u].x); x[1] = bf16_hi(w[u].x); x[2] = bf16_lo(w[u].y); x[3] = bf16_hi(w[u].y);
          x[4] = bf16_lo(w[u].z); x[5] = bf16_hi(w[u].z); x[6] = bf16_lo(w[u].w); x[7] = bf16_hi(w[u].w);
        } else {
          load8<DT>(p + (g + u) * hstep, x);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += x[e];
      }
    }
    for (; g < gend; ++g) {
      float x[8];
      load8<DT>(p + g * hstep, x);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += x[e];
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[slice][tid % (kSigTok * 16)][e] = acc[e];
  __syncthreads();
  if (slice == 0 && tok < lay.n) {
    const float inv = 1.0f / static_cast<float>(group);
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float t = part[0][tid][e];
#pragma unroll
      for (int q = 1; q < kSigSlices; ++q) t += part[q][tid][e];
      o[e] = t * inv;
    }
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
