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
//
// Inside the flat-mode event the rows of tokens that can never be selected are not computed:
// while fewer than b tokens are selected one of the b best-scored is free and gains at least
// s_(b) - lambda (Eq. 2, a cosine is at most 1), a token gains at most its score, so a token with
// s_j < s_(b) - lambda never wins Eq. 3 and its signature row is never needed.  flat_bound_kernel
// finds that threshold per sequence; the signature kernel then skips such tokens' loads and writes
// zero rows for them (cosine 0 to everything: harmless wherever a later kernel still looks at them).
#include "kvr_device.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

constexpr int kSigThreads = 512;
constexpr int kSigTok = 4;                     // tokens per workgroup
constexpr int kSigSlices = kSigThreads / (16 * kSigTok);   // slices of the group per token

// thr[seq * thr_stride] = s_(b) - lambda (minus a margin for fp32 cosines a few ulp above 1), s_(b) from
// the leading 16 bits of the ordered keys (at most s_(b): the bound only loosens).  One workgroup of WV waves
// per sequence: the keys of up to 64 * NQ * WV tokens sit in registers, a wave's count is NQ ballots, and with
// more than one wave the counts meet in LDS once per bit.
template <int NQ, int WV>
__global__ __launch_bounds__(64 * WV) void flat_bound_kernel(const float* __restrict__ s, int n, int b, float lambda,
                                                             float* __restrict__ thr, int thr_stride) {
  __shared__ int cnt_l[2][WV];
  const int seq = blockIdx.x, tid = threadIdx.x, wave = tid >> 6;
  const float* sh = s + static_cast<long long>(seq) * n;
  uint32_t k[NQ];
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int j = tid + 64 * WV * q;
    k[q] = j < n ? ordered_key(sh[j] + 0.0f) : 0u;
  }
  uint32_t T = 0;
  int par = 0;
  for (int bit = 31; bit >= 16; --bit) {
    const uint32_t cand = T | (1u << bit);
    int tot = 0;
#pragma unroll
    for (int q = 0; q < NQ; ++q) tot += __popcll(__ballot(k[q] >= cand));
    if constexpr (WV > 1) {
      if ((tid & 63) == 0) cnt_l[par][wave] = tot;
      __syncthreads();
      tot = 0;
#pragma unroll
      for (int u = 0; u < WV; ++u) tot += cnt_l[par][u];
      par ^= 1;
    }
    if (tot >= b) T = cand;
  }
  if (tid == 0) {
    const float sb = key_to_float(T);
    thr[static_cast<long long>(seq) * thr_stride] = sb - lambda * 1.00001f - 1e-5f * fabsf(sb);
  }
}

template <int DT>
__global__ __launch_bounds__(kSigThreads) void signature_flat_kernel(const char* __restrict__ V, Layout lay,
                                                                     int group, float* __restrict__ u_out,
                                                                     const float* __restrict__ s,
                                                                     const float* __restrict__ thr, int thr_stride) {
  __shared__ float part[kSigSlices][kSigTok * 16][8];
  const int seq = blockIdx.y;
  const int tid = threadIdx.x;
  const int chunk = tid & 15, tk = (tid >> 4) & (kSigTok - 1), slice = tid / (kSigTok * 16);
  const int tok = blockIdx.x * kSigTok + tk;
  constexpr int eb = DT == DT_BF16 ? 2 : 4;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  // (a token below its sequence's threshold keeps a zero row; a NaN score or threshold keeps the token)
  const bool live = tok < lay.n && !(s && s[static_cast<long long>(seq) * lay.n + tok] < thr[static_cast<long long>(seq) * thr_stride]);
  if (live) {
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

hipError_t launch_signature_flat(const void* V, const Layout& lay, int group, float* u_out, hipStream_t st,
                                 const float* s, int b, float lambda, float* thr, int thr_stride) {
  const int seqs = lay.heads / group;
  if (s) {                                         // the rows of tokens the score bound rules out stay zero
    auto go = [&](auto kern, int threads) {
      hipLaunchKernelGGL(kern, dim3(seqs), dim3(threads), 0, st, s, lay.n, b, lambda, thr, thr_stride);
    };
    if (lay.n <= 512) go(&flat_bound_kernel<8, 1>, 64);
    else if (lay.n <= 2048) go(&flat_bound_kernel<8, 4>, 256);
    else go(&flat_bound_kernel<32, 4>, 256);         // (n <= 8192 is checked by the entry points)
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  dim3 grid((lay.n + kSigTok - 1) / kSigTok, seqs);
  if (lay.dtype == DT_BF16)
    hipLaunchKernelGGL((signature_flat_kernel<DT_BF16>), grid, dim3(kSigThreads), 0, st,
                       static_cast<const char*>(V), lay, group, u_out, s, thr, thr_stride);
  else
    hipLaunchKernelGGL((signature_flat_kernel<DT_F32>), grid, dim3(kSigThreads), 0, st,
                       static_cast<const char*>(V), lay, group, u_out, s, thr, thr_stride);
  return hipGetLastError();
}

}  // namespace kvr
