// Base scores: s_i = (1/G) sum_g softmax_i(q_g . k_i / sqrt(d)).
// (Stand-in for the external scorer of paper Sec. 4.1, which takes s as given.)
//
// One workgroup per head.  A group of 16 lanes owns one K row per step (16
// bytes of bf16 or 32 bytes of fp32 per lane, so a wave reads four whole rows
// with one coalesced request); the query slices a lane needs stay in
// registers.  The logits of the head are kept in LDS when G*n floats fit, so K
// is read from HBM exactly once; otherwise the logits are recomputed in a
// second pass.
#include "kvr_device.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

constexpr int kScoreThreads = 256;
constexpr int kGT = 8;                       // queries handled per register tile
constexpr int kZMaxFloats = 16384;           // logits kept in LDS (64 KB)

template <int DT>
__device__ __forceinline__ void row_logits(const char* Kh, long long stride_tok, int j, int c,
                                           const float (&q)[kGT][8], int gcount, float scale,
                                           float (&z)[kGT]) {
  float k[8];
  load8<DT>(Kh + (static_cast<long long>(j) * stride_tok + c * 8) * elem_bytes<DT>(), k);
#pragma unroll
  for (int g = 0; g < kGT; ++g) {
    float acc = 0.f;
    if (g < gcount) {
#pragma unroll
      for (int e = 0; e < 8; ++e) acc = fmaf(k[e], q[g][e], acc);
      acc = group16_sum(acc) * scale;
    }
    z[g] = acc;
  }
}

template <int DT, bool ZFITS>
__global__ __launch_bounds__(kScoreThreads) void score_kernel(const void* __restrict__ K,
                                                              const void* __restrict__ Q, int G,
                                                              Layout lay,
                                                              float* __restrict__ s_out) {
  extern __shared__ float smem[];
  // smem: zbuf[G*n] (ZFITS) | acc[n] ; then red[2*kGT*4]
  const int n = lay.n;
  float* zbuf = smem;                                 // ZFITS: [G][n]
  float* acc = smem + (ZFITS ? G * n : 0);            // [n] running mean
  float* red = acc + n;                               // [4 waves][kGT] x2
  const int h = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 15;                            // 16-byte chunk of the row
  const int rsub = tid >> 4;                          // row within a step (0..15)
  const char* Kh = static_cast<const char*>(K) + h * lay.stride_head * elem_bytes<DT>();
  const char* Qh = static_cast<const char*>(Q) +
                   static_cast<long long>(h) * G * kD * elem_bytes<DT>();
  const float scale = 0.08838834764831845f;           // 1/sqrt(128)
  const float invG = 1.0f / static_cast<float>(G);

  for (int j = tid; j < n; j += kScoreThreads) acc[j] = 0.f;

  for (int g0 = 0; g0 < G; g0 += kGT) {
    const int gcount = min(kGT, G - g0);
    float q[kGT][8];
#pragma unroll
    for (int g = 0; g < kGT; ++g) {
      if (g < gcount) {
        load8<DT>(Qh + (static_cast<long long>(g0 + g) * kD + c * 8) * elem_bytes<DT>(), q[g]);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) q[g][e] = 0.f;
      }
    }
    // pass A: logits, running max per query
    float zmax[kGT];
#pragma unroll
    for (int g = 0; g < kGT; ++g) zmax[g] = -INFINITY;
    for (int j0 = 0; j0 < n; j0 += kScoreThreads / 16) {
      const int j = j0 + rsub;
      if (j < n) {
        float z[kGT];
        row_logits<DT>(Kh, lay.stride_tok, j, c, q, gcount, scale, z);
#pragma unroll
        for (int g = 0; g < kGT; ++g) {
          zmax[g] = fmaxf(zmax[g], z[g]);
          if (ZFITS && c == 0 && g < gcount) zbuf[(g0 + g) * n + j] = z[g];
        }
      }
    }
    // block max per query
#pragma unroll
    for (int g = 0; g < kGT; ++g) {
      float v = zmax[g];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
      if (lane == 0) red[wave * kGT + g] = v;
    }
    __syncthreads();
#pragma unroll
    for (int g = 0; g < kGT; ++g)
      zmax[g] = fmaxf(fmaxf(red[g], red[kGT + g]), fmaxf(red[2 * kGT + g], red[3 * kGT + g]));
    __syncthreads();
    // pass B: sum of exp per query
    float zsum[kGT];
#pragma unroll
    for (int g = 0; g < kGT; ++g) zsum[g] = 0.f;
    if (ZFITS) {
      for (int j = tid; j < n; j += kScoreThreads) {
#pragma unroll
        for (int g = 0; g < kGT; ++g)
          if (g < gcount) {
            const float e = __expf(zbuf[(g0 + g) * n + j] - zmax[g]);
            zbuf[(g0 + g) * n + j] = e;
            zsum[g] += e;
          }
      }
    } else {
      for (int j0 = 0; j0 < n; j0 += kScoreThreads / 16) {
        const int j = j0 + rsub;
        if (j < n) {
          float z[kGT];
          row_logits<DT>(Kh, lay.stride_tok, j, c, q, gcount, scale, z);
          if (c == 0) {
#pragma unroll
            for (int g = 0; g < kGT; ++g)
              if (g < gcount) zsum[g] += __expf(z[g] - zmax[g]);
          }
        }
      }
    }
#pragma unroll
    for (int g = 0; g < kGT; ++g) {
      float v = zsum[g];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
      if (lane == 0) red[wave * kGT + g] = v;
    }
    __syncthreads();
    float rinv[kGT];
#pragma unroll
    for (int g = 0; g < kGT; ++g)
      rinv[g] = 1.0f / (red[g] + red[kGT + g] + red[2 * kGT + g] + red[3 * kGT + g]);
    __syncthreads();
    // pass C: accumulate the mean of the softmax rows
    if (ZFITS) {
      for (int j = tid; j < n; j += kScoreThreads) {
        float a = acc[j];
#pragma unroll
        for (int g = 0; g < kGT; ++g)
          if (g < gcount) a = fmaf(zbuf[(g0 + g) * n + j], rinv[g] * invG, a);
        acc[j] = a;
      }
    } else {
      for (int j0 = 0; j0 < n; j0 += kScoreThreads / 16) {
        const int j = j0 + rsub;
        if (j < n) {
          float z[kGT];
          row_logits<DT>(Kh, lay.stride_tok, j, c, q, gcount, scale, z);
          if (c == 0) {
            float a = acc[j];
#pragma unroll
            for (int g = 0; g < kGT; ++g)
              if (g < gcount) a = fmaf(__expf(z[g] - zmax[g]), rinv[g] * invG, a);
            acc[j] = a;
          }
        }
      }
    }
    __syncthreads();
  }
  float* so = s_out + static_cast<long long>(h) * n;
  for (int j = tid; j < n; j += kScoreThreads) so[j] = acc[j];
}

// ---------------------------------------------------------------------------
// bf16, G <= 32 (GQ = 8 or 32 query rows of the MFMA's 32-row operand in use): the logits are a thin dense contraction ([G x d] x [d x n]), so
// they go through the matrix cores.  K is streamed from HBM once, straight into MFMA
// operand registers.  The logits of the head wait in LDS for the softmax.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

template <int GQ, int NW>
__global__ __launch_bounds__(64 * NW) void score_mfma_kernel(const char* __restrict__ K,
                                                                   const char* __restrict__ Q, int G,
                                                                   Layout lay,
                                                                   float* __restrict__ s_out) {
  extern __shared__ __align__(16) char smem_raw[];
  float* zbuf = reinterpret_cast<float*>(smem_raw);                         // [G][n]
  const int n = lay.n;
  float* red = zbuf + G * n;                                                // [2][NW][GQ]
  const int h = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const char* Kh = K + h * lay.stride_head * 2;
  bf16x8 qf[8];
  {
    const int g = lane & 31;
    const char* qp = Q + (static_cast<long long>(h) * G + g) * kD * 2 + hf * 16;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      uint4 w = make_uint4(0u, 0u, 0u, 0u);
      if (g < G) w = *reinterpret_cast<const uint4*>(qp + ks * 32);
      qf[ks] = *reinterpret_cast<bf16x8*>(&w);
    }
  }
  // Wave w takes the 32-token tiles w, w+NW, ...: the rows go straight into the registers in the
  // MFMA operand layout (lane l: token l % 32, eight consecutive k at 8 * (l / 32) per step; the
  // two halves of a row are 32 contiguous bytes per request), the next tile is in flight while
  // the current one is multiplied, and no wave waits for another until the softmax.
  const int ntiles = (n + 31) >> 5;
  const long long tok_bytes = lay.stride_tok * 2;
  bf16x8 kf[8], kn[8];
  auto fetch = [&](int t, bf16x8 (&dst)[8]) {
    const char* p = Kh + min(t * 32 + (lane & 31), n - 1) * tok_bytes + hf * 16;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const uint4 w = *reinterpret_cast<const uint4*>(p + ks * 32);
      dst[ks] = *reinterpret_cast<const bf16x8*>(&w);
    }
  };
  const float scale = 0.08838834764831845f;
  if (wave < ntiles) fetch(wave, kf);
  for (int t = wave; t < ntiles; t += NW) {
    if (t + NW < ntiles) fetch(t + NW, kn);
    f32x16 acc = {0};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[ks], kf[ks], acc, 0, 0, 0);
    const int j = t * 32 + (lane & 31);
    if (j < n) {
      // lane (token, hf) holds query rows (r/4)*8 + hf*4 + r%4 of the 32x32 tile
#pragma unroll
      for (int r = 0; r < GQ / 2; ++r) {
        const int g = (r >> 2) * 8 + hf * 4 + (r & 3);
        if (g < G) zbuf[g * n + j] = acc[r] * scale;
      }
    }
    if (t + NW < ntiles) {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) kf[ks] = kn[ks];
    }
  }
  __syncthreads();
  // softmax over the tokens for each query, then the mean over queries
  float zmax[GQ], zsum[GQ];
#pragma unroll
  for (int g = 0; g < GQ; ++g) { zmax[g] = -INFINITY; zsum[g] = 0.f; }
  for (int j = tid; j < n; j += 64 * NW)
#pragma unroll
    for (int g = 0; g < GQ; ++g)
      if (g < G) zmax[g] = fmaxf(zmax[g], zbuf[g * n + j]);
#pragma unroll
  for (int g = 0; g < GQ; ++g) {
    float v = zmax[g];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    if (lane == 0) red[wave * GQ + g] = v;
  }
  __syncthreads();
#pragma unroll
  for (int g = 0; g < GQ; ++g) {
    float v = red[g];
#pragma unroll
    for (int u = 1; u < NW; ++u) v = fmaxf(v, red[u * GQ + g]);
    zmax[g] = v;
  }
  for (int j = tid; j < n; j += 64 * NW)
#pragma unroll
    for (int g = 0; g < GQ; ++g)
      if (g < G) {
        const float e = __expf(zbuf[g * n + j] - zmax[g]);
        zbuf[g * n + j] = e;
        zsum[g] += e;
      }
#pragma unroll
  for (int g = 0; g < GQ; ++g) {
    float v = zsum[g];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
    if (lane == 0) red[(NW + wave) * GQ + g] = v;
  }
  __syncthreads();
  const float invG = 1.0f / static_cast<float>(G);
  float wgt[GQ];
#pragma unroll
  for (int g = 0; g < GQ; ++g) {
    float v = red[NW * GQ + g];
#pragma unroll
    for (int u = 1; u < NW; ++u) v += red[(NW + u) * GQ + g];
    wgt[g] = invG / v;
  }
  float* so = s_out + static_cast<long long>(h) * n;
  for (int j = tid; j < n; j += 64 * NW) {
    float p = 0.f;
#pragma unroll
    for (int g = 0; g < GQ; ++g)
      if (g < G) p = fmaf(zbuf[g * n + j], wgt[g], p);
    so[j] = p;
  }
}

hipError_t launch_score(const void* K, const void* Q, int G, const Layout& lay, float* s_out,
                        hipStream_t st) {
  // the logits of a head (G x n floats) wait in LDS
  if (lay.dtype == DT_BF16 && G <= 32 && static_cast<long long>(G) * lay.n <= (G <= 8 ? 24576 : 31488)) {
    const int gq = G <= 8 ? 8 : 32;
    // The logit buffer sets how many workgroups share a CU; when it leaves room for two or fewer, eight waves per
    // workgroup keep as many rows in flight as four waves do with a small buffer.
    const int smem_one = (G * lay.n + 8 * gq) * 4;
    const bool big = 3 * smem_one > 160 * 1024;
    const int nw = big ? 8 : 4;
    const int smem_m = (G * lay.n + 2 * nw * gq) * 4;
    auto go_m = [&](auto kern) -> hipError_t {
      const hipError_t em = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, smem_m);
      if (em != hipSuccess) return em;
      hipLaunchKernelGGL(kern, dim3(lay.heads), dim3(64 * nw), smem_m, st,
                         static_cast<const char*>(K), static_cast<const char*>(Q), G, lay, s_out);
      return hipGetLastError();
    };
    if (big) return gq == 8 ? go_m(&score_mfma_kernel<8, 8>) : go_m(&score_mfma_kernel<32, 8>);
    return gq == 8 ? go_m(&score_mfma_kernel<8, 4>) : go_m(&score_mfma_kernel<32, 4>);
  }
  if (score_wide_supported(lay, G)) return launch_score_wide(K, Q, G, lay, s_out, st);
  const bool zfits = static_cast<long long>(G) * lay.n <= kZMaxFloats;
  const size_t smem = (static_cast<size_t>(zfits ? G * lay.n : 0) + lay.n + 2 * kGT * 4) * 4;
  dim3 grid(lay.heads), block(kScoreThreads);
  auto go = [&](auto kern) -> hipError_t {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize,
                                             static_cast<int>(smem));
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, block, smem, st, K, Q, G, lay, s_out);
    return hipSuccess;
  };
  hipError_t e;
  if (lay.dtype == DT_BF16) e = zfits ? go(&score_kernel<DT_BF16, true>) : go(&score_kernel<DT_BF16, false>);
  else e = zfits ? go(&score_kernel<DT_F32, true>) : go(&score_kernel<DT_F32, false>);
  if (e != hipSuccess) return e;
  return hipGetLastError();
}

}  // namespace kvr
