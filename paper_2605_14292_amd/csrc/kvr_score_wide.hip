// Base scores from a wide observation window: s_i = (1/G) sum_g softmax_i(q_g . k_i / sqrt(d))
// for up to 256 queries per KV head (an observation window of W recent positions times
// the grouped query heads, the scorer family the paper compares against and builds on,
// Sec. 2 and Sec. 4.1's "external scorer"), bf16, any n.
//
// G x n logits do not fit LDS here, so the softmax is taken in two passes over K, both on
// the matrix cores (32x32x16 bf16, fp32 accumulate), and no logit is ever stored:
//   pass 1: per query, the running maximum and the sum of exponentials (kept per lane);
//   pass 2: the logits again, p = exp(z - max)/sum, summed over the queries.
// The two operands of the MFMA have the same register layout (lane l: row or column
// l % 32, eight consecutive k at 8 * (l / 32)), so pass 1 puts the tokens on the rows and
// the queries on the columns -- a lane then owns one query and its statistics need no
// cross-lane traffic until the end -- and pass 2 swaps them: a lane owns one token and
// the sum over queries is a sum over its own registers.
// One workgroup per head; wave w takes the 32-token tiles w, w+4, ...; the queries wait
// in LDS (272-byte pitch).  Everything is done in base 2: z2 = z * log2(e).
// Bound: for G of a few dozen the two reads of K (fabric rate); for G = 256 the matrix
// cores and the vector ALU together -- a 32x32 block costs 8 MFMAs and about 60 vector
// instructions (16 of them exponentials) per pass, the two kinds of work share the SIMD's
// issue port and overlap only partly across waves (measured on this chip: a wave of MFMA
// chains beside a wave of fma+exp+add on one SIMD takes 0.76 of the sum of their times).
// Variants measured and not kept because they change nothing: query fragments prefetched
// one block ahead, two token tiles per query fragment (half the LDS reads, independent
// accumulator chains), sixteen waves per workgroup.
#include "kvr_dense_common.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

constexpr int kWideThreads = 256;
constexpr int kWideMaxBlocks = 8;             // query blocks of 32: G <= 256
constexpr int kWidePitch = 272;

__host__ __device__ constexpr int wide_smem_bytes(int gb) {
  // queries | c[gb*32] | per-wave max [4][gb*32] | per-wave sum [4][gb*32]
  return gb * 32 * kWidePitch + gb * 32 * 4 * 9;
}

__global__ __launch_bounds__(kWideThreads, 2) void score_wide_kernel(const char* __restrict__ K,
                                                                     const char* __restrict__ Q, int G,
                                                                     Layout lay, float* __restrict__ s_out) {
  extern __shared__ __align__(16) char smem_raw[];
  const int GB = (G + 31) >> 5;
  const int GP = GB * 32;
  char* q_l = smem_raw;
  float* c_l = reinterpret_cast<float*>(smem_raw + GP * kWidePitch);   // [GP] max2 + log2(sum), +inf for padding
  float* pm = c_l + GP;                                                 // [4][GP]
  float* pl = pm + 4 * GP;                                              // [4][GP]
  const int n = lay.n;
  const int h = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, l32 = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const char* Kh = K + h * lay.stride_head * 2;
  const long long tok_bytes = lay.stride_tok * 2;
  const int ntiles = (n + 31) >> 5;
  const float sc2 = 0.08838834764831845f * 1.4426950408889634f;        // log2(e) / sqrt(128)

  // ---- queries -> LDS, rows past G zero
  {
    const int c16 = tid & 15, r0 = tid >> 4;
    const char* Qh = Q + static_cast<long long>(h) * G * kD * 2;
    for (int g = r0; g < GP; g += kWideThreads / 16) {
      uint4 w = make_uint4(0u, 0u, 0u, 0u);
      if (g < G) w = *reinterpret_cast<const uint4*>(Qh + g * (kD * 2) + c16 * 16);
      *reinterpret_cast<uint4*>(q_l + g * kWidePitch + c16 * 16) = w;
    }
  }
  __syncthreads();

  bf16x8 kf[8], kn[8];
  auto fetch = [&](int t, bf16x8 (&dst)[8]) {
    const char* p = Kh + min(t * 32 + l32, n - 1) * tok_bytes + hf * 16;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const uint4 w = *reinterpret_cast<const uint4*>(p + ks * 32);
      dst[ks] = *reinterpret_cast<const bf16x8*>(&w);
    }
  };
  const char* qp = q_l + l32 * kWidePitch + hf * 16;

  // ================= pass 1: per-query maximum and sum =================
  float m2[kWideMaxBlocks], l2[kWideMaxBlocks];
#pragma unroll
  for (int qb = 0; qb < kWideMaxBlocks; ++qb) { m2[qb] = -INFINITY; l2[qb] = 0.f; }
  if (wave < ntiles) fetch(wave, kf);
  for (int t = wave; t < ntiles; t += 4) {
    if (t + 4 < ntiles) fetch(t + 4, kn);
    const bool ragged = t * 32 + 32 > n;
#pragma unroll
    for (int qb = 0; qb < kWideMaxBlocks; ++qb) {
      if (qb < GB) {
        f32x16 acc = {0};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              kf[ks], *reinterpret_cast<const bf16x8*>(qp + qb * 32 * kWidePitch + ks * 32), acc, 0, 0, 0);
        // lane (query l32, hf) holds token rows (r/4)*8 + hf*4 + r%4 of the tile
        if (ragged) {
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (t * 32 + (r >> 2) * 8 + hf * 4 + (r & 3) >= n) acc[r] = -INFINITY;
        }
        float amax = acc[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) amax = fmaxf(amax, acc[r]);
        const float mnew = fmaxf(m2[qb], amax * sc2);
        const float msafe = mnew == -INFINITY ? 0.f : mnew;
        float sum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(fmaf(acc[r], sc2, -msafe));
        l2[qb] = fmaf(l2[qb], __builtin_amdgcn_exp2f(m2[qb] - msafe), sum);
        m2[qb] = mnew;
      }
    }
    if (t + 4 < ntiles) {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) kf[ks] = kn[ks];
    }
  }
  // the two half-waves of a query, then the four waves
#pragma unroll
  for (int qb = 0; qb < kWideMaxBlocks; ++qb) {
    if (qb < GB) {
      const float mo = __shfl_xor(m2[qb], 32, kWave), lo = __shfl_xor(l2[qb], 32, kWave);
      const float mm = fmaxf(m2[qb], mo);
      const float ms = mm == -INFINITY ? 0.f : mm;
      const float ll = l2[qb] * __builtin_amdgcn_exp2f(m2[qb] - ms) + lo * __builtin_amdgcn_exp2f(mo - ms);
      if (hf == 0) { pm[wave * GP + qb * 32 + l32] = mm; pl[wave * GP + qb * 32 + l32] = ll; }
    }
  }
  __syncthreads();
  for (int g = tid; g < GP; g += kWideThreads) {
    float mm = fmaxf(fmaxf(pm[g], pm[GP + g]), fmaxf(pm[2 * GP + g], pm[3 * GP + g]));
    float ll = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) ll += pl[w * GP + g] * __builtin_amdgcn_exp2f(pm[w * GP + g] - mm);
    c_l[g] = g < G ? mm + __builtin_amdgcn_logf(ll) : INFINITY;
  }
  __syncthreads();

  // ================= pass 2: probabilities, summed over the queries =================
  const float invG = 1.0f / static_cast<float>(G);
  float* so = s_out + static_cast<long long>(h) * n;
  if (wave < ntiles) fetch(wave, kf);
  for (int t = wave; t < ntiles; t += 4) {
    if (t + 4 < ntiles) fetch(t + 4, kn);
    float colsum = 0.f;
#pragma unroll
    for (int qb = 0; qb < kWideMaxBlocks; ++qb) {
      if (qb < GB) {
        f32x16 acc = {0};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              *reinterpret_cast<const bf16x8*>(qp + qb * 32 * kWidePitch + ks * 32), kf[ks], acc, 0, 0, 0);
        // lane (token l32, hf) holds query rows (r/4)*8 + hf*4 + r%4 of the block
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const float4 c = *reinterpret_cast<const float4*>(c_l + qb * 32 + r4 * 8 + hf * 4);
          colsum += __builtin_amdgcn_exp2f(fmaf(acc[r4 * 4 + 0], sc2, -c.x));
          colsum += __builtin_amdgcn_exp2f(fmaf(acc[r4 * 4 + 1], sc2, -c.y));
          colsum += __builtin_amdgcn_exp2f(fmaf(acc[r4 * 4 + 2], sc2, -c.z));
          colsum += __builtin_amdgcn_exp2f(fmaf(acc[r4 * 4 + 3], sc2, -c.w));
        }
      }
    }
    colsum += __shfl_xor(colsum, 32, kWave);
    const int j = t * 32 + l32;
    if (hf == 0 && j < n) so[j] = colsum * invG;
    if (t + 4 < ntiles) {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) kf[ks] = kn[ks];
    }
  }
}

bool score_wide_supported(const Layout& lay, int G) {
  return lay.dtype == DT_BF16 && G >= 1 && G <= 32 * kWideMaxBlocks;
}

hipError_t launch_score_wide(const void* K, const void* Q, int G, const Layout& lay, float* s_out,
                             hipStream_t st) {
  const int smem = wide_smem_bytes((G + 31) / 32);
  const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_wide_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(score_wide_kernel, dim3(lay.heads), dim3(kWideThreads), smem, st,
                     static_cast<const char*>(K), static_cast<const char*>(Q), G, lay, s_out);
  return hipGetLastError();
}

}  // namespace kvr
