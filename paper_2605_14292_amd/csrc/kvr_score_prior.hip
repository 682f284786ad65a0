// The one-term modular scoring variant the paper tested and rejected (its table of
// negative gates, scoring family, "variant_b"; discussed again in Sec. 5): the
// cosine of a token's value row with the head's mean value direction, added to the
// base score with a weight,
//   s'_i = s_i + lambda_p * (V_i . dir) / ((||V_i|| + eps) (||dir|| + eps)),
//   dir = (1/n) sum_j V_j.
// One workgroup per head; a group of 16 lanes owns a row (eight elements per lane).
// The mean has to be complete before the first cosine, so the rows are needed
// twice.  KEEP variant: the head's rows stay in the workgroup's registers between
// the two uses (up to 16 rows per lane group: 256 bf16 or 128 fp32 rows), so HBM
// is read once.  Streaming variant (larger heads): two passes over global memory,
// which runs at the fabric's rate; holding a 1024-row head in the registers of a
// 1024-thread workgroup was measured and is no faster (one workgroup per CU, no
// overlap of its load phase with anything).  The column sums are taken in fp64: rows that nearly
// cancel leave a mean whose direction fp32 sums would not determine, and the extra
// arithmetic is hidden behind the loads.
#include "kvr_device.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

template <int DT> struct PriorRaw;
template <> struct PriorRaw<DT_BF16> { uint4 a; };
template <> struct PriorRaw<DT_F32> { float4 a, b; };

template <int DT> __device__ __forceinline__ PriorRaw<DT> prior_load(const char* p) {
  PriorRaw<DT> r;
  if constexpr (DT == DT_BF16) {
    r.a = *reinterpret_cast<const uint4*>(p);
  } else {
    r.a = reinterpret_cast<const float4*>(p)[0];
    r.b = reinterpret_cast<const float4*>(p)[1];
  }
  return r;
}
template <int DT> __device__ __forceinline__ void prior_widen(const PriorRaw<DT>& r, float (&x)[8]) {
  if constexpr (DT == DT_BF16) {
    x[0] = bf16_lo(r.a.x); x[1] = bf16_hi(r.a.x); x[2] = bf16_lo(r.a.y); x[3] = bf16_hi(r.a.y);
    x[4] = bf16_lo(r.a.z); x[5] = bf16_hi(r.a.z); x[6] = bf16_lo(r.a.w); x[7] = bf16_hi(r.a.w);
  } else {
    x[0] = r.a.x; x[1] = r.a.y; x[2] = r.a.z; x[3] = r.a.w;
    x[4] = r.b.x; x[5] = r.b.y; x[6] = r.b.z; x[7] = r.b.w;
  }
}

// rows a lane group holds (KEEP) or has in flight per step (streaming)
template <int DT> constexpr int prior_depth() { return DT == DT_BF16 ? 16 : 8; }

template <int DT, int NT, bool KEEP>
__global__ __launch_bounds__(NT) void score_prior_kernel(
    const char* __restrict__ V, Layout lay, const float* s_in, float lambda_p, float eps, float* s_out) {
  constexpr int EB = elem_bytes<DT>();
  constexpr int ROWS = NT / 16;                  // rows per request of the workgroup
  constexpr int DEPTH = prior_depth<DT>();
  __shared__ double red[NT / 64][kD];
  __shared__ float dir_l[kD];
  const int h = blockIdx.x, tid = threadIdx.x;
  const int c16 = tid & 15, rg = tid >> 4;
  const int n = lay.n;
  const char* Vh = V + h * lay.stride_head * EB + c16 * 8 * EB;
  const long long tok_bytes = lay.stride_tok * EB;
  const float* sh = s_in + static_cast<long long>(h) * n;
  float* so = s_out + static_cast<long long>(h) * n;

  PriorRaw<DT> raw[DEPTH];
  // Lane c of a group handles the score of the group's c-th request of a batch: it reads the
  // base score (before any store of the batch: s_out may be s_in) and writes the result.
  const int jmine = c16 * ROWS + rg;
  float sv = 0.f;
  double acc[8] = {0., 0., 0., 0., 0., 0., 0., 0.};
  auto load_batch = [&](int j0, bool with_scores) {
#pragma unroll
    for (int u = 0; u < DEPTH; ++u) {
      raw[u] = PriorRaw<DT>{};
      if (j0 + u * ROWS < n)                     // uniform: whole requests past the end are skipped
        raw[u] = prior_load<DT>(Vh + min(j0 + u * ROWS + rg, n - 1) * tok_bytes);
    }
    if (with_scores && c16 < DEPTH && j0 + jmine < n) sv = sh[j0 + jmine];
  };
  auto add_batch = [&](int j0) {
#pragma unroll
    for (int u = 0; u < DEPTH; ++u) {
      float x[8];
      prior_widen<DT>(raw[u], x);
      const bool on = j0 + u * ROWS + rg < n;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += on ? static_cast<double>(x[e]) : 0.0;
    }
  };

  // ---- column sums
  if constexpr (KEEP) {
    load_batch(0, true);
    add_batch(0);
  } else {
    for (int j0 = 0; j0 < n; j0 += ROWS * DEPTH) { load_batch(j0, false); add_batch(j0); }
  }
  // the four lane groups of a wave first, then the waves through LDS
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    acc[e] += __shfl_xor(acc[e], 16, kWave);
    acc[e] += __shfl_xor(acc[e], 32, kWave);
  }
  if ((tid & 63) < 16) {
#pragma unroll
    for (int e = 0; e < 8; ++e) red[tid >> 6][c16 * 8 + e] = acc[e];
  }
  __syncthreads();
  if (tid < kD) {
    double t = 0.;
#pragma unroll
    for (int g = 0; g < NT / 64; ++g) t += red[g][tid];
    dir_l[tid] = static_cast<float>(t / static_cast<double>(n));
  }
  __syncthreads();
  float dir[8];
  float dd = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) { dir[e] = dir_l[c16 * 8 + e]; dd = fmaf(dir[e], dir[e], dd); }
  const float rdir = 1.0f / (sqrtf(group16_sum(dd)) + eps);

  // ---- one cosine per row
  auto emit_batch = [&](int j0) {
    float dot_mine = 0.f, ss_mine = 0.f;
#pragma unroll
    for (int u = 0; u < DEPTH; ++u) {
      if constexpr (DT == DT_BF16)   // widen again here rather than keep the fp32 copies of the first use alive
        asm volatile("" : "+v"(raw[u].a.x), "+v"(raw[u].a.y), "+v"(raw[u].a.z), "+v"(raw[u].a.w));
      float x[8];
      prior_widen<DT>(raw[u], x);
      float dot = 0.f, ss = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) { dot = fmaf(x[e], dir[e], dot); ss = fmaf(x[e], x[e], ss); }
      dot = group16_sum(dot);
      ss = group16_sum(ss);
      if (c16 == u) { dot_mine = dot; ss_mine = ss; }
    }
    if (c16 < DEPTH && j0 + jmine < n)
      so[j0 + jmine] = sv + lambda_p * (dot_mine * rdir / (sqrtf(ss_mine) + eps));
  };
  if constexpr (KEEP) {
    emit_batch(0);
  } else {
    for (int j0 = 0; j0 < n; j0 += ROWS * DEPTH) { load_batch(j0, true); emit_batch(j0); }
  }
}

hipError_t launch_score_prior(const void* V, const Layout& lay, const float* s_in, float lambda_p, float eps,
                              float* s_out, hipStream_t st) {
  const char* v = static_cast<const char*>(V);
  const dim3 grid(lay.heads);
#define KVR_PRIOR(DT, NT, KEEP)                                                                         \
  hipLaunchKernelGGL((score_prior_kernel<DT, NT, KEEP>), grid, dim3(NT), 0, st, v, lay, s_in, lambda_p, \
                     eps, s_out)
  if (lay.dtype == DT_BF16) {
    if (lay.n <= 16 * prior_depth<DT_BF16>()) KVR_PRIOR(DT_BF16, 256, true);
    else KVR_PRIOR(DT_BF16, 256, false);
  } else {
    if (lay.n <= 16 * prior_depth<DT_F32>()) KVR_PRIOR(DT_F32, 256, true);
    else KVR_PRIOR(DT_F32, 256, false);
  }
#undef KVR_PRIOR
  return hipGetLastError();
}

}  // namespace kvr
