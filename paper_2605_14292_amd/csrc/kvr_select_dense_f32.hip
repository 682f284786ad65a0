// Algorithm 1 (paper Sec. 4.1, Eq. 1-3) for heads of n <= 256 tokens whose rows are fp32: the
// flat-signature mode, whose signature rows are means over layers and heads and so are not
// bf16 numbers, and fp32 caches.  One workgroup of sixteen wave64s per head (such launches have
// few heads, so the latency of one head is what counts):
//
//   rows     staged in LDS as fp32, 129-float pitch (column reads of 32 rows hit 32 banks)
//   Gram     lower-triangular 32x32 tiles on the fp32 MFMA (32x32x2, fp32 products and sums)
//   norms    r_j = 1/(||V_j|| + eps) from the Gram diagonal              (Eq. 1)
//   cosines  packed fp32 triangle in the space the rows were staged in   (Algorithm 1, Sims)
//   greedy   the single-wave pick loop of the bf16 kernels                (Eq. 2-3)
//
// Only the selection is done here; rows are compacted by compact_kernel.
#include "kvr_dense_common.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

constexpr int kF32Pitch = 129;                 // floats per staged row
constexpr int kF32MaxB = 256;
constexpr int kF32Threads = 1024;
constexpr int kF32Waves = kF32Threads / 64;

__host__ __device__ constexpr int f32_region_a(int NT) {
  const int tri = dense_tri_floats(NT) * 4, stage = NT * 32 * kF32Pitch * 4;
  return ((tri > stage ? tri : stage) + 15) & ~15;
}
__host__ __device__ constexpr int f32_smem_bytes(int NT) {
  // region A | s_l[N32] | rinv[N32] | idx_l | order_l | gain_l
  return f32_region_a(NT) + NT * 32 * 4 * 2 + kF32MaxB * 4 * 3;
}

struct F32Args {
  const float* V; const float* s;
  int32_t* idx_sorted; int32_t* pick_order; float* pick_gain;
  long long stride_head, stride_tok;   // elements
  int n, b;
  float lambda, eps;
};

template <int NT>
__global__ __launch_bounds__(kF32Threads, 1) void select_dense_f32_kernel(F32Args a) {
  constexpr int N32 = NT * 32;
  constexpr int NQ = NT / 2;
  constexpr int NTILES = NT * (NT + 1) / 2;
  constexpr int MAXT = (NTILES + kF32Waves - 1) / kF32Waves;
  extern __shared__ __align__(16) char smem[];
  float* stage = reinterpret_cast<float*>(smem);
  float* tri = reinterpret_cast<float*>(smem);
  float* s_l = reinterpret_cast<float*>(smem + f32_region_a(NT));
  float* rinv = s_l + N32;
  int32_t* idx_l = reinterpret_cast<int32_t*>(rinv + N32);
  int32_t* order_l = idx_l + kF32MaxB;
  float* gain_l = reinterpret_cast<float*>(order_l + kF32MaxB);

  const int tid = threadIdx.x;
  const int lane = tid & 63, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int h = blockIdx.x;
  const int n = a.n, b = a.b;
  const bool diverse = a.lambda != 0.0f && b > 1;

  if (tid < N32) s_l[tid] = tid < n ? a.s[static_cast<long long>(h) * n + tid] : -INFINITY;
  typedef __attribute__((ext_vector_type(16))) float f32x16_t;
  f32x16_t acc[MAXT];
  if (diverse) {
    // rows -> LDS, 32 threads per row (float4 each), rows past n read as zero
    const float* Vh = a.V + h * a.stride_head;
    for (int r = tid >> 5; r < N32; r += kF32Threads / 32) {
      float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
      if (r < n) x = *reinterpret_cast<const float4*>(Vh + r * a.stride_tok + (tid & 31) * 4);
      float* d = stage + r * kF32Pitch + (tid & 31) * 4;
      d[0] = x.x; d[1] = x.y; d[2] = x.z; d[3] = x.w;
    }
    __syncthreads();
    // tile t of the lower triangle: row block I, column block J <= I
#pragma unroll
    for (int sl = 0; sl < MAXT; ++sl) {
      const int tile = wave + kF32Waves * sl;
      acc[sl] = f32x16_t{0};
      if (tile < NTILES) {
        int I = 0;
        while ((I + 1) * (I + 2) / 2 <= tile) ++I;
        const int J = tile - I * (I + 1) / 2;
        const float* pa = stage + (I * 32 + (lane & 31)) * kF32Pitch + hf;
        const float* pb = stage + (J * 32 + (lane & 31)) * kF32Pitch + hf;
#pragma unroll 8
        for (int ks = 0; ks < kD / 2; ++ks)
          acc[sl] = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[2 * ks], pb[2 * ks], acc[sl], 0, 0, 0);
        if (I == J) {                                 // squared norms sit on the diagonal
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int il = (r >> 2) * 8 + hf * 4 + (r & 3);
            if (il == (lane & 31)) rinv[I * 32 + il] = acc[sl][r];
          }
        }
      }
    }
    __syncthreads();                                  // staged rows are dead from here on
    if (tid < N32) rinv[tid] = 1.0f / (sqrtf(rinv[tid]) + a.eps);
    __syncthreads();
#pragma unroll
    for (int sl = 0; sl < MAXT; ++sl) {
      const int tile = wave + kF32Waves * sl;
      if (tile < NTILES) {
        int I = 0;
        while ((I + 1) * (I + 2) / 2 <= tile) ++I;
        const int J = tile - I * (I + 1) / 2;
        write_cos_tile(tri, rinv, acc[sl], I, J, lane);
      }
    }
  }
  __syncthreads();

  if (wave == 0) {
    pick_chain<NQ>(s_l, tri, order_l, gain_l, n, b, a.lambda, diverse, lane);
    sort_picks<NQ>(order_l, idx_l, reinterpret_cast<int32_t*>(rinv), b, lane, nullptr);
  }
  __syncthreads();
  const long long ob = static_cast<long long>(h) * b;
  for (int t = tid; t < b; t += kF32Threads) {
    a.idx_sorted[ob + t] = idx_l[t];
    if (a.pick_order) a.pick_order[ob + t] = order_l[t];
    if (a.pick_gain) a.pick_gain[ob + t] = gain_l[t];
  }
}

bool dense_f32_supported(const Layout& lay, int b) {
  return lay.dtype == DT_F32 && lay.n <= 256 && b <= kF32MaxB;
}

hipError_t launch_select_dense_f32(const void* V, const float* s, const Layout& lay, int b, float lambda,
                                   float eps, int32_t* idx_sorted, int32_t* pick_order, float* pick_gain,
                                   hipStream_t st) {
  F32Args a;
  a.V = static_cast<const float*>(V); a.s = s;
  a.idx_sorted = idx_sorted; a.pick_order = pick_order; a.pick_gain = pick_gain;
  a.stride_head = lay.stride_head; a.stride_tok = lay.stride_tok;
  a.n = lay.n; a.b = b; a.lambda = lambda; a.eps = eps;
  auto go = [&](auto kern, int smem) -> hipError_t {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(lay.heads), dim3(kF32Threads), smem, st, a);
    return hipGetLastError();
  };
  if (lay.n <= 64) return go(&select_dense_f32_kernel<2>, f32_smem_bytes(2));
  if (lay.n <= 128) return go(&select_dense_f32_kernel<4>, f32_smem_bytes(4));
  if (lay.n <= 192) return go(&select_dense_f32_kernel<6>, f32_smem_bytes(6));
  return go(&select_dense_f32_kernel<8>, f32_smem_bytes(8));
}

}  // namespace kvr
