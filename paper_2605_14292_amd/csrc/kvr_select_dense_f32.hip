// Algorithm 1 (paper Sec. 4.1, Eq. 1-3) for heads of n <= 256 tokens whose rows are fp32: the
// flat-signature mode, whose signature rows are means over layers and heads and so are not
// bf16 numbers, and fp32 caches.  One workgroup of sixteen wave64s per head (such launches have
// few heads, so the latency of one head is what counts):
//
//   rows     staged in LDS as fp32, 132-float pitch (16-byte aligned rows; eight consecutive rows
//            cover the 32 banks with their 16-byte pieces)
//   Gram     lower-triangular 32x32 tiles on the fp32 MFMA (32x32x2, fp32 products and sums).  Which
//            two of the 128 k an MFMA multiplies is free as long as both operands agree: MFMA m
//            takes k = m for the lower half-wave and k = 64 + m for the upper one, so a lane reads
//            64 consecutive floats of its row, four per LDS request
//   norms    r_j = 1/(||V_j|| + eps) from the Gram diagonal              (Eq. 1)
//   cosines  packed fp32 triangle in the space the rows were staged in   (Algorithm 1, Sims)
//   greedy   the single-wave pick loop of the bf16 kernels                (Eq. 2-3)
//
// With Q the kernel also computes the base scores (up to 16 queries), and with K_out / V_out it
// copies the kept rows: a single fp32 head is then one launch instead of three.
#include "kvr_dense_common.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

constexpr int kF32Pitch = 132;                 // floats per staged row
constexpr int kF32MaxB = 256;
constexpr int kF32Threads = 1024;
constexpr int kF32Waves = kF32Threads / 64;

__host__ __device__ constexpr int f32_region_a(int NT) {
  const int tri = dense_tri_floats(NT) * 4, stage = NT * 32 * kF32Pitch * 4;
  return ((tri > stage ? tri : stage) + 15) & ~15;
}
__host__ __device__ constexpr int f32_smem_bytes(int NT) {
  // region A | s_l[N32] | rinv[N32] | idx_l | order_l | gain_l | tok_c[N32] | meta[4]
  return f32_region_a(NT) + NT * 32 * 4 * 2 + kF32MaxB * 4 * 3 + NT * 32 * 4 + 16;
}

struct F32Args {
  const float* V; const float* s;
  int32_t* idx_sorted; int32_t* pick_order; float* pick_gain;
  long long stride_head, stride_tok;   // elements
  int n, b;
  float lambda, eps;
  // optional: the scores are computed here from K and Q (then `s` is unused and s_out receives them),
  // and the kept rows are written here
  const float* K; const float* Q; int G; float* s_out;
  float* K_out; float* V_out;
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
  int32_t* tok_c = reinterpret_cast<int32_t*>(gain_l + kF32MaxB);     // [N32] tokens of the reduced problem
  int32_t* meta = tok_c + N32;                                         // [0] its size, 0 = not reduced

  const int tid = threadIdx.x;
  const int lane = tid & 63, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int h = blockIdx.x;
  const int n = a.n, b = a.b;
  const bool diverse = a.lambda != 0.0f && b > 1;

  if (a.Q) {
    // Base scores (the stand-in for the paper's external scorer): s_i = (1/G) sum_g softmax_i(q_g . k_i / sqrt(d)).
    // 32 threads per row (float4 each) take the dot products in fp32, one wave per query takes its softmax.
    const float* Kh = a.K + h * a.stride_head;
    float4 kr[NT];
#pragma unroll
    for (int k = 0; k < NT; ++k) {
      const int r = (tid >> 5) + 32 * k;
      kr[k] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (r < n) kr[k] = *reinterpret_cast<const float4*>(Kh + r * a.stride_tok + (tid & 31) * 4);
    }
    float* zl = stage;                                 // [G][N32] logits, then probabilities (the stage is free until the rows arrive)
    const float scale = 0.08838834764831845f;          // 1/sqrt(128)
    for (int g = 0; g < a.G; ++g) {
      const float4 qv = *reinterpret_cast<const float4*>(a.Q + (static_cast<long long>(h) * a.G + g) * kD + (tid & 31) * 4);
#pragma unroll
      for (int k = 0; k < NT; ++k) {
        float p = fmaf(kr[k].x, qv.x, fmaf(kr[k].y, qv.y, fmaf(kr[k].z, qv.z, kr[k].w * qv.w)));
#pragma unroll
        for (int off = 16; off >= 1; off >>= 1) p += __shfl_xor(p, off, kWave);
        const int r = (tid >> 5) + 32 * k;
        if ((tid & 31) == 0) zl[g * N32 + r] = r < n ? p * scale : -INFINITY;
      }
    }
    __syncthreads();
    if (wave < a.G) {
      float v[NQ];
      float mx = -INFINITY;
#pragma unroll
      for (int q = 0; q < NQ; ++q) { v[q] = zl[wave * N32 + lane + 64 * q]; mx = fmaxf(mx, v[q]); }
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
      float sum = 0.f;
#pragma unroll
      for (int q = 0; q < NQ; ++q) { v[q] = __expf(v[q] - mx); sum += v[q]; }   // exp(-inf) = 0 for padding
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, kWave);
      const float inv = 1.0f / sum;
#pragma unroll
      for (int q = 0; q < NQ; ++q) zl[wave * N32 + lane + 64 * q] = v[q] * inv;
    }
    __syncthreads();
    if (tid < N32) {
      float p = 0.f;
      for (int g = 0; g < a.G; ++g) p += zl[g * N32 + tid];
      p /= static_cast<float>(a.G);
      s_l[tid] = tid < n ? p : -INFINITY;                // padding never competes
      if (tid < n && a.s_out) a.s_out[static_cast<long long>(h) * n + tid] = p;
    }
    __syncthreads();                                     // the stage is free again
  } else {
    if (tid < N32) s_l[tid] = tid < n ? a.s[static_cast<long long>(h) * n + tid] : -INFINITY;
  }
  if (tid == 0) meta[0] = 0;
  typedef __attribute__((ext_vector_type(16))) float f32x16_t;
  f32x16_t acc[MAXT];
  int ns = 0;                                       // size of the reduced problem, 0 = all n tokens
  if (diverse) {
    // the rows start their trip from memory before anything else: 32 threads per row (float4
    // each), rows past n read as zero
    const float* Vh = a.V + h * a.stride_head;
    float4 xr[NT];
#pragma unroll
    for (int k = 0; k < NT; ++k) {
      const int r = (tid >> 5) + 32 * k;
      xr[k] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (r < n) xr[k] = *reinterpret_cast<const float4*>(Vh + r * a.stride_tok + (tid & 31) * 4);
    }
    // Exact candidate reduction for heads of more than 128 tokens: a token with s_j < s_(b) - lambda
    // never wins Eq. 3 (while fewer than b tokens are selected one of the b best-scored is free and
    // gains at least s_(b) - lambda; the token itself gains at most s_j).  When at most 128 tokens
    // remain, the head shrinks to them: fewer Gram tiles, two tokens per lane in the pick loop.
    // The survivors keep their order, so ties break as before.
    if constexpr (NT > 4) {
      __syncthreads();
      if (wave == 0) {
        float sv[NQ];
        uint32_t key[NQ];
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
          sv[q] = s_l[lane + 64 * q];
          key[q] = lane + 64 * q < n ? ordered_key(sv[q] + 0.0f) : 0u;
        }
        // s_(b) from the leading 16 bits of the ordered keys: at most s_(b), so the bound only loosens
        uint32_t T = 0;
        for (int bit = 31; bit >= 16; --bit) {
          const uint32_t cand = T | (1u << bit);
          int cnt = 0;
#pragma unroll
          for (int q = 0; q < NQ; ++q) cnt += __popcll(__ballot(key[q] >= cand));
          if (cnt >= b) T = cand;
        }
        const float sb = key_to_float(T);
        const float thr = sb - a.lambda * 1.00001f - 1e-5f * fabsf(sb);   // cosines may exceed 1 by a few ulp
        unsigned long long keep[NQ];
        int cnt = 0;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
          keep[q] = __ballot(lane + 64 * q < n && !(sv[q] < thr));
          cnt += __popcll(keep[q]);
        }
        if (cnt >= b && cnt <= 128) {
          wave_lds_sync();                            // every lane holds its scores before s_l is rewritten
          int base = 0;
#pragma unroll
          for (int q = 0; q < NQ; ++q) {
            const bool kept = (keep[q] >> lane) & 1ull;
            const int c = base + __popcll(keep[q] & ((1ull << lane) - 1ull));
            if (kept) {
              tok_c[c] = lane + 64 * q;
              s_l[c] = sv[q];
            }
            idx_l[lane + 64 * q] = kept ? c : -1;        // where the token's row goes (idx_l is free until the sort)
            base += __popcll(keep[q]);
          }
          for (int c = cnt + lane; c < 128; c += kWave) s_l[c] = -INFINITY;   // padding never competes
          if (lane == 0) meta[0] = cnt;
        }
      }
      __syncthreads();
      ns = meta[0];
    }
    // rows -> LDS: at their own position, or at their position in the reduced problem
#pragma unroll
    for (int k = 0; k < NT; ++k) {
      const int r = (tid >> 5) + 32 * k;
      const int dst = ns ? idx_l[r] : r;
      if (dst >= 0) *reinterpret_cast<float4*>(stage + dst * kF32Pitch + (tid & 31) * 4) = xr[k];
    }
    if (ns)                                           // rows between the survivors and the end of their last block
      for (int r = ns + (tid >> 5); r < ((ns + 31) & ~31); r += kF32Threads / 32)
        *reinterpret_cast<float4*>(stage + r * kF32Pitch + (tid & 31) * 4) = make_float4(0.f, 0.f, 0.f, 0.f);
    __syncthreads();
    // tile t of the lower triangle: row block I, column block J <= I (only the blocks in use)
    const int nblk = ns ? (ns + 31) >> 5 : NT;
    const int ntiles = nblk * (nblk + 1) / 2;
#pragma unroll
    for (int sl = 0; sl < MAXT; ++sl) {
      const int tile = wave + kF32Waves * sl;
      acc[sl] = f32x16_t{0};
      if (tile < ntiles) {
        int I = 0;
        while ((I + 1) * (I + 2) / 2 <= tile) ++I;
        const int J = tile - I * (I + 1) / 2;
        const float* pa = stage + (I * 32 + (lane & 31)) * kF32Pitch + hf * (kD / 2);
        const float* pb = stage + (J * 32 + (lane & 31)) * kF32Pitch + hf * (kD / 2);
#pragma unroll 4
        for (int q = 0; q < kD / 8; ++q) {
          const float4 xa = *reinterpret_cast<const float4*>(pa + 4 * q);
          const float4 xb = *reinterpret_cast<const float4*>(pb + 4 * q);
          acc[sl] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa.x, xb.x, acc[sl], 0, 0, 0);
          acc[sl] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa.y, xb.y, acc[sl], 0, 0, 0);
          acc[sl] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa.z, xb.z, acc[sl], 0, 0, 0);
          acc[sl] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa.w, xb.w, acc[sl], 0, 0, 0);
        }
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
    if (tid < nblk * 32) rinv[tid] = 1.0f / (sqrtf(rinv[tid]) + a.eps);
    __syncthreads();
#pragma unroll
    for (int sl = 0; sl < MAXT; ++sl) {
      const int tile = wave + kF32Waves * sl;
      if (tile < ntiles) {
        int I = 0;
        while ((I + 1) * (I + 2) / 2 <= tile) ++I;
        const int J = tile - I * (I + 1) / 2;
        write_cos_tile(tri, rinv, acc[sl], I, J, lane);
      }
    }
  }
  __syncthreads();

  if (wave == 0) {
    if (ns) {                                           // the reduced problem: indices go back through tok_c
      pick_chain<2>(s_l, tri, order_l, gain_l, ns, b, a.lambda, diverse, lane);
      sort_picks<2>(order_l, idx_l, reinterpret_cast<int32_t*>(rinv), b, lane, tok_c);
    } else {
      pick_chain<NQ>(s_l, tri, order_l, gain_l, n, b, a.lambda, diverse, lane);
      sort_picks<NQ>(order_l, idx_l, reinterpret_cast<int32_t*>(rinv), b, lane, nullptr);
    }
  }
  __syncthreads();
  const long long ob = static_cast<long long>(h) * b;
  for (int t = tid; t < b; t += kF32Threads) {
    a.idx_sorted[ob + t] = idx_l[t];
    if (a.pick_order) a.pick_order[ob + t] = order_l[t];
    if (a.pick_gain) a.pick_gain[ob + t] = gain_l[t];
  }
  // kept rows: 32 threads per row, four rows per thread in flight
  if (a.K_out || a.V_out) {
    const int c4 = (tid & 31) * 4;
    for (int t0 = 0; t0 < b; t0 += 128) {
      float4 xk[4], xv[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int t = min(t0 + (tid >> 5) + 32 * k, b - 1);
        const long long src = h * a.stride_head + min(max(idx_l[t], 0), n - 1) * a.stride_tok + c4;
        xk[k] = xv[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (a.K_out) xk[k] = *reinterpret_cast<const float4*>(a.K + src);
        if (a.V_out) xv[k] = *reinterpret_cast<const float4*>(a.V + src);
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int t = t0 + (tid >> 5) + 32 * k;
        if (t < b) {
          if (a.K_out) *reinterpret_cast<float4*>(a.K_out + (ob + t) * kD + c4) = xk[k];
          if (a.V_out) *reinterpret_cast<float4*>(a.V_out + (ob + t) * kD + c4) = xv[k];
        }
      }
    }
  }
}

bool dense_f32_supported(const Layout& lay, int b) {
  return lay.dtype == DT_F32 && lay.n <= 256 && b <= kF32MaxB;
}

hipError_t launch_select_dense_f32(const void* V, const float* s, const Layout& lay, int b, float lambda,
                                   float eps, int32_t* idx_sorted, int32_t* pick_order, float* pick_gain,
                                   hipStream_t st) {
  return launch_retain_dense_f32(nullptr, V, nullptr, 0, s, lay, b, lambda, eps, nullptr, idx_sorted, pick_order,
                                 pick_gain, nullptr, nullptr, st);
}

hipError_t launch_retain_dense_f32(const void* K, const void* V, const void* Q, int G, const float* s,
                                   const Layout& lay, int b, float lambda, float eps, float* s_out,
                                   int32_t* idx_sorted, int32_t* pick_order, float* pick_gain, void* K_out,
                                   void* V_out, hipStream_t st) {
  F32Args a;
  a.K = static_cast<const float*>(K); a.Q = static_cast<const float*>(Q); a.G = G; a.s_out = s_out;
  a.K_out = static_cast<float*>(K_out); a.V_out = static_cast<float*>(V_out);
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
