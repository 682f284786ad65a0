// Fused retention step for heads with n <= 256 bf16 tokens: one workgroup (four
// wave64s) per head takes the head from HBM to its compacted rows.
//
//   score    (optional, G <= 8)  logits Q K^T on bf16 MFMA, softmax over the
//            tokens per query, mean over queries             (base-score stand-in)
//   norms    r_j = 1/(||V_j|| + eps) from the Gram diagonal  (paper Eq. 1)
//   Gram     lower-triangular 32x32 tiles of V V^T on bf16 MFMA with fp32
//            accumulation, scaled to cosines and parked in LDS as a packed
//            triangle of fp32                                (Algorithm 1, Sims)
//   greedy   one wave keeps s, m and the alive set in registers (token j lives
//            in lane j%64); each pick is a DPP max-reduction of the gains, a
//            ballot for the lowest tied index, and one LDS row read that is
//            folded into m                                   (Eq. 2-3, Alg. 1)
//   compact  rows at the ascending picks are copied to the dense outputs
//
// The raw bf16 rows go through the MFMA un-normalised (bf16 x bf16 products are
// exact in fp32); the cosine is dot * r_i * r_j in fp32.  Rounding normalised
// rows to bf16 first would put ~4e-3 on every cosine.
//
// LDS: the packed triangle (n=192: 74 KB, n=256: 132 KB) reuses the space the
// rows were staged in, so two heads fit a CU at n <= 192.
#include "kvr_device.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kDenseThreads = 256;
constexpr int kRowPitch = 272;   // bytes per staged row: 256 + 16 so that 8 consecutive rows hit distinct banks
constexpr int kMaxB = 256;

__host__ __device__ constexpr int dense_tri_floats(int NT) { return (NT * 32) * (NT * 32 + 1) / 2; }
__host__ __device__ constexpr int dense_region_a(int NT) {
  const int tri = dense_tri_floats(NT) * 4, stage = NT * 32 * kRowPitch;
  return ((tri > stage ? tri : stage) + 15) & ~15;
}
__host__ __device__ constexpr int dense_smem_bytes(int NT) {
  // region A | s_l[N32] | rinv[N32] | red[64] | idx_l[kMaxB] | order_l[kMaxB] | gain_l[kMaxB]
  return dense_region_a(NT) + NT * 32 * 4 * 2 + 64 * 4 + kMaxB * 4 * 3;
}

#define KVR_DPP_MAX(v, ctrl, rmask)                                                        \
  {                                                                                        \
    const int _o = __builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), ctrl, \
                                               rmask, 0xf, false);                        \
    v = fmaxf(v, __int_as_float(_o));                                                      \
  }
#define KVR_DPP_ADD(v, ctrl, rmask)                                                            \
  {                                                                                            \
    const int _o = __builtin_amdgcn_update_dpp(0, __float_as_int(v), ctrl, rmask, 0xf, false); \
    v += __int_as_float(_o);                                                                   \
  }

// Max over the wave, returned wave-uniform.  Each step is one v_max_f32 with a
// DPP source (the compiler's own lowering of a DPP move plus fmaxf costs four
// instructions a step, which is most of a pick's latency); lanes whose DPP
// source is out of range keep their value.  s_nop 1 covers the two wait states
// a DPP read needs after a VALU write of the same register.
__device__ __forceinline__ float wave_max_uniform(float v) {
  asm volatile(
      "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_shr:1 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_shr:2 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_shr:4 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_shr:8 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
      "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
      "s_nop 1"
      : "+v"(v));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
// Orders LDS traffic between the lanes of one wave.  Lanes of a wave run in
// lock-step and the LDS pipeline is in order, but the compiler reasons per
// thread: without a fence it may forward a lane's own earlier store to a load
// that another lane has overwritten in between.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
// max(a, b) as the hardware does it (a NaN operand yields the other one), without
// the canonicalising self-max the compiler adds around fmaxf on loaded values
__device__ __forceinline__ float hw_max(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
// max / sum over each half of the wave (lanes 0-31 and 32-63); valid in lanes 31 and 63
__device__ __forceinline__ float half_max_at_31(float v) {
  KVR_DPP_MAX(v, 0x111, 0xf) KVR_DPP_MAX(v, 0x112, 0xf) KVR_DPP_MAX(v, 0x114, 0xf)
  KVR_DPP_MAX(v, 0x118, 0xf) KVR_DPP_MAX(v, 0x142, 0xa)
  return v;
}
__device__ __forceinline__ float half_sum_at_31(float v) {
  KVR_DPP_ADD(v, 0x111, 0xf) KVR_DPP_ADD(v, 0x112, 0xf) KVR_DPP_ADD(v, 0x114, 0xf)
  KVR_DPP_ADD(v, 0x118, 0xf) KVR_DPP_ADD(v, 0x142, 0xa)
  return v;
}

struct DenseArgs {
  const char* K; const char* V; const char* Q; const float* s_in;
  float* s_out; int32_t* idx_sorted; int32_t* pick_order; float* pick_gain;
  char* K_out; char* V_out;
  long long stride_head, stride_tok;   // elements
  int n, b, G;
  float lambda, eps;
};

// Stage one head's [n,128] bf16 rows into LDS (row pitch kRowPitch), zero rows
// beyond n, so MFMA fragments of padded blocks are zero.
template <int NT>
__device__ __forceinline__ void stage_rows(const char* __restrict__ src, long long stride_tok, int n,
                                           char* stage, int tid) {
  constexpr int kIters = NT * 32 * 16 / kDenseThreads;   // 16-byte chunks per thread
  uint4 reg[kIters];
  const int chunk = tid & 15, r0 = tid >> 4;
#pragma unroll
  for (int k = 0; k < kIters; ++k) {
    const int row = r0 + 16 * k;
    reg[k] = make_uint4(0u, 0u, 0u, 0u);
    if (row < n) reg[k] = *reinterpret_cast<const uint4*>(src + (row * stride_tok + chunk * 8) * 2);
  }
#pragma unroll
  for (int k = 0; k < kIters; ++k) {
    const int row = r0 + 16 * k;
    *reinterpret_cast<uint4*>(stage + row * kRowPitch + chunk * 16) = reg[k];
  }
}

__device__ __forceinline__ bf16x8 frag_at(const char* stage, int block, int ks, int lane) {
  const int row = block * 32 + (lane & 31), hf = lane >> 5;
  return *reinterpret_cast<const bf16x8*>(stage + row * kRowPitch + ks * 32 + hf * 16);
}

template <int NT>
__global__ __launch_bounds__(kDenseThreads) void retain_dense_kernel(DenseArgs a) {
  constexpr int N32 = NT * 32;
  constexpr int NQ = NT / 2;                         // tokens per lane in the greedy wave
  constexpr int NTILES = NT * (NT + 1) / 2;
  constexpr int MAXT = (NTILES + 3) / 4;             // Gram tiles per wave
  extern __shared__ __align__(16) char smem[];
  char* stage = smem;                                // staged rows (phase 1) ...
  float* tri = reinterpret_cast<float*>(smem);       // ... later the packed cosine triangle
  float* s_l = reinterpret_cast<float*>(smem + dense_region_a(NT));
  float* rinv = s_l + N32;
  float* red = rinv + N32;
  int32_t* idx_l = reinterpret_cast<int32_t*>(red + 64);
  int32_t* order_l = idx_l + kMaxB;
  float* gain_l = reinterpret_cast<float*>(order_l + kMaxB);

  const int h = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = a.n, b = a.b;
  const long long head_off = h * a.stride_head * 2;  // bytes
  const bool diverse = a.lambda != 0.0f;

  // ------------------------------------------------------------------ scores
  if (a.Q) {
    stage_rows<NT>(a.K + head_off, a.stride_tok, n, stage, tid);
    bf16x8 qf[8];
    {
      const int g = lane & 31;
      const char* qp = a.Q + (static_cast<long long>(h) * a.G + g) * kD * 2 + hf * 16;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        uint4 w = make_uint4(0u, 0u, 0u, 0u);
        if (g < a.G) w = *reinterpret_cast<const uint4*>(qp + ks * 32);
        qf[ks] = *reinterpret_cast<bf16x8*>(&w);
      }
    }
    __syncthreads();
    constexpr int BPW = (NT + 3) / 4;                // token blocks per wave
    float z[BPW][4];
    const float scale = 0.08838834764831845f;        // 1/sqrt(128)
    float zmax[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
    for (int k = 0; k < BPW; ++k) {
      const int I = wave + 4 * k;
      f32x16 acc = {0};
      if (I < NT) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[ks], frag_at(stage, I, ks, lane), acc, 0, 0, 0);
      }
      const bool live = I < NT && (I * 32 + (lane & 31)) < n;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        z[k][r] = live ? acc[r] * scale : -INFINITY;   // rows g = hf*4 + r of the 32x32 tile
        zmax[r] = fmaxf(zmax[r], z[k][r]);
      }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float v = half_max_at_31(zmax[r]);
      if ((lane & 31) == 31) red[wave * 8 + hf * 4 + r] = v;
    }
    __syncthreads();
    float zsum[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int g = hf * 4 + r;
      zmax[r] = fmaxf(fmaxf(red[g], red[8 + g]), fmaxf(red[16 + g], red[24 + g]));
      zsum[r] = 0.f;
    }
#pragma unroll
    for (int k = 0; k < BPW; ++k)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        z[k][r] = __expf(z[k][r] - zmax[r]);         // exp(-inf) = 0 for padded tokens
        zsum[r] += z[k][r];
      }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float v = half_sum_at_31(zsum[r]);
      if ((lane & 31) == 31) red[32 + wave * 8 + hf * 4 + r] = v;
    }
    __syncthreads();
    const float invG = 1.0f / static_cast<float>(a.G);
    float w[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int g = hf * 4 + r;
      const float tot = red[32 + g] + red[40 + g] + red[48 + g] + red[56 + g];
      w[r] = g < a.G ? invG / tot : 0.f;
    }
#pragma unroll
    for (int k = 0; k < BPW; ++k) {
      const int I = wave + 4 * k;
      float p = 0.f;
#pragma unroll
      for (int r = 0; r < 4; ++r) p = fmaf(z[k][r], w[r], p);
      p += __shfl_xor(p, 32, kWave);                 // queries 0-3 live in lanes 0-31, 4-7 in 32-63
      const int j = I * 32 + (lane & 31);
      if (I < NT && hf == 0) {
        s_l[j] = j < n ? p : -INFINITY;               // padding never competes
        if (j < n && a.s_out) a.s_out[static_cast<long long>(h) * n + j] = p;
      }
    }
    __syncthreads();                                  // K fragments are dead; s_l is complete
  } else {
    for (int j = tid; j < N32; j += kDenseThreads)
      s_l[j] = j < n ? a.s_in[static_cast<long long>(h) * n + j] : -INFINITY;
  }

  // -------------------------------------------------- Gram -> packed cosines
  if (diverse && b > 1) {
    stage_rows<NT>(a.V + head_off, a.stride_tok, n, stage, tid);
    __syncthreads();
    f32x16 acc[MAXT];
#pragma unroll
    for (int sl = 0; sl < MAXT; ++sl) {
      const int t = wave * MAXT + sl;
      acc[sl] = f32x16{0};
      if (t < NTILES) {
        int I = 0;
        while ((I + 1) * (I + 2) / 2 <= t) ++I;
        const int J = t - I * (I + 1) / 2;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
          acc[sl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_at(stage, I, ks, lane),
                                                            frag_at(stage, J, ks, lane), acc[sl], 0, 0, 0);
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
    for (int j = tid; j < N32; j += kDenseThreads) rinv[j] = 1.0f / (sqrtf(rinv[j]) + a.eps);
    __syncthreads();
#pragma unroll
    for (int sl = 0; sl < MAXT; ++sl) {
      const int t = wave * MAXT + sl;
      if (t < NTILES) {
        int I = 0;
        while ((I + 1) * (I + 2) / 2 <= t) ++I;
        const int J = t - I * (I + 1) / 2;
        const int j = J * 32 + (lane & 31);
        const float rc = rinv[j];
#pragma unroll
        for (int R = 0; R < 4; ++R) {
          const int i0 = I * 32 + R * 8 + hf * 4;
          const float4 rr = *reinterpret_cast<const float4*>(rinv + i0);
          const float rrow[4] = {rr.x, rr.y, rr.z, rr.w};
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int i = i0 + q;
            if (I != J || j <= i) tri[i * (i + 1) / 2 + j] = acc[sl][R * 4 + q] * rrow[q] * rc;
          }
        }
      }
    }
  }
  __syncthreads();

  // ------------------------------------------------------------------ greedy
  if (wave == 0) {
    // Token j lives in lane j%64, slot j/64.  A selected (or padding) token has
    // its score replaced by -inf, so its gain is -inf and it never ties with a
    // finite maximum; the exact selected set is rebuilt from the pick list.
    float sreg[NQ], mreg[NQ];
    int jb4[NQ], tjb4[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const int j = lane + 64 * q;
      sreg[q] = s_l[j];                                // -inf beyond n
      mreg[q] = 0.f;
      jb4[q] = j * 4;
      tjb4[q] = (j * (j + 1) / 2) * 4;
    }
    const float nlam = -a.lambda;
    const char* trib = reinterpret_cast<const char*>(tri);
    for (int t = 0; t < b; ++t) {
      float av[NQ];
#pragma unroll
      for (int q = 0; q < NQ; ++q) av[q] = fmaf(nlam, mreg[q], sreg[q]);
      float best = av[0];
#pragma unroll
      for (int q = 1; q < NQ; ++q) best = hw_max(best, av[q]);
      const float amax = wave_max_uniform(best);
      int i = -1;
#pragma unroll
      for (int q = NQ - 1; q >= 0; --q) {
        const unsigned long long eq = __ballot(av[q] == amax);
        if (eq) i = (__ffsll(static_cast<long long>(eq)) - 1) + 64 * q;
      }
      if (!(amax > -INFINITY)) {
        // Non-finite input only: every remaining gain is -inf or NaN.  Take the
        // lowest token that is not in the pick list yet (slow, never on finite data).
        i = -1;
#pragma unroll
        for (int q = NQ - 1; q >= 0; --q) {
          const int j = lane + 64 * q;
          bool free_tok = j < n;
          wave_lds_sync();                             // order_l is written by lane 0
          for (int u = 0; u < t; ++u) free_tok = free_tok && order_l[u] != j;
          const unsigned long long al = __ballot(free_tok);
          if (al) i = (__ffsll(static_cast<long long>(al)) - 1) + 64 * q;
        }
      }
#pragma unroll
      for (int q = 0; q < NQ; ++q) sreg[q] = (jb4[q] == i * 4) ? -INFINITY : sreg[q];
      if (lane == 0) { order_l[t] = i; gain_l[t] = amax; }
      if (t + 1 == b || !diverse) continue;
      // row i of the packed triangle: element (i,j) sits at max(T(i)+j, T(j)+i)
      const int ti4 = (i * (i + 1) / 2) * 4, i4 = i * 4;
#pragma unroll
      for (int q = 0; q < NQ; ++q) {
        const int a0 = ti4 + jb4[q], a1 = tjb4[q] + i4;
        const float c = *reinterpret_cast<const float*>(trib + (a0 > a1 ? a0 : a1));
        mreg[q] = hw_max(mreg[q], c);
      }
    }
    // sort(S): flag the picked tokens, then ascending indices by prefix popcount
    int32_t* flag = reinterpret_cast<int32_t*>(rinv);   // rinv is dead by now
#pragma unroll
    for (int q = 0; q < NQ; ++q) flag[lane + 64 * q] = 0;
    wave_lds_sync();                                   // order_l was written by lane 0
    for (int u = lane; u < b; u += kWave) flag[order_l[u]] = 1;
    wave_lds_sync();                                   // flags are set by other lanes
    int off = 0;
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const int j = lane + 64 * q;
      const bool picked = flag[j] != 0;
      const unsigned long long sel = __ballot(picked);
      if (picked) {
        const int rank = __popcll(sel & ((1ull << lane) - 1ull));
        idx_l[off + rank] = j;
      }
      off += __popcll(sel);
    }
  }
  __syncthreads();

  // --------------------------------------------------- outputs and compaction
  const long long ob = static_cast<long long>(h) * b;
  for (int t = tid; t < b; t += kDenseThreads) {
    a.idx_sorted[ob + t] = idx_l[t];
    if (a.pick_order) a.pick_order[ob + t] = order_l[t];
    if (a.pick_gain) a.pick_gain[ob + t] = gain_l[t];
  }
  if (a.K_out || a.V_out) {
    const int chunk = tid & 15;
    for (int t0 = 0; t0 < b; t0 += kDenseThreads / 16) {
      const int t = t0 + (tid >> 4);
      if (t < b) {
        const int it = min(max(idx_l[t], 0), n - 1);   // never read outside the head, whatever the scores were
        const long long src = head_off + (it * a.stride_tok + chunk * 8) * 2;
        const long long dst = ((ob + t) * kD + chunk * 8) * 2;
        uint4 kv, vv;
        if (a.K_out) kv = *reinterpret_cast<const uint4*>(a.K + src);
        if (a.V_out) vv = *reinterpret_cast<const uint4*>(a.V + src);
        if (a.K_out) *reinterpret_cast<uint4*>(a.K_out + dst) = kv;
        if (a.V_out) *reinterpret_cast<uint4*>(a.V_out + dst) = vv;
      }
    }
  }
}

bool dense_supported(const Layout& lay, int b, int G, bool has_q) {
  return lay.dtype == DT_BF16 && lay.n <= 256 && b <= kMaxB && (!has_q || G <= 8);
}

hipError_t launch_retain_dense(const void* K, const void* V, const void* Q, int G, const float* s_in,
                               const Layout& lay, int b, float lambda, float eps, float* s_out,
                               int32_t* idx_sorted, int32_t* pick_order, float* pick_gain,
                               void* K_out, void* V_out, hipStream_t st) {
  DenseArgs a;
  a.K = static_cast<const char*>(K); a.V = static_cast<const char*>(V);
  a.Q = static_cast<const char*>(Q); a.s_in = s_in; a.s_out = s_out;
  a.idx_sorted = idx_sorted; a.pick_order = pick_order; a.pick_gain = pick_gain;
  a.K_out = static_cast<char*>(K_out); a.V_out = static_cast<char*>(V_out);
  a.stride_head = lay.stride_head; a.stride_tok = lay.stride_tok;
  a.n = lay.n; a.b = b; a.G = G; a.lambda = lambda; a.eps = eps;
  dim3 grid(lay.heads), block(kDenseThreads);
  auto go = [&](auto kern, int smem) -> hipError_t {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, block, smem, st, a);
    return hipGetLastError();
  };
  if (lay.n <= 64) return go(&retain_dense_kernel<2>, dense_smem_bytes(2));
  if (lay.n <= 128) return go(&retain_dense_kernel<4>, dense_smem_bytes(4));
  if (lay.n <= 192) return go(&retain_dense_kernel<6>, dense_smem_bytes(6));
  return go(&retain_dense_kernel<8>, dense_smem_bytes(8));
}

}  // namespace kvr
