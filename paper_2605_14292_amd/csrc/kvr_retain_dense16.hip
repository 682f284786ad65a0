// The whole retention event (paper Sec. 4.1: scores -> Eq. 1 signatures -> Algorithm 1 ->
// kept rows) for bf16 heads of 128 < n <= 256 tokens when the call has so few heads that every
// workgroup gets a CU to itself (a decode-time event of one sequence: layers x KV heads <= CUs).
// Throughput is then the latency of one head, so the parallel phases -- rows, logits, Gram,
// cosine triangle, outputs -- are spread over sixteen wave64s instead of four; the b dependent
// picks stay on one wave.  Same arithmetic, same LDS layout and same helpers as
// retain_dense_kernel, which remains the kernel for batched calls (several heads per CU).
#include "kvr_dense_common.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

constexpr int kD16Threads = 1024;
constexpr int kD16Waves = kD16Threads / 64;
constexpr int kD16MaxB = 256;

__host__ __device__ constexpr int dense16_smem_bytes(int NT) {
  // region A | s_l[N32] | rinv[N32] | red[2][16][8] | idx_l | order_l | gain_l
  return dense_region_a(NT) + NT * 32 * 4 * 2 + 2 * kD16Waves * 8 * 4 + kD16MaxB * 4 * 3;
}

struct Dense16Args {
  const char* K; const char* V; const char* Q; const float* s_in;
  float* s_out; int32_t* idx_sorted; int32_t* pick_order; float* pick_gain;
  char* K_out; char* V_out;
  long long stride_head, stride_tok;   // elements
  int n, b, G;
  float lambda, eps;
  const int32_t* b_h;                  // per-head budgets <= b (rows of the outputs stay b apart), or null
};

template <int NT>
__global__ __launch_bounds__(kD16Threads, 1) void retain_dense16_kernel(Dense16Args a) {
  constexpr int N32 = NT * 32;
  constexpr int NQ = NT / 2;
  constexpr int NTILES = NT * (NT + 1) / 2;
  constexpr int MAXT = (NTILES + kD16Waves - 1) / kD16Waves;
  constexpr int kIters = N32 * 16 / kD16Threads;      // 16-byte pieces of the head's rows per thread
  extern __shared__ __align__(16) char smem[];
  char* stage = smem;                                // staged rows ...
  float* tri = reinterpret_cast<float*>(smem);       // ... later the packed cosine triangle
  float* s_l = reinterpret_cast<float*>(smem + dense_region_a(NT));
  float* rinv = s_l + N32;
  float* red = rinv + N32;                           // [2][16 waves][8 queries]
  int32_t* idx_l = reinterpret_cast<int32_t*>(red + 2 * kD16Waves * 8);
  int32_t* order_l = idx_l + kD16MaxB;
  float* gain_l = reinterpret_cast<float*>(order_l + kD16MaxB);

  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int h = blockIdx.x;
  const int n = a.n, b = a.b;
  const int bh = a.b_h ? min(max(a.b_h[h], 0), b) : b;  // the head's own budget
  const bool diverse = a.lambda != 0.0f;
  const bool need_v = diverse && b > 1;
  const long long head_off = h * a.stride_head * 2;   // bytes
  const int chunk = tid & 15, r0 = tid >> 4;          // 64 rows per step of the row loops

  // both tensors start their trip from memory at once; rows past n read as zero
  uint4 vreg[kIters], kreg[kIters];
#pragma unroll
  for (int k = 0; k < kIters; ++k) {
    const int row = r0 + 64 * k;
    vreg[k] = kreg[k] = make_uint4(0u, 0u, 0u, 0u);
    if (row < n) {
      const long long off = head_off + (row * a.stride_tok + chunk * 8) * 2;
      if (a.Q) kreg[k] = *reinterpret_cast<const uint4*>(a.K + off);
      if (need_v) vreg[k] = *reinterpret_cast<const uint4*>(a.V + off);
    }
  }

  // ---------------------------------------------------------------- scores
  if (a.Q) {
#pragma unroll
    for (int k = 0; k < kIters; ++k)
      *reinterpret_cast<uint4*>(stage + (r0 + 64 * k) * kRowPitch + chunk * 16) = kreg[k];
    bf16x8 qf[8];
    {
      const int g = lane & 31;
      const char* qp = a.Q + (static_cast<long long>(h) * a.G + g) * kD * 2 + hf * 16;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        uint4 w = make_uint4(0u, 0u, 0u, 0u);
        if (g < a.G && wave < NT) w = *reinterpret_cast<const uint4*>(qp + ks * 32);
        qf[ks] = *reinterpret_cast<bf16x8*>(&w);
      }
    }
    lds_barrier();
    // wave I < NT takes token block I: lane (token, hf) ends up with the logits of queries hf*4 .. hf*4+3
    const bool has_block = wave < NT;
    const bool live = has_block && (wave * 32 + (lane & 31)) < n;
    const float scale = 0.08838834764831845f;      // 1/sqrt(128)
    float z[4];
    {
      f32x16 acc = {0};
      if (has_block) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[ks], frag_at(stage, wave, ks, lane), acc, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) z[r] = live ? acc[r] * scale : -INFINITY;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float v = half_max_at_31(z[r]);
      if ((lane & 31) == 31) red[wave * 8 + hf * 4 + r] = v;
    }
    lds_barrier();
    float zmax[4], zsum[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int g = hf * 4 + r;
      float m = red[g];
#pragma unroll
      for (int u = 1; u < NT; ++u) m = fmaxf(m, red[u * 8 + g]);
      zmax[r] = m;
      z[r] = __expf(z[r] - zmax[r]);                 // exp(-inf) = 0 for padded tokens
      zsum[r] = z[r];
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float v = half_sum_at_31(zsum[r]);
      if ((lane & 31) == 31) red[kD16Waves * 8 + wave * 8 + hf * 4 + r] = v;
    }
    lds_barrier();
    const float invG = 1.0f / static_cast<float>(a.G);
    float p = 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int g = hf * 4 + r;
      float tot = 0.f;
#pragma unroll
      for (int u = 0; u < NT; ++u) tot += red[kD16Waves * 8 + u * 8 + g];
      p = fmaf(z[r], g < a.G ? invG / tot : 0.f, p);
    }
    p += __shfl_xor(p, 32, kWave);                 // queries 0-3 live in lanes 0-31, 4-7 in 32-63
    if (has_block && hf == 0) {
      const int j = wave * 32 + (lane & 31);
      s_l[j] = j < n ? p : -INFINITY;               // padding never competes
      if (j < n && a.s_out) a.s_out[static_cast<long long>(h) * n + j] = p;
    }
    lds_barrier();                                // K fragments are dead; s_l is complete
  } else {
    if (tid < N32) s_l[tid] = tid < n ? a.s_in[static_cast<long long>(h) * n + tid] : -INFINITY;
  }

  // ------------------------------------------------ Gram -> packed cosines
  if (need_v) {
#pragma unroll
    for (int k = 0; k < kIters; ++k)
      *reinterpret_cast<uint4*>(stage + (r0 + 64 * k) * kRowPitch + chunk * 16) = vreg[k];
    lds_barrier();
    // tile t of the lower triangle: row block I, column block J <= I; wave w takes tiles w, w + 16, ...
    f32x16 acc[MAXT];
#pragma unroll
    for (int sl = 0; sl < MAXT; ++sl) {
      const int tile = wave + kD16Waves * sl;
      acc[sl] = f32x16{0};
      if (tile < NTILES) {
        int I = 0;
        while ((I + 1) * (I + 2) / 2 <= tile) ++I;
        const int J = tile - I * (I + 1) / 2;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
          acc[sl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_at(stage, I, ks, lane), frag_at(stage, J, ks, lane),
                                                            acc[sl], 0, 0, 0);
        if (I == J) {                               // squared norms sit on the diagonal
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int il = (r >> 2) * 8 + hf * 4 + (r & 3);
            if (il == (lane & 31)) rinv[I * 32 + il] = acc[sl][r];
          }
        }
      }
    }
    lds_barrier();                                // staged rows are dead from here on
    if (tid < N32) rinv[tid] = 1.0f / (sqrtf(rinv[tid]) + a.eps);
    lds_barrier();
#pragma unroll
    for (int sl = 0; sl < MAXT; ++sl) {
      const int tile = wave + kD16Waves * sl;
      if (tile < NTILES) {
        int I = 0;
        while ((I + 1) * (I + 2) / 2 <= tile) ++I;
        const int J = tile - I * (I + 1) / 2;
        write_cos_tile(tri, rinv, acc[sl], I, J, lane);
      }
    }
  }
  lds_barrier();

  // ---------------------------------------------------------------- greedy
  if (wave == 0) {
    const int brun = bh < 1 ? 1 : bh;
    pick_chain<NQ>(s_l, tri, order_l, gain_l, n, brun, a.lambda, diverse, lane);
    sort_picks<NQ>(order_l, idx_l, reinterpret_cast<int32_t*>(rinv), brun, lane, nullptr);   // rinv is dead by now
  }
  lds_barrier();

  // ------------------------------------------------- outputs and compaction
  const long long ob = static_cast<long long>(h) * b;
  for (int t = tid; t < b; t += kD16Threads) {                   // entries past the head's budget are padding
    a.idx_sorted[ob + t] = t < bh ? idx_l[t] : -1;
    if (a.pick_order) a.pick_order[ob + t] = t < bh ? order_l[t] : -1;
    if (a.pick_gain) a.pick_gain[ob + t] = t < bh ? gain_l[t] : -INFINITY;
  }
  if ((a.K_out || a.V_out) && bh > 0)
    compact_rows<4>(a.K, a.V, a.K_out, a.V_out, head_off, a.stride_tok, idx_l, n, bh, ob, tid, kD16Threads);
}

bool dense16_supported(const Layout& lay, int b, int G, bool has_q, int cus) {
  return lay.dtype == DT_BF16 && lay.n > 128 && lay.n <= 256 && b <= kD16MaxB && (!has_q || G <= 8) &&
         lay.heads <= cus;
}

hipError_t launch_retain_dense16(const void* K, const void* V, const void* Q, int G, const float* s_in,
                                 const Layout& lay, int b, float lambda, float eps, float* s_out,
                                 int32_t* idx_sorted, int32_t* pick_order, float* pick_gain, void* K_out,
                                 void* V_out, hipStream_t st, const int32_t* b_h) {
  Dense16Args a;
  a.K = static_cast<const char*>(K); a.V = static_cast<const char*>(V);
  a.Q = static_cast<const char*>(Q); a.s_in = s_in; a.s_out = s_out;
  a.idx_sorted = idx_sorted; a.pick_order = pick_order; a.pick_gain = pick_gain;
  a.K_out = static_cast<char*>(K_out); a.V_out = static_cast<char*>(V_out);
  a.stride_head = lay.stride_head; a.stride_tok = lay.stride_tok;
  a.n = lay.n; a.b = b; a.G = G; a.lambda = lambda; a.eps = eps; a.b_h = b_h;
  auto go = [&](auto kern, int smem) -> hipError_t {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(lay.heads), dim3(kD16Threads), smem, st, a);
    return hipGetLastError();
  };
  if (lay.n <= 192) return go(&retain_dense16_kernel<6>, dense16_smem_bytes(6));
  return go(&retain_dense16_kernel<8>, dense16_smem_bytes(8));
}

}  // namespace kvr
