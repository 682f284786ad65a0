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
#include "kvr_dense_common.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

constexpr int kMaxB = 256;
__host__ __device__ constexpr int dense_smem_bytes(int NT) {
  // region A | s_l[N32] | rinv[N32] | red[64] | idx_l[kMaxB] | order_l[kMaxB] | gain_l[kMaxB]
  return dense_region_a(NT) + NT * 32 * 4 * 2 + 64 * 4 + kMaxB * 4 * 3;
}

struct DenseArgs {
  const char* K; const char* V; const char* Q; const float* s_in;
  float* s_out; int32_t* idx_sorted; int32_t* pick_order; float* pick_gain;
  char* K_out; char* V_out;
  long long stride_head, stride_tok;   // elements
  int n, b, G, heads;
  float lambda, eps;
  int only_marked;                     // process only heads whose idx_sorted[h*b] is -1
  const int32_t* b_h;                  // per-head budgets <= b (rows of the outputs stay b apart), or null
};

// Workgroups are persistent: each walks over heads blockIdx.x, blockIdx.x + gridDim.x, ...
// While one wave runs the pick chain of a head, the rows (and scores) of the workgroup's next
// head are already on their way from HBM into registers.
template <int NT>
__global__ __launch_bounds__(kDenseThreads, (NT <= 6 ? 2 : 1)) void retain_dense_kernel(DenseArgs a) {
  constexpr int N32 = NT * 32;
  constexpr int NQ = NT / 2;                         // tokens per lane in the greedy wave
  constexpr int NTILES = NT * (NT + 1) / 2;
  constexpr int MAXT = NT + 1;                       // Gram tiles per working wave
  constexpr int kIters = NT * 32 * 16 / kDenseThreads;
  extern __shared__ __align__(16) char smem[];
  char* stage = smem;                                // staged rows (phase 1) ...
  float* tri = reinterpret_cast<float*>(smem);       // ... later the packed cosine triangle
  float* s_l = reinterpret_cast<float*>(smem + dense_region_a(NT));
  float* rinv = s_l + N32;
  float* red = rinv + N32;
  int32_t* idx_l = reinterpret_cast<int32_t*>(red + 64);
  int32_t* order_l = idx_l + kMaxB;
  float* gain_l = reinterpret_cast<float*>(order_l + kMaxB);

  const int tid0 = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid0 >> 6);
  const int n = a.n, b = a.b;
  const bool diverse = a.lambda != 0.0f;
  const bool need_v = diverse && b > 1;

  uint4 vpre[kIters];                                // rows of V of the head about to be processed
  float spre = -INFINITY;                            // its score for token `tid` (scores given)
  auto prefetch = [&](int hh, int tid) {
    if (need_v) load_rows<NT>(a.V + hh * a.stride_head * 2, a.stride_tok, n, tid, vpre);
    if (!a.Q && tid < N32) spre = tid < n ? a.s_in[static_cast<long long>(hh) * n + tid] : -INFINITY;
  };
  // First head at or after h0 on this workgroup's stride that is to be processed.  With
  // only_marked set, an earlier kernel has already finished every head it did not mark; 64
  // marks are looked at per round trip to memory.
  auto next_head = [&](int h0) -> int {
    if (!a.only_marked) return h0;
    const int ln = tid0 & 63;
    for (long long base = h0; base < a.heads; base += 64ll * gridDim.x) {
      const long long hh = base + static_cast<long long>(ln) * gridDim.x;
      const bool todo = hh < a.heads && a.idx_sorted[hh * a.b] == -1;
      const unsigned long long m = __ballot(todo);
      if (m) return static_cast<int>(base) + (__ffsll(static_cast<long long>(m)) - 1) * static_cast<int>(gridDim.x);
    }
    return a.heads;
  };
  int h = next_head(blockIdx.x);
  if (h < a.heads) prefetch(h, tid0);

  while (h < a.heads) {
    const int h_next = next_head(h + gridDim.x);
    const long long head_off = h * a.stride_head * 2;  // bytes
    // The thread index is made opaque once per head: otherwise every per-lane LDS address of
    // the body is loop-invariant, gets hoisted out of the head loop and lives in registers.
    int tid = tid0;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, hf = lane >> 5;
    // ---------------------------------------------------------------- scores
    if (a.Q) {
      {
        uint4 kreg[kIters];
        load_rows<NT>(a.K + head_off, a.stride_tok, n, tid, kreg);
        store_rows<NT>(stage, tid, kreg);
      }
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
      lds_barrier();
      constexpr int BPW = (NT + 3) / 4;              // token blocks per wave
      float z[BPW][4];
      const float scale = 0.08838834764831845f;      // 1/sqrt(128)
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
          z[k][r] = live ? acc[r] * scale : -INFINITY; // rows g = hf*4 + r of the 32x32 tile
          zmax[r] = fmaxf(zmax[r], z[k][r]);
        }
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float v = half_max_at_31(zmax[r]);
        if ((lane & 31) == 31) red[wave * 8 + hf * 4 + r] = v;
      }
      lds_barrier();
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
          z[k][r] = __expf(z[k][r] - zmax[r]);       // exp(-inf) = 0 for padded tokens
          zsum[r] += z[k][r];
        }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float v = half_sum_at_31(zsum[r]);
        if ((lane & 31) == 31) red[32 + wave * 8 + hf * 4 + r] = v;
      }
      lds_barrier();
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
        p += __shfl_xor(p, 32, kWave);               // queries 0-3 live in lanes 0-31, 4-7 in 32-63
        const int j = I * 32 + (lane & 31);
        if (I < NT && hf == 0) {
          s_l[j] = j < n ? p : -INFINITY;             // padding never competes
          if (j < n && a.s_out) a.s_out[static_cast<long long>(h) * n + j] = p;
        }
      }
      lds_barrier();                                // K fragments are dead; s_l is complete
    } else {
      if (tid < N32) s_l[tid] = spre;
    }

    // ------------------------------------------------ Gram -> packed cosines
    if (need_v) {
      store_rows<NT>(stage, tid, vpre);
      lds_barrier();
      // Tile rows are paired so that every working wave owns NT+1 tiles: wave w takes row
      // NT-1-w (tiles J = 0..NT-1-w) and row w (tiles J = 0..w).  The row block's fragments stay
      // in registers while the column blocks stream out of LDS.
      f32x16 acc[MAXT];
      const bool working = wave < NT / 2;
      const int n1 = NT - wave;                       // tiles of the first row
      if (working) {
        bf16x8 af[8];
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) af[ks] = frag_at(stage, NT - 1 - wave, ks, lane);
#pragma unroll
        for (int sl = 0; sl < MAXT; ++sl) {
          if (sl == n1) {
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) af[ks] = frag_at(stage, wave, ks, lane);
          }
          const int I = sl < n1 ? NT - 1 - wave : wave;
          const int J = sl < n1 ? sl : sl - n1;
          acc[sl] = f32x16{0};
          __builtin_amdgcn_sched_barrier(0);          // keep one tile's fragment loads in flight, not all of them
#pragma unroll
          for (int ks = 0; ks < 8; ++ks)
            acc[sl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks], frag_at(stage, J, ks, lane), acc[sl], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
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
      for (int j = tid; j < N32; j += kDenseThreads) rinv[j] = 1.0f / (sqrtf(rinv[j]) + a.eps);
      lds_barrier();
      if (working) {
#pragma unroll
        for (int sl = 0; sl < MAXT; ++sl) {
          const int I = sl < n1 ? NT - 1 - wave : wave;
          const int J = sl < n1 ? sl : sl - n1;
          write_cos_tile(tri, rinv, acc[sl], I, J, lane);
        }
      }
    }
    lds_barrier();
    // the next head of this workgroup starts its trip from HBM now
    if (h_next < a.heads) prefetch(h_next, tid);

    // ---------------------------------------------------------------- greedy
    // the head's own budget: its picks are the first bh picks of a run for b, so the chain stops there
    const int bh = a.b_h ? __builtin_amdgcn_readfirstlane(min(max(a.b_h[h], 0), b)) : b;
    if (wave == 0) {
      const int brun = bh < 1 ? 1 : bh;
      pick_chain<NQ>(s_l, tri, order_l, gain_l, n, brun, a.lambda, diverse, lane);
      sort_picks<NQ>(order_l, idx_l, reinterpret_cast<int32_t*>(rinv), brun, lane, nullptr);   // rinv is dead by now
    }
    lds_barrier();

    // ------------------------------------------------- outputs and compaction
    const long long ob = static_cast<long long>(h) * b;
    for (int t = tid; t < b; t += kDenseThreads) {              // entries past the head's budget are padding
      a.idx_sorted[ob + t] = t < bh ? idx_l[t] : -1;
      if (a.pick_order) a.pick_order[ob + t] = t < bh ? order_l[t] : -1;
      if (a.pick_gain) a.pick_gain[ob + t] = t < bh ? gain_l[t] : -INFINITY;
    }
    if ((a.K_out || a.V_out) && bh > 0)
      compact_rows<4>(a.K, a.V, a.K_out, a.V_out, head_off, a.stride_tok, idx_l, n, bh, ob, tid, kDenseThreads);
    lds_barrier();                                   // idx_l / s_l are reused by the next head
    h = h_next;
  }
}

bool dense_supported(const Layout& lay, int b, int G, bool has_q) {
  return lay.dtype == DT_BF16 && lay.n <= 256 && b <= kMaxB && (!has_q || G <= 8);
}

hipError_t launch_retain_dense(const void* K, const void* V, const void* Q, int G, const float* s_in,
                               const Layout& lay, int b, float lambda, float eps, float* s_out,
                               int32_t* idx_sorted, int32_t* pick_order, float* pick_gain,
                               void* K_out, void* V_out, hipStream_t st, bool only_marked, const int32_t* b_h) {
  DenseArgs a;
  a.only_marked = only_marked ? 1 : 0;
  a.b_h = b_h;
  a.K = static_cast<const char*>(K); a.V = static_cast<const char*>(V);
  a.Q = static_cast<const char*>(Q); a.s_in = s_in; a.s_out = s_out;
  a.idx_sorted = idx_sorted; a.pick_order = pick_order; a.pick_gain = pick_gain;
  a.K_out = static_cast<char*>(K_out); a.V_out = static_cast<char*>(V_out);
  a.stride_head = lay.stride_head; a.stride_tok = lay.stride_tok;
  a.n = lay.n; a.b = b; a.G = G; a.heads = lay.heads; a.lambda = lambda; a.eps = eps;
  const int cus = cu_count();
  dim3 block(kDenseThreads);
  auto go = [&](auto kern, int smem) -> hipError_t {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    // persistent workgroups: as many as fit the chip at once (LDS-limited), never more than heads
    int per_cu = 160 * 1024 / smem;
    per_cu = per_cu < 1 ? 1 : (per_cu > 4 ? 4 : per_cu);
    const int blocks = lay.heads < cus * per_cu ? lay.heads : cus * per_cu;
    dim3 grid(blocks);
    hipLaunchKernelGGL(kern, grid, block, smem, st, a);
    return hipGetLastError();
  };
  if (lay.n <= 64) return go(&retain_dense_kernel<2>, dense_smem_bytes(2));
  if (lay.n <= 128) return go(&retain_dense_kernel<4>, dense_smem_bytes(4));
  if (lay.n <= 192) return go(&retain_dense_kernel<6>, dense_smem_bytes(6));
  return go(&retain_dense_kernel<8>, dense_smem_bytes(8));
}

}  // namespace kvr
