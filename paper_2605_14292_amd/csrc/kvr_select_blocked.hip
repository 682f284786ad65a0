// Greedy selection (paper Sec. 4.1, Algorithm 1) for heads with 256 < n <= 4096
// bf16 tokens, followed by the compaction of the kept rows.
//
// Algorithm 1 reads only the b rows of its n x n cosine matrix that belong to
// picked tokens, one row per pick.  A single row is a matrix-vector product and
// would leave the matrix cores idle, so rows are produced sixteen at a time,
// speculatively: whenever the next pick has no row yet, the sixteen currently
// best candidates (the top few of every wave's token range) get their rows
// against all n tokens in one pass of bf16 MFMA (16x16x32, fp32 accumulate) over
// V.  Gains only ever decrease, so the following picks mostly come from those
// sixteen; on the benchmark inputs about eight picks are served per pass, i.e. V
// is streamed ~b/8 times instead of b times.  Nothing is approximated: every
// pick is still the exact argmax of Eq. 2 over all unselected tokens, and a pick
// outside the speculated set simply starts a new pass.
//
// Layout: one workgroup per head, W = n/256 (rounded up to a power of two)
// wave64s.  Token j = 256*w + 64*k + lane belongs to wave w, lane `lane`, slot k
// (k < 4); its score, running maximum m and inverse norm stay in that lane's
// registers for the whole event.  The MFMA result tile has candidates along
// rows and tokens along columns; a small per-wave LDS scratch turns it into
// "my four tokens x sixteen candidates" per lane, after which serving a pick
// is lane-local.  Each pick is a DPP max-reduction inside every wave, one
// 8-byte slot per wave in LDS, one barrier, and a second DPP reduction over the
// wave results (ties go to the lowest token index at both levels).
#include "kvr_device.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kBlkRows = 16;        // speculated rows per pass
constexpr int kBlkMaxB = 1024;      // pick lists kept in LDS
constexpr int kScrPitch = 20;       // floats per token column in the transpose scratch (bank spread)

__device__ __forceinline__ float blk_wave_max(float v) {
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
__device__ __forceinline__ float blk_hw_max(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ void blk_wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

struct BlockedArgs {
  const char* K; const char* V; const float* s_in;
  int32_t* idx_sorted; int32_t* pick_order; float* pick_gain;
  char* K_out; char* V_out;
  long long stride_head, stride_tok;   // elements
  int n, b;
  float lambda, eps;
};

__host__ __device__ constexpr int blocked_smem_bytes(int W) {
  // slots[2][16]{gain,idx} | cand[16] | candr[16] | wcount[16] | order[kBlkMaxB] | gain[kBlkMaxB] |
  // idxs[kBlkMaxB] | rn[256*W] (inverse norms, later pick flags) | scratch[W][16*kScrPitch]
  return (64 + 16 + 16 + 16 + 3 * kBlkMaxB + 256 * W + W * 16 * kScrPitch) * 4;
}

#define KVR_CASE(C)                                                      \
  case C:                                                                \
    v0 = vals[0][C]; v1 = vals[1][C]; v2 = vals[2][C]; v3 = vals[3][C];  \
    break;

template <int W>
__global__ __launch_bounds__(64 * W) void select_blocked_kernel(BlockedArgs a) {
  constexpr int NT = 64 * W;                       // threads
  constexpr int RW = kBlkRows / W;                 // candidates contributed per wave and pass
  extern __shared__ __align__(16) float smem[];
  float* slot_gain = smem;                         // [2][16]
  int32_t* slot_idx = reinterpret_cast<int32_t*>(smem + 32);   // [2][16]
  int32_t* cand_l = reinterpret_cast<int32_t*>(smem + 64);     // [16] token of each speculated row, -1 = none
  float* candr = smem + 80;                        // [16] its inverse norm
  int32_t* wcount = reinterpret_cast<int32_t*>(smem + 96);     // [16]
  int32_t* order_l = reinterpret_cast<int32_t*>(smem + 112);
  float* gain_l = smem + 112 + kBlkMaxB;
  int32_t* idxs_l = reinterpret_cast<int32_t*>(smem + 112 + 2 * kBlkMaxB);
  float* rn = smem + 112 + 3 * kBlkMaxB;           // [256*W]
  int32_t* flag = reinterpret_cast<int32_t*>(rn);
  float* scratch_all = rn + 256 * W;

  const int h = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = a.n, b = a.b;
  const long long head_off = h * a.stride_head * 2;           // bytes
  const char* Vh = a.V + head_off;
  const bool diverse = a.lambda != 0.0f;
  const int base = w * 256;
  float* scratch = scratch_all + w * 16 * kScrPitch;

  // ---- per-token state in registers
  float s[4], m[4], r[4];
  int tok[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    tok[k] = base + 64 * k + lane;
    s[k] = tok[k] < n ? a.s_in[static_cast<long long>(h) * n + tok[k]] : -INFINITY;
    m[k] = 0.f;
    r[k] = 0.f;
  }
  if (diverse && b > 1) {
    // inverse norms (Eq. 1): 16 lanes per row, coalesced; this is the one full read of V from HBM
    const int c16 = tid & 15;
    for (int j0 = 0; j0 < n; j0 += NT / 16) {
      const int j = j0 + (tid >> 4);
      if (j < n) {
        float x[8];
        load8<DT_BF16>(Vh + (static_cast<long long>(j) * a.stride_tok + c16 * 8) * 2, x);
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = fmaf(x[e], x[e], ss);
        ss = group16_sum(ss);
        if (c16 == 0) rn[j] = 1.0f / (sqrtf(ss) + a.eps);
      }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; ++k) r[k] = tok[k] < n ? rn[tok[k]] : 0.f;
  }

  float vals[4][kBlkRows];       // cos numerators: my token k against speculated row c
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int c = 0; c < kBlkRows; ++c) vals[k][c] = 0.f;
  int cm = -2;                   // lanes 0..15: token of speculated row `lane`
  float crv = 0.f;               // lanes 0..15: its inverse norm
  const float nlam = -a.lambda;
  int par = 0;
  int t = 0;
  bool starved = false;          // no finite gain left (non-finite input only)

  for (; t < b; ++t) {
    // ---- wave-local argmax of the marginal gain
    float av[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) av[k] = fmaf(nlam, m[k], s[k]);
    const float best = blk_hw_max(blk_hw_max(av[0], av[1]), blk_hw_max(av[2], av[3]));
    const float amax_w = blk_wave_max(best);
    int i_w = -1;
#pragma unroll
    for (int k = 3; k >= 0; --k) {
      const unsigned long long eq = __ballot(av[k] == amax_w);
      if (eq) i_w = base + 64 * k + (__ffsll(static_cast<long long>(eq)) - 1);
    }
    if (lane == 0) { slot_gain[par * 16 + w] = amax_w; slot_idx[par * 16 + w] = i_w; }
    __syncthreads();
    // ---- across waves: larger gain, then lower wave (= lower token range)
    const float g = lane < W ? slot_gain[par * 16 + lane] : -INFINITY;
    const int ii = lane < W ? slot_idx[par * 16 + lane] : -1;
    par ^= 1;
    const float gmax = blk_wave_max(g);
    if (!(gmax > -INFINITY)) { starved = true; break; }
    const unsigned long long eqw = __ballot(lane < W && g == gmax);
    const int win = __ffsll(static_cast<long long>(eqw)) - 1;
    const int i = __builtin_amdgcn_readlane(ii, win);
    if (tid == 0) { order_l[t] = i; gain_l[t] = gmax; }
    if (t + 1 == b) { ++t; break; }
    if (!diverse) {
#pragma unroll
      for (int k = 0; k < 4; ++k) s[k] = tok[k] == i ? -INFINITY : s[k];
      continue;
    }
    // ---- is the row of pick i among the speculated ones?
    unsigned long long hit = __ballot(cm == i);
    if (!hit) {
      // ---- new pass: every wave nominates its RW best unselected tokens (i is one of them)
      float ts[4] = {av[0], av[1], av[2], av[3]};
#pragma unroll
      for (int q = 0; q < RW; ++q) {
        const float bq = blk_hw_max(blk_hw_max(ts[0], ts[1]), blk_hw_max(ts[2], ts[3]));
        const float mx = blk_wave_max(bq);
        int cj = -1, ck = 0, cl = 0;
#pragma unroll
        for (int k = 3; k >= 0; --k) {
          const unsigned long long eq = __ballot(ts[k] == mx);
          if (eq) { cl = __ffsll(static_cast<long long>(eq)) - 1; ck = k; cj = base + 64 * k + cl; }
        }
        const float rsel = ck == 0 ? r[0] : ck == 1 ? r[1] : ck == 2 ? r[2] : r[3];
        const float rc = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(rsel), cl));
        const bool ok = mx > -INFINITY;
#pragma unroll
        for (int k = 0; k < 4; ++k) ts[k] = (k == ck && lane == cl) ? -INFINITY : ts[k];
        if (lane == 0) { cand_l[w * RW + q] = ok ? cj : -1; candr[w * RW + q] = ok ? rc : 0.f; }
      }
      __syncthreads();
      cm = lane < kBlkRows ? cand_l[lane] : -2;
      crv = lane < kBlkRows ? candr[lane] : 0.f;
      // A operand: the sixteen candidate rows (lane: row lane%16, k-group lane/16)
      const int kg = lane >> 4;
      const int ci = cand_l[lane & 15];
      bf16x8 af[4];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        uint4 x = make_uint4(0u, 0u, 0u, 0u);
        if (ci >= 0) x = *reinterpret_cast<const uint4*>(Vh + (static_cast<long long>(ci) * a.stride_tok + ks * 32 + kg * 8) * 2);
        af[ks] = *reinterpret_cast<bf16x8*>(&x);
      }
      // stream this wave's 256 tokens through the matrix cores, 16 at a time
      f32x4 acc[16];
#pragma unroll
      for (int sub = 0; sub < 16; ++sub) {
        const int tb = base + sub * 16 + (lane & 15);
        acc[sub] = f32x4{0.f, 0.f, 0.f, 0.f};
        uint4 x[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          x[ks] = make_uint4(0u, 0u, 0u, 0u);
          if (tb < n) x[ks] = *reinterpret_cast<const uint4*>(Vh + (static_cast<long long>(tb) * a.stride_tok + ks * 32 + kg * 8) * 2);
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
          acc[sub] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[ks], *reinterpret_cast<bf16x8*>(&x[ks]), acc[sub], 0, 0, 0);
      }
      // A result tile has token column lane%16 and candidates 4*(lane/16)+0..3 in each lane.
      // Turn it into "token sub*16+col against all sixteen candidates" in the lane that owns
      // that token (lane group sub%4, slot sub/4) through the wave's LDS scratch.
#pragma unroll
      for (int sub = 0; sub < 16; ++sub) {
        *reinterpret_cast<f32x4*>(scratch + (lane & 15) * kScrPitch + 4 * kg) = acc[sub];
        blk_wave_sync();
        if (kg == (sub & 3)) {
#pragma unroll
          for (int c4 = 0; c4 < 4; ++c4) {
            const f32x4 vv = *reinterpret_cast<const f32x4*>(scratch + (lane & 15) * kScrPitch + 4 * c4);
            vals[sub >> 2][4 * c4 + 0] = vv[0]; vals[sub >> 2][4 * c4 + 1] = vv[1];
            vals[sub >> 2][4 * c4 + 2] = vv[2]; vals[sub >> 2][4 * c4 + 3] = vv[3];
          }
        }
        blk_wave_sync();
      }
      hit = __ballot(cm == i);
    }
    const int c = __ffsll(static_cast<long long>(hit)) - 1;      // 0..15 (i is always nominated)
    const float rc = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(crv), c & 15));
    float v0 = 0.f, v1 = 0.f, v2 = 0.f, v3 = 0.f;
    switch (c) {
      KVR_CASE(0) KVR_CASE(1) KVR_CASE(2) KVR_CASE(3) KVR_CASE(4) KVR_CASE(5) KVR_CASE(6) KVR_CASE(7)
      KVR_CASE(8) KVR_CASE(9) KVR_CASE(10) KVR_CASE(11) KVR_CASE(12) KVR_CASE(13) KVR_CASE(14) KVR_CASE(15)
      default: break;
    }
    m[0] = blk_hw_max(m[0], v0 * rc * r[0]);
    m[1] = blk_hw_max(m[1], v1 * rc * r[1]);
    m[2] = blk_hw_max(m[2], v2 * rc * r[2]);
    m[3] = blk_hw_max(m[3], v3 * rc * r[3]);
#pragma unroll
    for (int k = 0; k < 4; ++k) s[k] = tok[k] == i ? -INFINITY : s[k];
  }

  // ---- sort(S): flag the picked tokens, ascending indices by prefix counts
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 4; ++k) flag[base + 64 * k + lane] = 0;
  __syncthreads();
  for (int u = tid; u < t; u += NT) flag[order_l[u]] = 1;
  __syncthreads();
  if (starved) {
    // Non-finite input only: fill the remaining picks with the lowest unpicked tokens.
    if (tid == 0) {
      int j = 0;
      for (int u = t; u < b; ++u) {
        while (j < n && flag[j]) ++j;
        order_l[u] = j; gain_l[u] = -INFINITY; flag[j] = 1;
      }
    }
    __syncthreads();
  }
  {
    unsigned long long sel[4];
    int cnt = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      sel[k] = __ballot(tok[k] < n && flag[tok[k]] != 0);
      cnt += __popcll(sel[k]);
    }
    if (lane == 0) wcount[w] = cnt;
    __syncthreads();
    int off = 0;
    for (int u = 0; u < w; ++u) off += wcount[u];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if ((sel[k] >> lane) & 1ull) {
        const int rank = off + __popcll(sel[k] & ((1ull << lane) - 1ull));
        if (rank < b) idxs_l[rank] = tok[k];
      }
      off += __popcll(sel[k]);
    }
  }
  __syncthreads();
  const long long ob = static_cast<long long>(h) * b;
  for (int u = tid; u < b; u += NT) {
    a.idx_sorted[ob + u] = idxs_l[u];
    if (a.pick_order) a.pick_order[ob + u] = order_l[u];
    if (a.pick_gain) a.pick_gain[ob + u] = gain_l[u];
  }
  if (a.K_out || a.V_out) {
    const int chunk = tid & 15;
    for (int t0 = 0; t0 < b; t0 += NT / 16) {
      const int u = t0 + (tid >> 4);
      if (u < b) {
        const int it = min(max(idxs_l[u], 0), n - 1);
        const long long src = head_off + (static_cast<long long>(it) * a.stride_tok + chunk * 8) * 2;
        const long long dst = ((ob + u) * kD + chunk * 8) * 2;
        uint4 kv, vv;
        if (a.K_out) kv = *reinterpret_cast<const uint4*>(a.K + src);
        if (a.V_out) vv = *reinterpret_cast<const uint4*>(a.V + src);
        if (a.K_out) *reinterpret_cast<uint4*>(a.K_out + dst) = kv;
        if (a.V_out) *reinterpret_cast<uint4*>(a.V_out + dst) = vv;
      }
    }
  }
}

bool blocked_supported(const Layout& lay, int b) {
  return lay.dtype == DT_BF16 && lay.n > 256 && lay.n <= 4096 && b <= kBlkMaxB;
}

hipError_t launch_select_blocked(const void* K, const void* V, const float* s, const Layout& lay, int b,
                                 float lambda, float eps, int32_t* idx_sorted, int32_t* pick_order,
                                 float* pick_gain, void* K_out, void* V_out, hipStream_t st) {
  BlockedArgs a;
  a.K = static_cast<const char*>(K); a.V = static_cast<const char*>(V); a.s_in = s;
  a.idx_sorted = idx_sorted; a.pick_order = pick_order; a.pick_gain = pick_gain;
  a.K_out = static_cast<char*>(K_out); a.V_out = static_cast<char*>(V_out);
  a.stride_head = lay.stride_head; a.stride_tok = lay.stride_tok;
  a.n = lay.n; a.b = b; a.lambda = lambda; a.eps = eps;
  dim3 grid(lay.heads);
  auto go = [&](auto kern, int W) -> hipError_t {
    const int smem = blocked_smem_bytes(W);
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, dim3(64 * W), smem, st, a);
    return hipGetLastError();
  };
  const int waves = (lay.n + 255) / 256;
  if (waves <= 2) return go(&select_blocked_kernel<2>, 2);
  if (waves <= 4) return go(&select_blocked_kernel<4>, 4);
  if (waves <= 8) return go(&select_blocked_kernel<8>, 8);
  return go(&select_blocked_kernel<16>, 16);
}

}  // namespace kvr
