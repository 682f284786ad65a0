// Greedy selection (paper Sec. 4.1, Algorithm 1) for heads with 256 < n <= 4096
// bf16 tokens, followed by the compaction of the kept rows.
//
// Algorithm 1 reads only the b rows of its n x n cosine matrix that belong to
// picked tokens, one row per pick.  A single row is a matrix-vector product and
// would leave the matrix cores idle, so rows are produced sixteen at a time,
// speculatively: whenever the next pick has no row yet, sixteen currently
// strong candidates (the best few of every wave's token range) get their rows
// against all n tokens in one pass of bf16 MFMA (16x16x32, fp32 accumulate) over
// V.  Gains only ever decrease (m only grows), so the following picks mostly
// come from those sixteen: V is streamed roughly b/8 times instead of b times.
//
// Nothing is approximated.  Between passes the sixteen candidates race among
// themselves with exact gains (all candidate-to-candidate cosines are in the
// pass), against the best gain any other token had when the others were last
// brought up to date.  That value can only have dropped since, so a candidate
// that beats it (gain, then lower index) is the exact argmax of Eq. 2 over all
// unselected tokens.  When no candidate beats it, the rows picked since are
// applied to every token's m, the bound is recomputed, and if an outside token
// still wins a new pass starts with that token among the nominees.
//
// Layout: one workgroup per head, W = n/256 (rounded up to a power of two)
// wave64s.  Token j = 256*w + 64*k + lane belongs to wave w, lane `lane`, slot k
// (k < 4); its score, running maximum m and inverse norm stay in that lane's
// registers for the whole event.  V is streamed through a wave-private padded
// LDS stage (coalesced 16-byte global loads, next chunk in flight while the
// current one is multiplied).  The MFMA result tile has candidates along rows
// and tokens along columns; the same LDS area turns it into "my four tokens x
// sixteen candidates" per lane, after which serving a pick is lane-local.
#include "kvr_device.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kBlkRows = 16;        // speculated rows per pass
constexpr int kBlkMaxB = 1024;      // pick lists kept in LDS
constexpr int kScrPitch = 20;       // floats per token column in the transpose scratch (bank spread)
constexpr int kStgPitch = 272;      // bytes per staged row (256 + 16)

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
// max over lanes 0..15 only (the sixteen candidates), wave-uniform result
__device__ __forceinline__ float blk_row0_max(float v) {
  asm volatile(
      "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_shr:1 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_shr:2 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_shr:4 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_shr:8 row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 1"
      : "+v"(v));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 15));
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
// (gain, index) order of every argmax: larger gain first, then the lower index
__device__ __forceinline__ bool key_beats(float ga, int ia, float gb, int ib) {
  return ga > gb || (ga == gb && ia < ib);
}

struct BlockedArgs {
  const char* K; const char* V; const float* s_in;
  int32_t* idx_sorted; int32_t* pick_order; float* pick_gain;
  char* K_out; char* V_out;
  long long stride_head, stride_tok;   // elements
  int n, b;
  float lambda, eps;
};

template <int W, int S> struct BlkCfg {
  static constexpr int kChunkTok = W <= 4 ? 32 : 16;                // tokens staged per step and wave
  static constexpr int kStageBytes = kChunkTok * kStgPitch + 16 * kScrPitch * 4;   // row stage + transpose scratch
  // floats: slots[2][16]{gain,idx}=64 | cand 16 | candr 16 | cs 16 | cm 16 | wcount 16 | cc 256 |
  //         order kBlkMaxB | gain kBlkMaxB | idxs kBlkMaxB | rn 256*W ; then the per-wave stages
  static constexpr int kFixedFloats = 64 + 16 * 5 + 256 + 3 * kBlkMaxB + 64 * S * W;
  static constexpr int kSmemBytes = kFixedFloats * 4 + W * kStageBytes;
};

#define KVR_CASE(C)                                  \
  case C:                                            \
    _Pragma("unroll") for (int k = 0; k < S; ++k) v[k] = vals[k][C]; \
    break;

template <int W, int S>
__global__ __launch_bounds__(64 * W, (W <= 4 ? 2 : 1)) void select_blocked_kernel(BlockedArgs a) {
  using Cfg = BlkCfg<W, S>;
  constexpr int TPW = 64 * S;                      // tokens per wave
  constexpr int NT = 64 * W;                       // threads
  constexpr int RW = kBlkRows / W;                 // nominees per wave and pass
  constexpr int CH = Cfg::kChunkTok;
  constexpr int LPC = CH / 4;                      // 16-byte global loads per lane and chunk
  extern __shared__ __align__(16) float smem[];
  float* slot_gain = smem;                                         // [2][16]
  int32_t* slot_idx = reinterpret_cast<int32_t*>(smem + 32);       // [2][16]
  int32_t* cand_l = reinterpret_cast<int32_t*>(smem + 64);         // [16] token of each speculated row, -1 = none
  float* candr = smem + 80;                                        // [16] its inverse norm
  float* cs_l = smem + 96;                                         // [16] its score
  float* cm_l = smem + 112;                                        // [16] its m when the pass was built
  int32_t* wcount = reinterpret_cast<int32_t*>(smem + 128);        // [16]
  float* cc = smem + 144;                                          // [16][16] cosine(candidate x, candidate c)
  int32_t* order_l = reinterpret_cast<int32_t*>(smem + 400);
  float* gain_l = smem + 400 + kBlkMaxB;
  int32_t* idxs_l = reinterpret_cast<int32_t*>(smem + 400 + 2 * kBlkMaxB);
  float* rn = smem + 400 + 3 * kBlkMaxB;                           // [256*W] inverse norms, later pick flags
  int32_t* flag = reinterpret_cast<int32_t*>(rn);
  char* stage_all = reinterpret_cast<char*>(rn + TPW * W);

  const int h = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = a.n, b = a.b;
  const long long head_off = h * a.stride_head * 2;               // bytes
  const char* Vh = a.V + head_off;
  const bool diverse = a.lambda != 0.0f;
  const int base = w * TPW;
  char* stage = stage_all + w * Cfg::kStageBytes;
  float* scratch = reinterpret_cast<float*>(stage + Cfg::kChunkTok * kStgPitch);

  // ---- per-token state in registers
  float s[S], m[S], r[S];
  int tok[S], cslot[S];          // cslot: row of the current pass that belongs to this token, or -1
#pragma unroll
  for (int k = 0; k < S; ++k) {
    tok[k] = base + 64 * k + lane;
    s[k] = tok[k] < n ? a.s_in[static_cast<long long>(h) * n + tok[k]] : -INFINITY;
    m[k] = 0.f;
    r[k] = 0.f;
    cslot[k] = -1;
  }
  const float nlam = -a.lambda;
  int par = 0;
  int t = 0;
  bool starved = false;          // no finite gain left (non-finite input only)

  // Workgroup-wide argmax of up to four per-lane values with token ids tok[k]:
  // DPP inside the wave, one LDS slot per wave, one barrier, DPP over the slots.
  auto wg_argmax = [&](const float (&av)[S], float& gbest, int& ibest) {
    float best = av[0];
#pragma unroll
    for (int k = 1; k < S; ++k) best = blk_hw_max(best, av[k]);
    const float amax_w = blk_wave_max(best);
    int i_w = -1;
#pragma unroll
    for (int k = S - 1; k >= 0; --k) {
      const unsigned long long eq = __ballot(av[k] == amax_w);
      if (eq) i_w = base + 64 * k + (__ffsll(static_cast<long long>(eq)) - 1);
    }
    if (lane == 0) { slot_gain[par * 16 + w] = amax_w; slot_idx[par * 16 + w] = i_w; }
    __syncthreads();
    const float g = lane < W ? slot_gain[par * 16 + lane] : -INFINITY;
    const int ii = lane < W ? slot_idx[par * 16 + lane] : -1;
    par ^= 1;
    gbest = blk_wave_max(g);
    const unsigned long long eqw = __ballot(lane < W && g == gbest);   // lowest wave = lowest token range
    ibest = eqw ? __builtin_amdgcn_readlane(ii, __ffsll(static_cast<long long>(eqw)) - 1) : -1;
  };

  if (!diverse || b == 1) {
    // lambda = 0 (or a single pick): plain top-b of the scores, V is never read
    for (; t < b; ++t) {
      float gmax; int i;
      wg_argmax(s, gmax, i);
      if (!(gmax > -INFINITY)) { starved = true; break; }
      if (tid == 0) { order_l[t] = i; gain_l[t] = gmax; }
#pragma unroll
      for (int k = 0; k < S; ++k) s[k] = tok[k] == i ? -INFINITY : s[k];
    }
  } else {
    // ---- inverse norms (Eq. 1): 16 lanes per row, coalesced; the one full read of V from HBM
    {
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
      for (int k = 0; k < S; ++k) r[k] = tok[k] < n ? rn[tok[k]] : 0.f;
    }

    float vals[S][kBlkRows];       // dot products: my token k against speculated row c (set by every pass)
    // candidate state, replicated in lanes 0..15 of every wave (lane = row of the pass)
    int ctok = -1;                 // token of the row, -1 = empty
    float crv = 0.f;               // its inverse norm
    float gs = -INFINITY;          // its score; -inf once picked
    float gm = 0.f;                // its running maximum
    unsigned long long pend = 0;   // rows picked since the other tokens were last updated, 4 bits each
    int np = 0;
    float gout = -INFINITY;        // best gain outside the candidates, as of the last update
    int jout = -1;
    bool out_valid = false;
#ifdef KVR_STATS
    int st_blocks = 0, st_syncs = 0;
#endif

    while (t < b) {
      if (!out_valid) {
        // ---- bring every token up to date with the rows picked since the last update
        for (int q = 0; q < np; ++q) {
          const int c = static_cast<int>((pend >> (4 * q)) & 15ull);
          const float rc = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(crv), c));
          float v[S];
          switch (c) {
            KVR_CASE(0) KVR_CASE(1) KVR_CASE(2) KVR_CASE(3) KVR_CASE(4) KVR_CASE(5) KVR_CASE(6) KVR_CASE(7)
            KVR_CASE(8) KVR_CASE(9) KVR_CASE(10) KVR_CASE(11) KVR_CASE(12) KVR_CASE(13) KVR_CASE(14) KVR_CASE(15)
            default:
#pragma unroll
              for (int k = 0; k < S; ++k) v[k] = 0.f;
              break;
          }
#pragma unroll
          for (int k = 0; k < S; ++k) m[k] = blk_hw_max(m[k], v[k] * rc * r[k]);
#pragma unroll
          for (int k = 0; k < S; ++k) s[k] = cslot[k] == c ? -INFINITY : s[k];   // the picked token itself
        }
        np = 0; pend = 0;
        // ---- best gain among the tokens that are not candidates
        float av[S];
#pragma unroll
        for (int k = 0; k < S; ++k) av[k] = cslot[k] >= 0 ? -INFINITY : fmaf(nlam, m[k], s[k]);
        wg_argmax(av, gout, jout);
        out_valid = true;
#ifdef KVR_STATS
        ++st_syncs;
#endif
      }
      // ---- race: the best live candidate against the best outside token
      const float gcand = lane < kBlkRows ? fmaf(nlam, gm, gs) : -INFINITY;
      const float gc = blk_row0_max(gcand);
      int uc = -1, tc = 0x7fffffff;
      if (gc > -INFINITY) {
        const unsigned long long eq = __ballot(lane < kBlkRows && gcand == gc);
        uc = __ffsll(static_cast<long long>(eq)) - 1;
        tc = __builtin_amdgcn_readlane(ctok, uc);
        if (eq & (eq - 1)) {                           // equal gains: the lowest token id wins
          for (unsigned long long rest = eq & (eq - 1); rest; rest &= rest - 1) {
            const int u2 = __ffsll(static_cast<long long>(rest)) - 1;
            const int t2 = __builtin_amdgcn_readlane(ctok, u2);
            if (t2 < tc) { tc = t2; uc = u2; }
          }
        }
      }
      if (uc >= 0 && key_beats(gc, tc, gout, jout < 0 ? 0x7fffffff : jout)) {
        // the candidate is the exact argmax over all unselected tokens
        if (tid == 0) { order_l[t] = tc; gain_l[t] = gc; }
        ++t;
        pend |= static_cast<unsigned long long>(uc) << (4 * np);
        ++np;
        if (lane == uc) gs = -INFINITY;
        if (lane < kBlkRows) gm = blk_hw_max(gm, cc[uc * 16 + lane]);
        continue;
      }
      if (np > 0) { out_valid = false; continue; }     // the outside bound is stale: refresh it first
      if (jout < 0 || !(gout > -INFINITY)) { starved = true; break; }   // nothing finite left anywhere
      if (t + 1 == b) {                                // last pick needs no row
        if (tid == 0) { order_l[t] = jout; gain_l[t] = gout; }
        ++t;
        break;
      }
      // ---- new pass.  Every token's m is up to date here.  Each wave nominates its RW best
      // unselected tokens (the winning outside token is the best of its wave) and reports the
      // best of the rest, which becomes the new outside bound.
      {
        float ts[S];
#pragma unroll
        for (int k = 0; k < S; ++k) { ts[k] = fmaf(nlam, m[k], s[k]); cslot[k] = -1; }
#pragma unroll
        for (int q = 0; q < RW; ++q) {
          float bq = ts[0];
#pragma unroll
          for (int k = 1; k < S; ++k) bq = blk_hw_max(bq, ts[k]);
          const float mx = blk_wave_max(bq);
          int cj = -1, ck = 0, cl = 0;
#pragma unroll
          for (int k = S - 1; k >= 0; --k) {
            const unsigned long long eq = __ballot(ts[k] == mx);
            if (eq) { cl = __ffsll(static_cast<long long>(eq)) - 1; ck = k; cj = base + 64 * k + cl; }
          }
          const bool ok = mx > -INFINITY && cj >= 0;
          float rsel = r[0], ssel = s[0], msel = m[0];
#pragma unroll
          for (int k = 1; k < S; ++k) {
            rsel = ck == k ? r[k] : rsel; ssel = ck == k ? s[k] : ssel; msel = ck == k ? m[k] : msel;
          }
          const float rc = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(rsel), cl));
          const float sc = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(ssel), cl));
          const float mc = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(msel), cl));
#pragma unroll
          for (int k = 0; k < S; ++k) {
            const bool mine = ok && k == ck && lane == cl;
            ts[k] = mine ? -INFINITY : ts[k];
            cslot[k] = mine ? w * RW + q : cslot[k];
          }
          if (lane == 0) {
            const int slot = w * RW + q;
            cand_l[slot] = ok ? cj : -1;
            candr[slot] = ok ? rc : 0.f;
            cs_l[slot] = ok ? sc : -INFINITY;
            cm_l[slot] = ok ? mc : 0.f;
          }
        }
        wg_argmax(ts, gout, jout);                     // barrier inside: the nominee tables are complete
      }
      ctok = lane < kBlkRows ? cand_l[lane] : -1;
      crv = lane < kBlkRows ? candr[lane] : 0.f;
      gs = lane < kBlkRows ? cs_l[lane] : -INFINITY;
      gm = lane < kBlkRows ? cm_l[lane] : 0.f;
      // ---- A operand: the sixteen nominated rows (lane: row lane%16, k-group lane/16)
      const int kg = lane >> 4;
      const int ci = cand_l[lane & 15];
      bf16x8 af[4];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        uint4 x = make_uint4(0u, 0u, 0u, 0u);
        if (ci >= 0) x = *reinterpret_cast<const uint4*>(Vh + (static_cast<long long>(ci) * a.stride_tok + ks * 32 + kg * 8) * 2);
        af[ks] = *reinterpret_cast<bf16x8*>(&x);
      }
      // ---- stream this wave's 256 tokens: coalesced loads -> padded LDS stage -> MFMA fragments.
      // 64 tokens (one slot k of every lane) at a time: their four 16x16 result tiles have token
      // column lane%16 and candidates 4*(lane/16)+0..3 in each lane; the wave's scratch turns them
      // into "token against all sixteen candidates" in the lane that owns the token (lane group
      // sub%4 owns sub-block sub of the 64).
      uint4 pre[LPC];
      auto fetch = [&](int ch) {
        // The row index is made opaque so that the unrolled pass does not keep sixty-four
        // precomputed 64-bit addresses alive across the whole selection loop.
        int row0 = base + (lane >> 4);
        asm volatile("" : "+v"(row0));
#pragma unroll
        for (int q = 0; q < LPC; ++q) {
          const int row = row0 + ch * CH + 4 * q;
          pre[q] = make_uint4(0u, 0u, 0u, 0u);
          if (row < n) pre[q] = *reinterpret_cast<const uint4*>(Vh + (static_cast<long long>(row) * a.stride_tok + (lane & 15) * 8) * 2);
        }
      };
      fetch(0);
#pragma unroll
      for (int k = 0; k < S; ++k) {
        f32x4 acc[4];
#pragma unroll
        for (int sub = 0; sub < 4; ++sub) acc[sub] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c2 = 0; c2 < 64 / CH; ++c2) {
          const int ch = k * (64 / CH) + c2;
          blk_wave_sync();                             // fragments of the previous chunk have been read
#pragma unroll
          for (int q = 0; q < LPC; ++q)
            *reinterpret_cast<uint4*>(stage + ((lane >> 4) + 4 * q) * kStgPitch + (lane & 15) * 16) = pre[q];
          blk_wave_sync();
          if (ch + 1 < TPW / CH) fetch(ch + 1);
#pragma unroll
          for (int s2 = 0; s2 < CH / 16; ++s2) {
            const char* fp = stage + (s2 * 16 + (lane & 15)) * kStgPitch + kg * 16;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
              acc[c2 * (CH / 16) + s2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                  af[ks], *reinterpret_cast<const bf16x8*>(fp + ks * 64), acc[c2 * (CH / 16) + s2], 0, 0, 0);
          }
        }
#pragma unroll
        for (int sub = 0; sub < 4; ++sub) {
          blk_wave_sync();
          *reinterpret_cast<f32x4*>(scratch + (lane & 15) * kScrPitch + 4 * kg) = acc[sub];
          blk_wave_sync();
          if (kg == sub) {
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4) {
              const f32x4 vv = *reinterpret_cast<const f32x4*>(scratch + (lane & 15) * kScrPitch + 4 * c4);
              vals[k][4 * c4 + 0] = vv[0]; vals[k][4 * c4 + 1] = vv[1];
              vals[k][4 * c4 + 2] = vv[2]; vals[k][4 * c4 + 3] = vv[3];
            }
          }
        }
      }
      // ---- candidate-to-candidate cosines, written by the lanes that own the candidate tokens
#pragma unroll
      for (int k = 0; k < S; ++k) {
        if (cslot[k] >= 0) {
#pragma unroll
          for (int x = 0; x < kBlkRows; ++x) cc[x * 16 + cslot[k]] = vals[k][x] * candr[x] * r[k];
        }
      }
      __syncthreads();
      // gout / jout from the nomination are exact for the new outside set
#ifdef KVR_STATS
      ++st_blocks;
#endif
    }
#ifdef KVR_STATS
    __syncthreads();
    if (tid == 0 && b >= 4) { gain_l[b - 1] = st_blocks; gain_l[b - 2] = st_syncs; }
#endif
  }

  // ---- sort(S): flag the picked tokens, ascending indices by prefix counts
  __syncthreads();
#pragma unroll
  for (int k = 0; k < S; ++k) flag[base + 64 * k + lane] = 0;
  __syncthreads();
  for (int u = tid; u < t; u += NT) flag[order_l[u]] = 1;
  __syncthreads();
  if (starved) {
    // Non-finite input only: fill the remaining picks with the lowest unpicked tokens.
    if (tid == 0) {
      int j = 0;
      for (int u = t; u < b; ++u) {
        while (j < n - 1 && flag[j]) ++j;
        order_l[u] = j; gain_l[u] = -INFINITY; flag[j] = 1;
      }
    }
    __syncthreads();
  }
  {
    unsigned long long sel[S];
    int cnt = 0;
#pragma unroll
    for (int k = 0; k < S; ++k) {
      sel[k] = __ballot(tok[k] < n && flag[tok[k]] != 0);
      cnt += __popcll(sel[k]);
    }
    if (lane == 0) wcount[w] = cnt;
    __syncthreads();
    int off = 0;
    for (int u = 0; u < w; ++u) off += wcount[u];
#pragma unroll
    for (int k = 0; k < S; ++k) {
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
  auto go = [&](auto kern, int threads, int smem) -> hipError_t {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, dim3(threads), smem, st, a);
    return hipGetLastError();
  };
  if (lay.n <= 512) return go(&select_blocked_kernel<2, 4>, 128, BlkCfg<2, 4>::kSmemBytes);
  if (lay.n <= 1024) return go(&select_blocked_kernel<4, 4>, 256, BlkCfg<4, 4>::kSmemBytes);
  if (lay.n <= 2048) return go(&select_blocked_kernel<8, 4>, 512, BlkCfg<8, 4>::kSmemBytes);
  return go(&select_blocked_kernel<8, 8>, 512, BlkCfg<8, 8>::kSmemBytes);
}

}  // namespace kvr
