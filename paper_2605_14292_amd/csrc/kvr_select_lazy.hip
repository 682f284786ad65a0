// Greedy selection (paper Sec. 4.1, Algorithm 1) for heads with 256 < n <= 4096
// tokens and b <= 128: bf16 rows, followed by the compaction of the kept rows, or
// fp32 rows (selection only).
//
// Exact greedy with lazily refreshed penalties.  Algorithm 1 reads one cosine row per
// pick, i.e. all of V once per pick.  The running maximum m_i of Eq. 2 only grows, so a
// gain computed from an out-of-date m_i is an upper bound of the true one, and a token
// whose upper bound is low needs no update until the bound matters.  Every token is either
// "fresh" (its m covers all picks made so far) or "stale" (its m covers an earlier prefix of
// them).  An epoch:
//   1. the P = 128 best fresh unselected tokens form the pool (each wave contributes its
//      best P/W, found by a bitwise threshold search on the gains); the best gain of any
//      token outside the pool, fresh or stale, is the bound of the epoch;
//   2. the pool's rows are gathered into LDS and their P x P cosine triangle is computed
//      on bf16 MFMA (32x32x16, fp32 accumulate), then written over the rows;
//   3. one wave runs Algorithm 1 inside the pool (DPP argmax, one LDS row read per pick)
//      for as long as the pool's best (gain, lower index) beats the bound -- every outside
//      gain is at most its bound, so such a pick is the exact argmax of Eq. 2 over all
//      unselected tokens;
//   4. the rows of the epoch's picks join the rows of all earlier picks in LDS, and every
//      wave brings the quarter or so of its outside tokens with the highest bounds up to
//      date against ALL picks so far (16-row MFMA operands, 16x16x32): these are fresh for
//      the next epoch, the others keep their bound and go stale.  The first epoch's pass
//      covers every token (it also takes the inverse norms of Eq. 1).
// How many tokens step 4 refreshes is a matter of speed only: a stale token can only end an
// epoch early (it then carries the bound and is among the refreshed ones), never change a
// pick.  On the benchmark inputs an epoch serves 5-50 picks and a head reads its rows about
// 2.7 times (once per epoch with a full pass).  Nothing is approximated.
//
// F32 rows (the flat-signature mode's mean rows, fp32 caches) run the same epochs with the fp32 MFMAs (32x32x2 for
// the pool's Gram, 16x16x4 for the passes); their 512-byte rows leave no room for a stage, so the rows of a pass are
// loaded straight into the operand layout.
//
// Layout: one workgroup per head, W wave64s, token j = 64*S*w + 64*k + lane in
// wave w, lane `lane`, slot k; score, m and inverse norm of a token stay in its
// lane's registers for the whole event.
#define KVR_BOUNDS_FILE 1   // ids 1xx of the debug build's bounds checks (kvr_bounds.hpp)
#include "kvr_dense_common.hpp"
#include "kvr_kernels.hpp"
#include <type_traits>

namespace kvr {

typedef __attribute__((ext_vector_type(4))) float f32x4;

#ifndef KVR_POOL_WIDE
#define KVR_POOL_WIDE 128
#endif
constexpr int kLzPoolWide = KVR_POOL_WIDE;   // pool of the configurations with one workgroup per CU
constexpr int kLzMaxB = 128;        // largest budget: the rows of all picks stay in LDS
constexpr int kLzMaxPend = 64;      // picks per epoch (the chain logs pick u in lane u)
constexpr int kLzPitch = 272;       // bytes per pool row (256 + 16): conflict-free 32x32x16 operand reads
// Rows read as 16x16x32 operands (the picks' rows, the staged rows of a pass) are kept as two planes of half rows:
// 16-byte piece p of a row sits in plane p >> 3 at row * 144 + (p & 7) * 16, and the planes start a multiple of
// 256 bytes apart.  Lane (row c, k-group kg) of an operand reads piece (kg >> 1) + 2 * ks + 8 * (kg & 1) in step
// ks (both operands use the same order, so the sum over k is the row product).  Lanes l and l + 16 then hit the same
// banks, which is what a 128-bit LDS read needs to run at full rate: measured 221 B/clk against 123 B/clk for
// whole rows 272 bytes apart, where the four k-groups start four banks apart.  Row writes (16 lanes, one row)
// run at the write rate of whole rows.
constexpr int kLzHalf = 144;        // bytes between the half rows of a plane (128 + 16)
constexpr int kLzStagePlane = 16 * kLzHalf;      // 2304 = 9 * 256
constexpr int kLzPickPlane = 128 * kLzHalf;      // 18432 = 72 * 256
// fp32 rows: 32 pieces, pool rows 528 bytes apart, half rows of 16 pieces 272 bytes apart; lane (c, kg) of a
// 16x16x4 operand reads piece 4 j + kg (floats 16 j + 4 kg .. + 3) in step j, kept in plane kg & 1 at slot (kg >> 1) + 2 j
constexpr int kLzPitchF = 528;
constexpr int kLzHalfF = 272;
constexpr int kLzPickPlaneF = 128 * kLzHalfF;    // 34816 = 136 * 256
constexpr int kLzSelBits = 16;      // leading bits of a gain's ordered key used to choose the pool
constexpr int kLzChunk = 16;        // rows staged per step and wave in the refresh pass

struct LazyArgs {
  const char* K; const char* V; const float* s_in;
  int32_t* idx_sorted; int32_t* pick_order; float* pick_gain;
  char* K_out; char* V_out;
  long long stride_head, stride_tok;   // elements
  int n, b;
  float lambda, eps;
  const int32_t* b_h;                  // per-head budgets <= b (output rows stay b apart), or null
  int only_marked;                     // process only heads whose idx_sorted[h*b] is -1 (an earlier kernel has finished the others)
};

// P: pool size, a multiple of 64.  192 was measured where a head has the CU to itself (n > 1024): an epoch less per head,
// paid back by the larger triangle and the three-slot race, so every configuration runs 128.
template <int W, int S, int P, bool F32 = false> struct LazyCfg {
  static constexpr int TPW = 64 * S;
  // 16-row sub-blocks of the refresh list that a wave has in flight (one "group"): four, or two of fp32 rows
  static constexpr int GSUB = F32 ? 2 : 4;
  static constexpr int GR = 16 * GSUB;
  // per wave, during the pass: row stage | 256-float exchange | 64 squared norms | TPW inverse norms (first pass)
  // (fp32 rows: the inverse norms only)
  static constexpr int kWaveArea = F32 ? TPW * 4 : 2 * kLzStagePlane + 1024 + 256 + TPW * 4;
  static constexpr int kTriBytes = 8 * (P / 4) * (P / 4 + 1) * 4;    // rows padded to multiples of four floats
  static constexpr int kRowBytes = P * (F32 ? kLzPitchF : kLzPitch);
  static constexpr int kMax2 = kTriBytes > kRowBytes ? kTriBytes : kRowBytes;
  static constexpr int kUnion = ((W * kWaveArea > kMax2 ? W * kWaveArea : kMax2) + 15) & ~15;
  // floats: slots 64 | shared 16 | wcount 16 | pool_tok,r,s,m,picked 5*128 | pend 64 |
  //         order,gain,pick_r 3*128 ; then per wave TPW list entries / results (at the end the sorted
  //         indices) ; then the rows of the picks ; then the union area (pool rows -> triangle -> pass
  //         areas -> pick flags of the read-out)
  static constexpr int kFixedFloats = 96 + 5 * P + 64 + 3 * kLzMaxB;
  static constexpr int kListFloats = W * (TPW + 64);   // one group of padding past a full list
  static constexpr int kPickBytes = 2 * (F32 ? kLzPickPlaneF : kLzPickPlane);
  static_assert(64 * S * W * 4 <= kUnion, "the pick flags of the read-out fit the union area");
  // Where two workgroups share a CU (W <= 4) the triangle is written over the pool's rows and the rows of an epoch's
  // picks are read from memory again; a workgroup that has the CU to itself keeps the rows and copies them inside LDS.
  static constexpr bool kAlias = W <= 4 || F32;
  static constexpr int kKeepBytes = kAlias ? 0 : kRowBytes;
  static constexpr int smem_bytes() { return (kFixedFloats + kListFloats) * 4 + kPickBytes + kKeepBytes + kUnion; }
};

// The pool's cosine triangle keeps row i (columns 0..i) in (i + 4) & ~3 floats, so that four neighbouring columns of a
// row are one aligned 16-byte store: row i = 4g + r starts at float 4 (g + 1)(2g + r).  Element (i, j), j <= i, sits
// at start(i) + j; start(i) + j >= start(j) + i holds for i > j as in the packed triangle, so the race reads
// max(start(i) + j, start(j) + i) without knowing which index is the larger.
__device__ __forceinline__ int lz_row_start(int i) { return 4 * ((i >> 2) + 1) * (2 * (i >> 2) + (i & 3)); }

// Writes one 32x32 tile of the pool's Gram matrix as cosines into the triangle.  acc comes from the MFMA with the
// column block J as operand A and the row block I as operand B: lane (row = lane & 31, hf = lane >> 5) holds
// columns 8R + 4hf .. + 3 of its row in acc[4R .. 4R+3].  The diagonal holds +inf (the row of a pick retires it);
// what a store writes past the diagonal stays inside the row's padding and is never read.
__device__ __forceinline__ void lz_write_cos_tile(float* tri, const float* rinv, const f32x16& acc, int I, int J, int lane) {
  const int hf = lane >> 5;
  const int row = I * 32 + (lane & 31);
  const float rrow = rinv[row];
  float4 rc[4];                                       // the columns' inverse norms, all requested before the first use
#pragma unroll
  for (int R = 0; R < 4; ++R) rc[R] = *reinterpret_cast<const float4*>(rinv + J * 32 + 8 * R + 4 * hf);
  float* dst = tri + lz_row_start(row) + J * 32 + 4 * hf;
  if (I != J) {                                       // two code paths: no per-element predicate off the diagonal
#pragma unroll
    for (int R = 0; R < 4; ++R)
      *reinterpret_cast<float4*>(dst + 8 * R) = make_float4(acc[4 * R] * rrow * rc[R].x, acc[4 * R + 1] * rrow * rc[R].y,
                                                            acc[4 * R + 2] * rrow * rc[R].z, acc[4 * R + 3] * rrow * rc[R].w);
  } else {
#pragma unroll
    for (int R = 0; R < 4; ++R) {
      const int col = J * 32 + 8 * R + 4 * hf;
      float4 v = make_float4(acc[4 * R] * rrow * rc[R].x, acc[4 * R + 1] * rrow * rc[R].y,
                             acc[4 * R + 2] * rrow * rc[R].z, acc[4 * R + 3] * rrow * rc[R].w);
      if (col == row) v.x = INFINITY;
      if (col + 1 == row) v.y = INFINITY;
      if (col + 2 == row) v.z = INFINITY;
      if (col + 3 == row) v.w = INFINITY;
      if (col <= row) *reinterpret_cast<float4*>(dst + 8 * R) = v;
    }
  }
}

// BUD: per-head budgets are read from a.b_h.
template <int W, int S, int P, bool BUD, bool F32 = false>
__global__ __launch_bounds__(64 * W, (W <= 4 ? 2 : 1)) void select_lazy_kernel(LazyArgs a) {
  using Cfg = LazyCfg<W, S, P, F32>;
  constexpr int GSUB = Cfg::GSUB;                  // sub-blocks per group of the pass
  constexpr int GR = Cfg::GR;                      // rows per group
  constexpr int LPR = F32 ? 32 : 16;               // 16-byte pieces (and lanes of a gather) per row
  constexpr int kPitch = F32 ? kLzPitchF : kLzPitch;
  constexpr int kHalf = F32 ? kLzHalfF : kLzHalf;
  constexpr int kPickPlane = F32 ? kLzPickPlaneF : kLzPickPlane;
  constexpr int TPW = 64 * S;
  constexpr int NT = 64 * W;
  constexpr int Q = P / W;                   // pool members contributed per wave
  constexpr int CH = kLzChunk;
  constexpr int LPC = F32 ? 8 : CH / 4;            // loads per lane and sub-block
  constexpr int KR = W <= 4 ? TPW / 2 : TPW / 4;   // tokens a wave aims to refresh per pass (measured: c5 / c4)
  constexpr int NB = P / 32;                       // 32-token blocks of the pool
  constexpr int NTRI = NB * (NB + 1) / 2;          // lower-triangular 32x32 tiles of its cosine matrix
  constexpr int NTILE = (NTRI + W - 1) / W;        // ... per wave
  constexpr int NQ = P / 64;                       // pool slots per lane in the race
  static_assert(S <= 8 && Q <= 64, "token state lives in registers; a wave's pool share fits a ballot");
  extern __shared__ __align__(16) float smem[];
  float* slot_gain = smem;                                       // [2][16]
  int32_t* slot_idx = reinterpret_cast<int32_t*>(smem + 32);     // [2][16]
  int32_t* shared_i = reinterpret_cast<int32_t*>(smem + 64);     // [16] np, t, stop reason
  int32_t* wcount = reinterpret_cast<int32_t*>(smem + 80);       // [16]
  int32_t* pool_tok = reinterpret_cast<int32_t*>(smem + 96);     // [P] token of the member, -1 = none
  float* pool_r = smem + 96 + P;
  float* pool_s = smem + 96 + 2 * P;
  float* pool_m = smem + 96 + 3 * P;
  int32_t* pool_picked = reinterpret_cast<int32_t*>(smem + 96 + 4 * P);
  int32_t* pend_l = reinterpret_cast<int32_t*>(smem + 96 + 5 * P);        // [64] pool slots picked this epoch
  int32_t* order_l = reinterpret_cast<int32_t*>(smem + 96 + 5 * P + 64);
  float* gain_l = smem + 96 + 5 * P + 64 + kLzMaxB;
  float* pick_r = smem + 96 + 5 * P + 64 + 2 * kLzMaxB;                   // inverse norms of the picks, 0 past the last
  float* lr_all = smem + Cfg::kFixedFloats;                                     // [W][TPW] refresh lists / results
  int32_t* idxs_l = reinterpret_cast<int32_t*>(lr_all);                         // [128] sorted indices (the lists are dead by then)
  char* pk = reinterpret_cast<char*>(smem + Cfg::kFixedFloats + Cfg::kListFloats);   // [2 planes][128][144 B] rows of the picks
  char* uni = pk + Cfg::kPickBytes + Cfg::kKeepBytes;
  char* prow = Cfg::kAlias ? uni : pk + Cfg::kPickBytes;        // [P][272 B] pool rows (gather, Gram) ...
  float* tri = reinterpret_cast<float*>(uni);                    // ... then the packed P x P cosine triangle (race) ...
  // ... then the per-wave areas of the pass ...
  int32_t* flag = reinterpret_cast<int32_t*>(uni);               // ... and at the end [n padded] pick flags for the ascending read-out

  const int h = blockIdx.x;
  if (a.only_marked && a.idx_sorted[static_cast<long long>(h) * a.b] != -1) return;   // (uniform: a scalar load)
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = a.n;
  // the head's own budget: its picks are the first b picks of a run for a.b (the rows of the
  // outputs per head), so the epochs stop there
  const int b = BUD ? min(max(a.b_h[blockIdx.x], 0), a.b) : a.b;      // a scalar load: the index is uniform
  const long long head_off = h * a.stride_head * (F32 ? 4 : 2);   // bytes
  const char* Vh = a.V + head_off;
  const uint32_t pitch_b = static_cast<uint32_t>(a.stride_tok) * (F32 ? 4u : 2u);   // bytes between tokens: a head spans less than 4 GiB (checked by the host)
  const int base = w * TPW;
  char* stage = uni + w * Cfg::kWaveArea;
  float* scratch = reinterpret_cast<float*>(stage + 2 * kLzStagePlane);
  float* norm_x = scratch + 256;                                 // [64] squared norms of the wave's current 64 rows
  float* lr2 = F32 ? reinterpret_cast<float*>(stage) : norm_x + 64;   // [TPW] inverse norms found in the first pass
  float* lrw = lr_all + w * (TPW + 64);                                 // [TPW] list of tokens to refresh, then their raw maxima
  int32_t* lrw_i = reinterpret_cast<int32_t*>(lrw);
  const unsigned long long below = (1ull << lane) - 1ull;

  // where 16-byte piece p of a pick's row goes in the rows of the picks (without the row's offset)
  auto pick_piece = [](int p) -> int {
    if constexpr (F32) return (p & 1) * kLzPickPlaneF + (((p >> 1) & 1) + 2 * (p >> 2)) * 16;
    else return (p >> 3) * kLzPickPlane + (p & 7) * 16;
  };
  float s[S], m[S], r[S];
  int pslot[S];                  // >= 0: pool slot of this token in the current epoch; <= -2: position -2 - p in the wave's refresh list; -1: neither
  uint32_t fresh = 0xffffffffu;  // bit k: m[k] covers every pick made so far
  auto tok_of = [&](int k) -> int { return base + 64 * k + lane; };
#pragma unroll
  for (int k = 0; k < S; ++k) {
    s[k] = tok_of(k) < n ? a.s_in[static_cast<long long>(h) * n + tok_of(k)] : -INFINITY;
    m[k] = 0.f;
    r[k] = 0.f;
    pslot[k] = -1;
  }
  // rows of the picks: zero until written (a partly filled 16-row operand multiplies zeros)
  for (int u = tid; u < Cfg::kPickBytes / 16; u += NT) reinterpret_cast<uint4*>(pk)[u] = make_uint4(0u, 0u, 0u, 0u);
  if (tid < kLzMaxB) pick_r[tid] = 0.f;
  const float nlam = -a.lambda;
  int par = 0;
  int t = 0;
  int kbits = kLzSelBits;        // leading key bits the pool choice looks at (uniform)
  uint32_t tau_prev = 0;         // the wave's pool threshold of the last epoch (0: none)
  bool starved = false;
  float delta = -1.f;            // refresh threshold: this far below the wave's best outside gain (< 0: not yet known)

  // workgroup argmax over av (per slot); ibest carries bit 30 when the winner's slot has a stale m
  auto wg_argmax = [&](const float (&av)[S], float& gbest, int& ibest, float& amax_w) {
    float best = av[0];
#pragma unroll
    for (int k = 1; k < S; ++k) best = hw_max(best, av[k]);
    amax_w = wave_max_uniform(best);
    int i_w = -1;
#pragma unroll
    for (int k = S - 1; k >= 0; --k) {
      const unsigned long long eq = __ballot(av[k] == amax_w);
      if (eq) {
        const int l0 = __ffsll(static_cast<long long>(eq)) - 1;
        const int fr = (__builtin_amdgcn_readlane(static_cast<int>(fresh), l0) >> k) & 1;
        i_w = (base + 64 * k + l0) | (fr ? 0 : (1 << 30));
      }
    }
    if (lane == 0) { slot_gain[par * 16 + w] = amax_w; slot_idx[par * 16 + w] = i_w; }
    lds_barrier();
    const float g = lane < W ? slot_gain[par * 16 + lane] : -INFINITY;
    const int ii = lane < W ? slot_idx[par * 16 + lane] : -1;
    par ^= 1;
    gbest = wave_max_uniform(g);
    const unsigned long long eqw = __ballot(lane < W && g == gbest);
    ibest = eqw ? __builtin_amdgcn_readlane(ii, __ffsll(static_cast<long long>(eqw)) - 1) : -1;
  };

  if (b == 1) {
    float gmax, dummy; int i;
    wg_argmax(s, gmax, i, dummy);
    if (!(gmax > -INFINITY)) starved = true;
    else { if (tid == 0) { order_l[0] = i & 0x3fffffff; gain_l[0] = gmax; } t = 1; }
  } else {
    bool have_r = false;
    // Exact candidate reduction (as in the kernels for short heads): while fewer than b tokens are
    // selected one of the b best-scored is free and gains at least s_(b) - lambda, and a token gains
    // at most its score, so a token with s_j < s_(b) - lambda never wins Eq. 3.  Such tokens get the
    // score -inf: they are never a pool member, a pick or in a refresh list, and their rows are never
    // read.  Nothing can go when the finite scores spread by less than lambda (then s_(b) - lambda is
    // below all of them); one workgroup-wide min/max settles that before the search for s_(b).
    {
      float hi = -INFINITY, lo = INFINITY;
#pragma unroll
      for (int k = 0; k < S; ++k) {
        if (s[k] > -INFINITY && s[k] < INFINITY) { hi = hw_max(hi, s[k]); lo = fminf(lo, s[k]); }
      }
      hi = wave_max_uniform(hi);
      lo = -wave_max_uniform(-lo);
      if (lane == 0) { slot_gain[par * 16 + w] = hi; slot_gain[32 + w] = lo; }   // (smem 32.. is slot_idx: free until the first argmax)
      lds_barrier();
      float ghi = -INFINITY, glo = INFINITY;
#pragma unroll
      for (int u = 0; u < W; ++u) { ghi = hw_max(ghi, slot_gain[par * 16 + u]); glo = fminf(glo, slot_gain[32 + u]); }
      par ^= 1;
      const bool wide = __builtin_amdgcn_readfirstlane(ghi - glo > a.lambda ? 1 : 0) != 0;   // false also when no score is finite
      lds_barrier();                                 // the min/max slots are rewritten below
      if (wide) {
        uint32_t key[S];
#pragma unroll
        for (int k = 0; k < S; ++k) key[k] = tok_of(k) < n ? ordered_key(s[k] + 0.0f) : 0u;
        uint32_t T = 0;                              // s_(b) from the leading 16 bits: at most s_(b), the bound only loosens
        for (int bit = 31; bit >= 16; --bit) {
          const uint32_t cand = T | (1u << bit);
          int c = 0;
#pragma unroll
          for (int k = 0; k < S; ++k) c += __popcll(__ballot(key[k] >= cand));
          if (lane == 0) slot_idx[par * 16 + w] = c;
          lds_barrier();
          int tot = 0;
#pragma unroll
          for (int u = 0; u < W; ++u) tot += slot_idx[par * 16 + u];
          par ^= 1;
          if (tot >= b) T = cand;
        }
        const float sb = key_to_float(T);
        const float thr = sb - a.lambda * 1.00001f - 1e-5f * fabsf(sb);   // fp32 cosines may exceed 1 by a few ulp
#pragma unroll
        for (int k = 0; k < S; ++k)
          if (s[k] < thr) s[k] = -INFINITY;          // (a NaN threshold or score leaves the token in)
      }
    }
    auto sum_sq = [](const uint4& x) -> float {
      float ss = 0.f;
      if constexpr (F32) {
        const float e[4] = {__uint_as_float(x.x), __uint_as_float(x.y), __uint_as_float(x.z), __uint_as_float(x.w)};
#pragma unroll
        for (int q = 0; q < 4; ++q) ss = fmaf(e[q], e[q], ss);
      } else {
        const float e[8] = {bf16_lo(x.x), bf16_hi(x.x), bf16_lo(x.y), bf16_hi(x.y),
                            bf16_lo(x.z), bf16_hi(x.z), bf16_lo(x.w), bf16_hi(x.w)};
#pragma unroll
        for (int q = 0; q < 8; ++q) ss = fmaf(e[q], e[q], ss);
      }
      // the 16 lanes of a row hold its 16-byte chunks and form one DPP row: its last lane ends up with the total
      KVR_DPP_ADD(ss, 0x111, 0xf) KVR_DPP_ADD(ss, 0x112, 0xf) KVR_DPP_ADD(ss, 0x114, 0xf) KVR_DPP_ADD(ss, 0x118, 0xf)
      return ss;
    };

    int idle = 0;                                    // epochs in a row without a pick
    while (t < b) {
      // ================= 1. pool = the best Q fresh unselected tokens of every wave =================
      float g[S];
      uint32_t key[S];
      // Keys are cut to their leading kbits bits: the pool only has to be a good guess (the
      // race against the outside bound keeps the picks exact), and the search is shorter.
      // When the cut keys cannot tell a wave's best tokens apart the best one may be left outside
      // and the epoch ends without a pick; it is then repeated on the full keys, where the best
      // fresh token of every wave is a member (equal values join in token order).
      uint32_t ekey[S];                              // key + 1 of a fresh token, 0 of a stale one (never a member)
#pragma unroll
      for (int k = 0; k < S; ++k) {
        g[k] = fmaf(nlam, m[k], s[k]);
        key[k] = ordered_key(g[k]) >> (32 - kbits);
        const uint32_t k1 = key[k] + 1u;             // (wraps to 0 for an all-ones key, which only a NaN with full keys has)
        ekey[k] = ((fresh >> k) & 1u) ? k1 : 0u;
      }
      uint32_t tau = 0;                              // largest value with at least Q fresh keys >= it
      auto at_least_q = [&](uint32_t x) -> bool {
        int c = 0;
#pragma unroll
        for (int k = 0; k < S; ++k) c += __popcll(__ballot(ekey[k] >= x));
        return c >= Q;
      };
      if (kbits == kLzSelBits && tau_prev != 0) {
        // the value moves little from one epoch to the next: bracket it from the last one with doubling
        // steps, then bisect (a third of the counts of the bit-wise search on the benchmark inputs)
        constexpr uint32_t kTop = (1u << kLzSelBits) + 1u;   // no key + 1 reaches this
        uint32_t lo, hi;                             // at_least_q(lo), !at_least_q(hi)
        if (at_least_q(tau_prev)) {
          lo = tau_prev;
          for (uint32_t d = 1;; d <<= 1) {
            hi = lo + d;
            if (hi >= kTop) { hi = kTop; break; }
            if (!at_least_q(hi)) break;
            lo = hi;
          }
        } else {
          hi = tau_prev;
          for (uint32_t d = 1;; d <<= 1) {
            lo = hi > d ? hi - d : 0u;               // (every key is >= 0)
            if (lo == 0u || at_least_q(lo)) break;
            hi = lo;
          }
        }
        while (hi - lo > 1u) {
          const uint32_t mid = (lo + hi) >> 1;
          if (at_least_q(mid)) lo = mid; else hi = mid;
        }
        tau = lo;
      } else {
        for (int bit = kbits; bit >= 0; --bit) {
          if (bit == 32) continue;                   // keys + 1 of full-width keys are searched over 32 bits
          const uint32_t cand = tau | (1u << bit);
          if (at_least_q(cand)) tau = cand;
        }
      }
      tau_prev = tau;
      if (tau == 0) tau = 1;                         // fewer than Q fresh tokens: all of them join
      int taken = 0;                                 // members with key > tau come first, ties in token order
#pragma unroll
      for (int k = 0; k < S; ++k) taken += __popcll(__ballot(ekey[k] > tau));
      int need_eq = Q - taken;                       // how many of the key == tau tokens join
      int rank_base = 0;
      float go[S];                                   // gains (bounds) of the tokens left outside
#pragma unroll
      for (int k = 0; k < S; ++k) {
        const bool above = ekey[k] > tau, equal = ekey[k] == tau;
        const unsigned long long eqm = __ballot(equal);
        const int eq_before = __popcll(eqm & below);
        const bool in = above || (equal && eq_before < need_eq);
        const unsigned long long inm = __ballot(in);
        const int slot = w * Q + kvr_ix_if(in, rank_base + __popcll(inm & below), Q, 101);   // 101: a member's place in the wave's share
        pslot[k] = in ? slot : -1;
        if (in) {
          pool_tok[slot] = tok_of(k) < n ? tok_of(k) : -1;
          pool_r[slot] = r[k];
          pool_s[slot] = s[k];
          pool_m[slot] = m[k];
          pool_picked[slot] = 0;
        }
        go[k] = in ? -INFINITY : g[k];
        rank_base += __popcll(inm);
        const int eq_in = __popcll(eqm);
        need_eq -= eq_in < need_eq ? eq_in : need_eq;
      }
      if (lane >= rank_base && lane < Q) {           // fewer fresh tokens than the wave's share: empty slots
        const int slot = w * Q + lane;
        pool_tok[slot] = -1; pool_r[slot] = 0.f; pool_s[slot] = -INFINITY; pool_m[slot] = 0.f; pool_picked[slot] = 0;
      }
      float gout, gmax_w; int jout_f;
      wg_argmax(go, gout, jout_f, gmax_w);           // barrier inside: the pool tables are complete
      const int jout = jout_f < 0 ? -1 : (jout_f & 0x3fffffff);
      const bool jout_stale = jout_f >= 0 && (jout_f & (1 << 30));

      // the pool's rows are requested now; the refresh list is built while they are on their way
      // (all row loads of a thread are issued before the first one is stored: with the loads
      // and stores interleaved, every load waits for the one before it)
      constexpr int kGat = P * LPR / NT;         // rows per thread
      constexpr int kGatRows = NT / LPR;         // rows per round
      const int gat_row = tid / LPR, gat_piece = tid % LPR;
      uint4 x[kGat];
#pragma unroll
      for (int k = 0; k < kGat; ++k) {
        const int tk = pool_tok[k * kGatRows + gat_row];
        const int tkc = kvr_ix(tk < 0 ? 0 : tk, n, 103);   // an empty slot reads row 0 and stores zeros (103: token of a pool member)
        x[k] = *reinterpret_cast<const uint4*>(Vh + (static_cast<uint32_t>(tkc) * pitch_b + gat_piece * 16u));
      }
      // ---- the wave's refresh list for this epoch's pass: outside tokens whose bound lies within
      // delta of the wave's best one (all of them in the first pass).  delta is steered so that about
      // KR tokens qualify: a few bisection steps around the previous epoch's value.
      int cnt_r = 0;
      {
        auto count_ge = [&](float thr) -> int {
          int c = 0;
#pragma unroll
          for (int k = 0; k < S; ++k) c += __popcll(__ballot(go[k] >= thr && go[k] > -INFINITY));
          return c;
        };
        float thr_r = -INFINITY;                     // first pass: every outside token that can still be picked
        if (have_r && gmax_w > -INFINITY) {
          float lo_d, hi_d;
          int steps;
          if (delta < 0.f) {
            float gmin = INFINITY;
#pragma unroll
            for (int k = 0; k < S; ++k) if (go[k] > -INFINITY) gmin = fminf(gmin, go[k]);
            gmin = -wave_max_uniform(-gmin);
            lo_d = 0.f; hi_d = gmax_w - gmin; steps = 8;
          } else {
            lo_d = 0.5f * delta; hi_d = 2.0f * delta; steps = 3;
          }
          int c_lo = 1;                              // tokens within lo_d of the best (not counted for the first guess)
          bool above = false;                        // some count exceeded KR: more than KR tokens lie within hi_d
          for (int it = 0; it < steps; ++it) {       // count(delta) grows with delta
            const float mid = 0.5f * (lo_d + hi_d);
            const int c = count_ge(gmax_w - mid);
            if (c > KR) { hi_d = mid; above = true; } else { lo_d = mid; c_lo = c; }
          }
          // the lower end of the bracket: at most KR tokens (whole 64-row groups are what the pass costs), always
          // including the wave's best outside token, the one that can carry the epoch's bound
          delta = lo_d;
          thr_r = gmax_w - delta;
          if (4 * c_lo < KR) {
            // The guess has collapsed or run away: a full search next time.  When the bracket could not split a
            // crowd of bounds (scores within a hair of each other, not yet penalised: a handful of tokens inside
            // lo_d, more than KR inside hi_d) and the last epoch ended without a pick, the whole crowd is
            // refreshed, or the epochs would crawl through it a few tokens at a time (the list holds every token
            // of the wave).  While the epochs do pick, the short list is the cheaper one.
            if (above && idle > 0) thr_r = gmax_w - hi_d;
            delta = -1.f;
          }
        }
        int off = 0;
#pragma unroll
        for (int k = 0; k < S; ++k) {
          const bool mem = go[k] >= thr_r && go[k] > -INFINITY;     // (go is -inf for pool members and dead tokens)
          const unsigned long long mm = __ballot(mem);
          if (mem) {
            const int pos = kvr_ix(off + __popcll(mm & below), TPW, 102);   // 102: position in the refresh list
            lrw_i[pos] = tok_of(k);
            pslot[k] = -2 - pos;
          }
          off += __popcll(mm);
        }
        cnt_r = off;
        // pad to a multiple of 64 with a valid row (its results are never read)
        // (at least one group: the first group's rows are requested whether or not the list has entries)
        const int padded = (cnt_r == 0 ? GR : (cnt_r + GR - 1) & ~(GR - 1)) + GR;     // ... and one group more: the pass requests a group ahead
        for (int u = cnt_r + lane; u < padded; u += 64) lrw_i[u] = min(base, n - 1);
      }
      // The rows of the list's first 64 entries are requested here and travel while the pool's triangle is
      // computed and raced; further groups follow inside the pass, one group ahead.
      uint4 pre[GSUB][LPC];
      auto fetch = [&](int gi, int sub) {
        if constexpr (F32) {
          // straight into the operand layout of the 16x16x4 MFMA: lane (c, kg) holds pieces kg, kg + 4, .. of row c
          const int row = kvr_ix(lrw_i[gi * GR + sub * CH + (lane & 15)], n, 104);   // 104: token of a list entry
          const uint32_t o = static_cast<uint32_t>(row) * pitch_b + (lane >> 4) * 16u;
#pragma unroll
          for (int q = 0; q < LPC; ++q) pre[sub][q] = *reinterpret_cast<const uint4*>(Vh + (o + q * 64u));
        } else {
#pragma unroll
          for (int q = 0; q < LPC; ++q) {
            const int row = kvr_ix(lrw_i[gi * GR + sub * CH + (lane >> 4) + 4 * q], n, 104);
            pre[sub][q] = *reinterpret_cast<const uint4*>(Vh + (static_cast<uint32_t>(row) * pitch_b + (lane & 15) * 16u));
          }
        }
      };
      wave_lds_sync();                               // the list was written by other lanes of this wave
#pragma unroll
      for (int sub = 0; sub < GSUB; ++sub) fetch(0, sub);   // (no branch around them: the wait counts of what follows stay exact)

      // ================= 2. pool rows -> LDS, cosine triangle on MFMA (written over the rows) =================
      {
#pragma unroll
        for (int k = 0; k < kGat; ++k) {
          const int slot = k * kGatRows + gat_row;
          if (pool_tok[slot] < 0) x[k] = make_uint4(0u, 0u, 0u, 0u);   // (only here: a select between the loads would make each wait for the one before)
          *reinterpret_cast<uint4*>(prow + slot * kPitch + gat_piece * 16) = x[k];
        }
        if (!have_r) {
#pragma unroll
          for (int k = 0; k < kGat; ++k) {
            const int slot = k * kGatRows + gat_row;
            float ss = sum_sq(x[k]);
            if constexpr (F32) ss += __shfl_up(ss, 16);   // a row spans two 16-lane DPP rows
            if (gat_piece == LPR - 1) pool_r[slot] = pool_tok[slot] < 0 ? 0.f : 1.0f / (sqrtf(ss) + a.eps);
          }
        }
      }
      lds_barrier();
      {
        const int hf = lane >> 5;
        f32x16 acc[NTILE];
#pragma unroll
        for (int q = 0; q < NTILE; ++q) {
          const int tile = w + q * W;                  // lower-triangular 32x32 tiles of the P x P matrix
          acc[q] = f32x16{0};
          if (tile < NTRI) {
            int I = 0;
            while ((I + 1) * (I + 2) / 2 <= tile) ++I;
            const int J = tile - I * (I + 1) / 2;
            const char* pa = prow + (I * 32 + (lane & 31)) * kPitch + hf * 16;
            const char* pb = prow + (J * 32 + (lane & 31)) * kPitch + hf * 16;
            if constexpr (F32) {
              // 32x32x2: the lane's two k per four MFMAs are floats 8 ks + 4 hf .. + 3 of its row (one LDS request)
#pragma unroll 4
              for (int ks = 0; ks < 16; ++ks) {
                const float4 xa = *reinterpret_cast<const float4*>(pb + ks * 32);
                const float4 xb = *reinterpret_cast<const float4*>(pa + ks * 32);
                acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa.x, xb.x, acc[q], 0, 0, 0);
                acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa.y, xb.y, acc[q], 0, 0, 0);
                acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa.z, xb.z, acc[q], 0, 0, 0);
                acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa.w, xb.w, acc[q], 0, 0, 0);
              }
            } else {
#pragma unroll
              for (int ks = 0; ks < 8; ++ks)
                acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(pb + ks * 32),
                                                                 *reinterpret_cast<const bf16x8*>(pa + ks * 32), acc[q], 0, 0, 0);
            }
          }
        }
        if constexpr (Cfg::kAlias) lds_barrier();      // every wave has read its rows: the triangle takes their place
#pragma unroll
        for (int q = 0; q < NTILE; ++q) {
          const int tile = w + q * W;
          if (tile < NTRI) {
            int I = 0;
            while ((I + 1) * (I + 2) / 2 <= tile) ++I;
            const int J = tile - I * (I + 1) / 2;
            lz_write_cos_tile(tri, pool_r, acc[q], I, J, lane);   // the diagonal holds +inf: the row of a pick retires it
          }
        }
      }
      lds_barrier();
      // ================= 3. Algorithm 1 inside the pool, against the outside bound =================
      if (w == 0) {
        // Pool slots lane, lane + 64, .. live in lane `lane` (slots are in token order, so the lowest
        // slot is the lowest token; the mapping keeps the triangle reads free of bank conflicts).  A pick is parked in lane np of two registers; the
        // pick lists and the pending-row tables are written once, after the loop.
        typedef __attribute__((address_space(3))) const float* lds_fp;
        const int tri0 = static_cast<int>(reinterpret_cast<uintptr_t>(
            (__attribute__((address_space(3))) const char*)reinterpret_cast<const char*>(tri)));
        float sq[NQ], mq[NQ];
        int ja[NQ], tja[NQ];
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
          const int p = lane + 64 * q;
          sq[q] = pool_s[p];
          mq[q] = pool_m[p];
          ja[q] = p * 4 + tri0;                        // column offset of the slot
          tja[q] = lz_row_start(p) * 4 + tri0;         // start of its row
        }
        const int jb = __builtin_amdgcn_readfirstlane(jout < 0 ? 0x7fffffff : jout);
        const float gout_u = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(gout)));
        const bool no_out = __builtin_amdgcn_readfirstlane(jout) < 0;
        const int room = __builtin_amdgcn_readfirstlane(min(b - t, kLzMaxPend));
        int np = 0, stop = 0;                        // stop: 1 = bound wins, 2 = nothing finite left
        int rec_i = 0, rec_g = 0;
        while (np < room) {
          float av[NQ];
#pragma unroll
          for (int q = 0; q < NQ; ++q) av[q] = fmaf(nlam, mq[q], sq[q]);
          float best = av[0];
#pragma unroll
          for (int q = 1; q < NQ; ++q) best = hw_max(best, av[q]);
          const float amax = wave_max_uniform(best);
          unsigned long long e[NQ];
#pragma unroll
          for (int q = 0; q < NQ; ++q) e[q] = __ballot(av[q] == amax);
          const int i = first_of_slots<NQ>(e);       // negative when nothing compares equal (NaN)
          if (!(amax > gout_u)) {                    // rare: the bound wins, a tie with it, or nothing finite
            if (!(amax > -INFINITY)) { stop = no_out ? 2 : 1; break; }
            const int ti = __builtin_amdgcn_readfirstlane(pool_tok[i < 0 ? 0 : i]);
            if (!(amax == gout_u && ti < jb)) { stop = 1; break; }
          }
          write_lane2(rec_i, rec_g, i, __float_as_int(amax), np);
          np = __builtin_amdgcn_readfirstlane(np + 1);   // keeps the loop control on the scalar unit
          // element (i,j) of the triangle sits at max(start(i)+j, start(j)+i); the diagonal (+inf) retires i.
          // For any i in [-1, 64*NQ) the larger address stays inside the triangle.
          const int ti4 = lz_row_start(i) * 4, i4 = i * 4;
          float c[NQ];
#pragma unroll
          for (int q = 0; q < NQ; ++q) {
            const int x0 = ti4 + ja[q], x1 = tja[q] + i4;
#ifdef KVR_BOUNDS
            const int xa = kvr_ix(((x0 > x1 ? x0 : x1) - tri0) >> 2, Cfg::kTriBytes / 4, 105) * 4 + tri0;   // 105: triangle element of the race
#else
            const int xa = x0 > x1 ? x0 : x1;
#endif
            c[q] = *reinterpret_cast<lds_fp>(static_cast<uintptr_t>(static_cast<unsigned>(xa)));
          }
#pragma unroll
          for (int q = 0; q < NQ; ++q) mq[q] = hw_max(mq[q], c[q]);
        }
#pragma unroll
        for (int q = 0; q < NQ; ++q) pool_m[lane + 64 * q] = mq[q];   // the pool's m is authoritative
        if (lane < np) {
          const int ri = kvr_ix(rec_i, P, 106);          // 106: pool slot of a pick
          const int tp = kvr_ix(t + lane, kLzMaxB, 107); // 107: number of a pick
          order_l[tp] = pool_tok[ri]; gain_l[tp] = __int_as_float(rec_g);
          pend_l[lane] = ri; pick_r[tp] = pool_r[ri]; pool_picked[ri] = 1;
        }
        t += np;
        if (lane == 0) { shared_i[0] = np; shared_i[1] = t; shared_i[2] = stop; }
      }
      lds_barrier();
      const int np = shared_i[0];
      t = shared_i[1];
      const int stop = shared_i[2];
      // pool members: m from the race (it covers every pick so far), picked members leave
#pragma unroll
      for (int k = 0; k < S; ++k) {
        const int ps = pslot[k];
        if (ps >= 0) {
          m[k] = pool_m[ps];
          if (!have_r) r[k] = pool_r[ps];
          if (pool_picked[ps]) s[k] = -INFINITY;
        }
      }
      if (t >= b) break;
      if (stop == 2 || (np == 0 && !(gout > -INFINITY))) { starved = true; break; }
      if (np == 0) {
        // The bound won at once.  A stale token carried it: it is refreshed below and fresh from then on, so the
        // fresh set grows with every such epoch (at most n of them in a row).  A fresh one: the cut keys left it
        // outside the pool, full keys from here on; under full keys every wave's best fresh tokens are members
        // (equal gains join in token order), so a fresh token can only block on non-finite gains, and then
        // nothing would ever change.
        if (!jout_stale) {
          if (kbits == 32) { starved = true; break; }
          kbits = 32;
        }
        if (++idle > n + 8) { starved = true; break; }   // (never reached on finite input, by the count above)
      } else {
        idle = 0;
      }
      lds_barrier();                               // everyone is done with the triangle and the pool tables
      // ================= 4. picked rows -> LDS; the wave's refresh list against all picks so far =================
      if constexpr (!Cfg::kAlias) {
        // the rows of this epoch's picks, from the pool's rows to the rows of all picks: 16 threads per row
        for (int i = tid >> 4; i < np; i += NT / 16)
          *reinterpret_cast<uint4*>(pk + pick_piece(tid & 15) + kvr_ix(t - np + i, kLzMaxB, 108) * kHalf) =   // 108: row of a pick
              *reinterpret_cast<const uint4*>(prow + kvr_ix(pend_l[i], P, 109) * kPitch + (tid & 15) * 16);   // 109: its pool slot
      } else
      {
        // the rows of this epoch's picks, read again from memory (the triangle has taken the place of
        // the pool's rows): 16 threads per row
        constexpr int RPI = NT / LPR;                  // rows per round
        constexpr int kRounds = (kLzMaxPend + RPI - 1) / RPI;
        // (named registers, not an array: the array form of this block ended up in scratch memory)
        auto row_of = [&](int q) -> uint32_t {            // branch-free: rounds past np re-read the last pick's row
          const int i = min(q * RPI + tid / LPR, np - 1);
          const int tk = order_l[max(t - np + i, 0)];
          return static_cast<uint32_t>(min(max(tk, 0), n - 1)) * pitch_b + (tid % LPR) * 16u;
        };
        auto put = [&](int q, const uint4& v) {           // unconditional stores (rounds past np go to the union area, dead
          const int i = q * RPI + tid / LPR;              // here), so that every load is issued before the first store waits
          char* dst = i < np ? pk + pick_piece(tid % LPR) + kvr_ix(t - np + i, kLzMaxB, 108) * kHalf : uni + tid * 16;
          *reinterpret_cast<uint4*>(dst) = v;
        };
        static_assert(kRounds == 2 || kRounds == 4 || kRounds == 8, "rounds of the pick-row copy");
        for (int q0 = 0; q0 < kRounds; q0 += 4) {         // (one trip unless a workgroup has two waves)
          const uint32_t o0 = row_of(q0), o1 = row_of(q0 + 1);
          const uint32_t o2 = kRounds > 2 ? row_of(q0 + 2) : o0, o3 = kRounds > 2 ? row_of(q0 + 3) : o1;
          const uint4 x0 = *reinterpret_cast<const uint4*>(Vh + o0);
          const uint4 x1 = *reinterpret_cast<const uint4*>(Vh + o1);
          uint4 x2 = x0, x3 = x1;
          if constexpr (kRounds > 2) {
            x2 = *reinterpret_cast<const uint4*>(Vh + o2);
            x3 = *reinterpret_cast<const uint4*>(Vh + o3);
          }
          put(q0, x0);
          put(q0 + 1, x1);
          if constexpr (kRounds > 2) { put(q0 + 2, x2); put(q0 + 3, x3); }
        }
      }
      lds_barrier();
      const int groups = (cnt_r + GR - 1) / GR;
      if (groups > 0) {
        const int kg = lane >> 4;
        const int tiles = kvr_ix((t + 15) >> 4, kLzMaxB / 16 + 1, 110);   // 16-row operands of picked rows (0 when nothing is picked yet; 110)
        // One 64-row group of the list is in flight (the first since before the race): the registers of a
        // 16-row sub-block are refilled for the next group as soon as they have been written to the stage.
        // The groups are unrolled as nested conditionals (group g + 1 inside group g), not a loop: the
        // wait counts of straight-line code are exact, those at a loop head are not, and an inexact one
        // waits for the group just requested.  The next group's rows are requested unconditionally (the
        // list is padded by one group of valid rows).
        auto run_group = [&](auto self, auto gi_c) -> void {
          constexpr int gi = decltype(gi_c)::value;
          float part[GSUB];                          // per 16-row sub-block: max over my four picks of every operand
          if constexpr (F32) {
            // fp32 rows: the registers of the sub-block are its B operand (lane (c, kg): floats 16 j + 4 kg .. + 3 of row
            // c in pre[sub][j]); the rows of the picks give the A operand in the same order, 32 MFMAs of 16x16x4 per tile
#pragma unroll
            for (int sub = 0; sub < GSUB; ++sub) {
              if (!have_r) {
                float ss = 0.f;
#pragma unroll
                for (int q = 0; q < LPC; ++q) {
                  const uint4 x = pre[sub][q];
                  const float e[4] = {__uint_as_float(x.x), __uint_as_float(x.y), __uint_as_float(x.z), __uint_as_float(x.w)};
#pragma unroll
                  for (int u = 0; u < 4; ++u) ss = fmaf(e[u], e[u], ss);
                }
                ss += __shfl_xor(ss, 16);            // the four k-groups hold the four quarters of row c
                ss += __shfl_xor(ss, 32);
                if (kg == 0) lr2[gi * GR + sub * 16 + (lane & 15)] = 1.0f / (sqrtf(ss) + a.eps);
              }
              float pm = 0.f;                        // the floor of Eq. 2
              for (int tl = 0; tl < tiles; ++tl) {
                const char* ap = pk + (kg & 1) * kLzPickPlaneF + (tl * 16 + (lane & 15)) * kLzHalfF + (kg >> 1) * 16;
                float4 av[LPC];
#pragma unroll
                for (int q = 0; q < LPC; ++q) av[q] = *reinterpret_cast<const float4*>(ap + q * 32);
                const float4 p0 = *reinterpret_cast<const float4*>(pick_r + tl * 16 + 4 * kg);
                f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};   // two chains: even and odd pieces
#pragma unroll
                for (int q = 0; q < LPC; q += 2) {
                  const uint4 x0 = pre[sub][q], x1 = pre[sub][q + 1];
                  acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(av[q].x, __uint_as_float(x0.x), acc0, 0, 0, 0);
                  acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(av[q + 1].x, __uint_as_float(x1.x), acc1, 0, 0, 0);
                  acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(av[q].y, __uint_as_float(x0.y), acc0, 0, 0, 0);
                  acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(av[q + 1].y, __uint_as_float(x1.y), acc1, 0, 0, 0);
                  acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(av[q].z, __uint_as_float(x0.z), acc0, 0, 0, 0);
                  acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(av[q + 1].z, __uint_as_float(x1.z), acc1, 0, 0, 0);
                  acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(av[q].w, __uint_as_float(x0.w), acc0, 0, 0, 0);
                  acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(av[q + 1].w, __uint_as_float(x1.w), acc1, 0, 0, 0);
                }
                pm = hw_max(pm, hw_max(hw_max((acc0[0] + acc1[0]) * p0.x, (acc0[1] + acc1[1]) * p0.y),
                                       hw_max((acc0[2] + acc1[2]) * p0.z, (acc0[3] + acc1[3]) * p0.w)));
              }
              fetch(gi + 1, sub);                    // the operand registers are free again
              pm = hw_max(pm, __shfl_xor(pm, 16));   // the four k-groups hold the maxima over different picks
              pm = hw_max(pm, __shfl_xor(pm, 32));
              part[sub] = pm;
            }
            // (the list entries of this group have been consumed: entry 16 * sub + c takes its raw maximum)
#pragma unroll
            for (int sub = 0; sub < GSUB; ++sub)
              if (kg == sub) lrw[gi * GR + sub * 16 + (lane & 15)] = part[sub];
          } else {
#pragma unroll
          for (int sub = 0; sub < 4; ++sub) {
            wave_lds_sync();
#pragma unroll
            for (int q = 0; q < LPC; ++q) {
              const uint4 x = pre[sub][q];
              *reinterpret_cast<uint4*>(stage + ((lane & 15) >> 3) * kLzStagePlane + ((lane >> 4) + 4 * q) * kLzHalf + (lane & 7) * 16) = x;
              if (!have_r) {                         // row (lane >> 4) + 4q of the sub-block is list entry 16*sub + row of the group
                const float ss = sum_sq(x);
                if ((lane & 15) == 15) norm_x[sub * 16 + (lane >> 4) + 4 * q] = ss;
              }
            }
            fetch(gi + 1, sub);
            wave_lds_sync();
            const char* fp = stage + (kg & 1) * kLzStagePlane + (lane & 15) * kLzHalf + (kg >> 1) * 16;
            bf16x8 bfr[4];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bfr[ks] = *reinterpret_cast<const bf16x8*>(fp + ks * 32);
            float pm = 0.f;                          // the floor of Eq. 2
            for (int tl = 0; tl < tiles; tl += 2) {    // two operands at a time: their MFMA chains interleave
              const char* ap = pk + (kg & 1) * kLzPickPlane + (tl * 16 + (lane & 15)) * kLzHalf + (kg >> 1) * 16;
              bf16x8 a0[4];
#pragma unroll
              for (int ks = 0; ks < 4; ++ks) a0[ks] = *reinterpret_cast<const bf16x8*>(ap + ks * 32);
              const float4 p0 = *reinterpret_cast<const float4*>(pick_r + tl * 16 + 4 * kg);
              f32x4 acc0 = {0.f, 0.f, 0.f, 0.f};
              if (tl + 1 < tiles) {
                bf16x8 a1[4];
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) a1[ks] = *reinterpret_cast<const bf16x8*>(ap + 16 * kLzHalf + ks * 32);
                const float4 p1 = *reinterpret_cast<const float4*>(pick_r + tl * 16 + 16 + 4 * kg);
                f32x4 acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                  acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0[ks], bfr[ks], acc0, 0, 0, 0);
                  acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1[ks], bfr[ks], acc1, 0, 0, 0);
                }
                pm = hw_max(pm, hw_max(hw_max(acc1[0] * p1.x, acc1[1] * p1.y), hw_max(acc1[2] * p1.z, acc1[3] * p1.w)));
              } else {
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                  acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0[ks], bfr[ks], acc0, 0, 0, 0);
              }
              pm = hw_max(pm, hw_max(hw_max(acc0[0] * p0.x, acc0[1] * p0.y), hw_max(acc0[2] * p0.z, acc0[3] * p0.w)));
            }
            part[sub] = pm;
          }
          // lane (col, kg) holds partial maxima of row col of sub-block 0..3; list entry 16*sub + col of the
          // group is finished by lane (col, kg = sub).  Exchange through the wave's scratch: [sub][kg][col].
          wave_lds_sync();
#pragma unroll
          for (int sub = 0; sub < 4; ++sub) scratch[sub * 64 + kg * 16 + (lane & 15)] = part[sub];
          wave_lds_sync();
          const float* sp = scratch + kg * 64 + (lane & 15);
          const float mx = hw_max(hw_max(sp[0], sp[16]), hw_max(sp[32], sp[48]));
          lrw[gi * 64 + lane] = mx;                  // (the list entries of this group have been consumed)
          if (!have_r) lr2[gi * 64 + lane] = 1.0f / (sqrtf(norm_x[lane]) + a.eps);
          }
          if constexpr ((gi + 1) * GR < TPW) {
            if (gi + 1 < groups) self(self, std::integral_constant<int, gi + 1>{});
          }
        };
        run_group(run_group, std::integral_constant<int, 0>{});
        wave_lds_sync();
      }
      // refreshed tokens take their new m; who is fresh for the next epoch
      {
        uint32_t now = 0;
#pragma unroll
        for (int k = 0; k < S; ++k) {
          const int ps = pslot[k];
          if (ps <= -2) {
            const int pos = kvr_ix(-2 - ps, TPW, 111);   // 111: list position of a refreshed token
            if (!have_r) r[k] = lr2[pos];
            m[k] = hw_max(m[k], lrw[pos] * r[k]);
          }
          if (ps != -1) now |= 1u << k;              // pool members left the race up to date
          pslot[k] = -1;
        }
        fresh = np > 0 ? now : (fresh | now);
      }
      have_r = true;
      lds_barrier();                               // pass areas are dead: the next epoch reuses the union
    }
  }

  // ---- sort(S): flag the picked tokens, ascending indices by prefix counts
  lds_barrier();
#pragma unroll
  for (int k = 0; k < S; ++k) flag[base + 64 * k + lane] = 0;
  lds_barrier();
  for (int u = tid; u < t; u += NT) flag[kvr_ix(order_l[u], 64 * S * W, 112)] = 1;   // 112: token of a pick
  lds_barrier();
  if (starved) {
    if (tid == 0) {                                  // non-finite input only: lowest unpicked tokens fill up
      int j = 0;
      for (int u = t; u < b; ++u) {
        while (j < n - 1 && flag[j]) ++j;
        order_l[u] = j; gain_l[u] = -INFINITY; flag[j] = 1;
      }
    }
    lds_barrier();
  }
  {
    unsigned long long sel[S];
    int cnt = 0;
#pragma unroll
    for (int k = 0; k < S; ++k) {
      sel[k] = __ballot(tok_of(k) < n && flag[tok_of(k)] != 0);
      cnt += __popcll(sel[k]);
    }
    if (lane == 0) wcount[w] = cnt;
    lds_barrier();
    int off = 0;
    for (int u = 0; u < w; ++u) off += wcount[u];
#pragma unroll
    for (int k = 0; k < S; ++k) {
      if ((sel[k] >> lane) & 1ull) {
        const int rank = off + __popcll(sel[k] & below);
        if (rank < b) idxs_l[rank] = tok_of(k);
      }
      off += __popcll(sel[k]);
    }
  }
  lds_barrier();
  const int bs = a.b;
  const long long ob = static_cast<long long>(h) * bs;
  for (int u = tid; u < b; u += NT) {
    a.idx_sorted[ob + u] = idxs_l[u];
    if (a.pick_order) a.pick_order[ob + u] = order_l[u];
    if (a.pick_gain) a.pick_gain[ob + u] = gain_l[u];
  }
  if constexpr (BUD) {
    for (int u = b + tid; u < bs; u += NT) {                   // entries past the head's budget are padding
      a.idx_sorted[ob + u] = -1;
      if (a.pick_order) a.pick_order[ob + u] = -1;
      if (a.pick_gain) a.pick_gain[ob + u] = -INFINITY;
    }
  }
  if constexpr (!F32) {                                          // (fp32 rows: the caller compacts)
    if ((a.K_out || a.V_out) && (!BUD || b > 0))
      compact_rows<(NT >= 512 ? 2 : 4)>(a.K, a.V, a.K_out, a.V_out, head_off, a.stride_tok, idxs_l, n, b, ob, tid, NT);
  }
}

KVR_BOUNDS_TU(lazy)

// Debug aid: one thread passes the index 5 with the limit 3 through the range check (id 199); nothing is
// accessed.  The bounds build then reports 199, the product build nothing.
__global__ void bounds_selftest_kernel(int32_t* out) {
  const int v = kvr_ix(5, 3, 199);
  if (out) out[0] = v;
}

hipError_t launch_bounds_selftest(int32_t* out, hipStream_t st) {
  hipLaunchKernelGGL(bounds_selftest_kernel, dim3(1), dim3(1), 0, st, out);
  return hipGetLastError();
}

bool lazy_supported(const Layout& lay, int b, float lambda) {
  // (byte offsets inside a head are 32-bit in this kernel)
  return lay.dtype == DT_BF16 && lay.n > 256 && lay.n <= 4096 && b <= kLzMaxB && lambda > 0.0f &&
         static_cast<long long>(lay.n) * lay.stride_tok * 2 < (1ll << 31);
}

bool lazy_f32_supported(const Layout& lay, int b, float lambda) {
  return lay.dtype == DT_F32 && lay.n > 256 && lay.n <= 4096 && b <= kLzMaxB && lambda > 0.0f &&
         static_cast<long long>(lay.n) * lay.stride_tok * 4 < (1ll << 31);
}

// fp32 rows, selection only (the caller compacts): one workgroup of eight waves per head and CU
hipError_t launch_select_lazy_f32(const void* V, const float* s, const Layout& lay, int b, float lambda, float eps,
                                  int32_t* idx_sorted, int32_t* pick_order, float* pick_gain, hipStream_t st) {
  LazyArgs a;
  a.b_h = nullptr; a.only_marked = 0;
  a.K = nullptr; a.V = static_cast<const char*>(V); a.s_in = s;
  a.idx_sorted = idx_sorted; a.pick_order = pick_order; a.pick_gain = pick_gain;
  a.K_out = nullptr; a.V_out = nullptr;
  a.stride_head = lay.stride_head; a.stride_tok = lay.stride_tok;
  a.n = lay.n; a.b = b; a.lambda = lambda; a.eps = eps;
  auto go = [&](auto kern, int smem) -> hipError_t {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(lay.heads), dim3(512), smem, st, a);
    return hipGetLastError();
  };
  if (lay.n <= 2048) return go(&select_lazy_kernel<8, 4, 128, false, true>, LazyCfg<8, 4, 128, true>::smem_bytes());
  return go(&select_lazy_kernel<8, 8, 128, false, true>, LazyCfg<8, 8, 128, true>::smem_bytes());
}

hipError_t launch_select_lazy(const void* K, const void* V, const float* s, const Layout& lay, int b,
                              float lambda, float eps, int32_t* idx_sorted, int32_t* pick_order,
                              float* pick_gain, void* K_out, void* V_out, hipStream_t st, const int32_t* b_h,
                              bool only_marked) {
  LazyArgs a;
  a.b_h = b_h; a.only_marked = only_marked ? 1 : 0;
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
  auto by_shape = [&](auto bud) -> hipError_t {
    constexpr bool BUD = decltype(bud)::value;
    if (lay.n <= 512) return go(&select_lazy_kernel<2, 4, 128, BUD>, 128, LazyCfg<2, 4, 128>::smem_bytes());
    if (lay.n <= 1024) return go(&select_lazy_kernel<4, 4, 128, BUD>, 256, LazyCfg<4, 4, 128>::smem_bytes());
    if (lay.n <= 2048) return go(&select_lazy_kernel<8, 4, kLzPoolWide, BUD>, 512, LazyCfg<8, 4, kLzPoolWide>::smem_bytes());
    return go(&select_lazy_kernel<8, 8, kLzPoolWide, BUD>, 512, LazyCfg<8, 8, kLzPoolWide>::smem_bytes());
  };
  return b_h ? by_shape(std::true_type{}) : by_shape(std::false_type{});
}

}  // namespace kvr
