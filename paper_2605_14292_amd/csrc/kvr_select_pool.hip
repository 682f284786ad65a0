// Greedy selection (paper Sec. 4.1, Algorithm 1) for heads with 256 < n <= 8192
// bf16 tokens and b <= 1024, followed by the compaction of the kept rows.
//
// Exact greedy on a pool.  Streaming all of V for every pick (one cosine row per
// pick) is what Algorithm 1 asks for literally; it is also what makes large n
// memory-bound many times over.  Gains only ever decrease (m only grows), so the
// selection is organised in epochs:
//   1. every token's m is up to date; the P = 128 currently best unselected
//      tokens form the pool (each wave contributes its best P/W, found by a
//      bitwise threshold search on the gains), and the best gain outside the
//      pool is recorded as the bound;
//   2. the pool's rows are gathered into LDS and their P x P cosine triangle is
//      computed on bf16 MFMA (32x32x16, fp32 accumulate), exactly as in the
//      small-n kernel;
//   3. one wave runs Algorithm 1 inside the pool (DPP argmax, one LDS row read
//      per pick) for as long as the pool's best (gain, lower index) beats the
//      bound -- the bound can only have dropped since, so such a pick is the
//      exact argmax of Eq. 2 over all unselected tokens;
//   4. one pass over V applies the rows picked in the epoch (<= 32, as one or two
//      16-row MFMA operands, 16x16x32) to every token outside the pool.
// On the benchmark inputs an epoch serves ~20 picks, so V is streamed ~b/20
// times.  Nothing is approximated.  lambda = 0 has a kernel of its own (select_topb_kernel);
// this one would still return the right picks for it, after passes that change nothing.
//
// Layout: one workgroup per head, W wave64s, token j = 64*S*w + 64*k + lane in
// wave w, lane `lane`, slot k; score, m and inverse norm of a token stay in its
// lane's registers for the whole event (slots 0-7; with sixteen slots per lane,
// n > 4096, the state of slots 8-15 lives in LDS, one column per thread).
#define KVR_BOUNDS_FILE 2   // ids 2xx of the debug build's bounds checks (kvr_bounds.hpp)
#include "kvr_dense_common.hpp"
#include "kvr_kernels.hpp"
#include <type_traits>

namespace kvr {

typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kPool = 128;          // pool size
constexpr int kPoolMaxB = 1024;     // largest budget (the pick lists in LDS are sized for the call's b)
constexpr int kPoolMaxPend = 32;    // picks per epoch (two 16-row MFMA operands)
constexpr int kPoolPitch = 272;     // bytes per staged row (256 + 16)
constexpr int kSelBits = 16;        // leading bits of a gain's ordered key used to choose the pool
constexpr int kPoolChunk = 16;      // tokens staged per step and wave in the pass over V

struct PoolArgs {
  const char* K; const char* V; const float* s_in;
  int32_t* idx_sorted; int32_t* pick_order; float* pick_gain;
  char* K_out; char* V_out;
  long long stride_head, stride_tok;   // elements
  int n, b;
  float lambda, eps;
  const int32_t* b_h;                  // per-head budgets <= b (output rows stay b apart), or null
};

template <int W, int S> struct PoolCfg {
  static constexpr int kWaveStage = kPoolChunk * kPoolPitch + 1024 + 256;   // row stage + 256-float scratch + 64 squared norms per wave
  static constexpr int kTriBytes = kPool * (kPool + 1) / 2 * 4;
  static constexpr int kUnion = (W * kWaveStage > kTriBytes ? W * kWaveStage : kTriBytes);
  // floats: slots 64 | shared 16 | wcount 16 | pool_tok,r,s,m,picked 5*128 | pend 32 | pend_r 32 |
  //         order,gain,idxs 3*bcap (b rounded up to 64) ; then pool rows ; then the union area (triangle, stages, and at
  //         the end the pick flags of the read-out) ; then score, m, inverse norm and pool slot of the
  //         token slots that do not live in registers
  static constexpr int kFixedFloats = 64 + 16 + 16 + 5 * kPool + 64;          // without the pick lists
  static constexpr int kRegSlots = S > 8 ? 8 : S;
  static constexpr int kLdsState = (S - kRegSlots) * 64 * W * 16;
  static_assert(64 * S * W * 4 <= kUnion, "the pick flags of the read-out fit the union area");
  static constexpr int smem_bytes(int b) {
    return (kFixedFloats + 3 * ((b + 63) & ~63)) * 4 + kPool * kPoolPitch + kUnion + kLdsState;
  }
};

// BUD: per-head budgets are read from a.b_h (a variant of its own: the extra live value costs the
// plain kernel a register it does not have).
// PRUNE: the candidate reduction by the score bound (a variant of its own as well: where nothing
// can be dropped, its row masks cost a head 3 us).
template <int W, int S, bool BUD, bool PRUNE>
__global__ __launch_bounds__(64 * W, (W <= 4 ? 2 : 1)) void select_pool_kernel(PoolArgs a) {
  using Cfg = PoolCfg<W, S>;
  constexpr int TPW = 64 * S;
  constexpr int NT = 64 * W;
  constexpr int Q = kPool / W;                     // pool members contributed per wave
  constexpr int CH = kPoolChunk;
  constexpr int LPC = CH / 4;
  extern __shared__ __align__(16) float smem[];
  float* slot_gain = smem;                                       // [2][16]
  int32_t* slot_idx = reinterpret_cast<int32_t*>(smem + 32);     // [2][16]
  int32_t* shared_i = reinterpret_cast<int32_t*>(smem + 64);     // [16] np, t, stop reason
  int32_t* wcount = reinterpret_cast<int32_t*>(smem + 80);       // [16]
  int32_t* pool_tok = reinterpret_cast<int32_t*>(smem + 96);     // [P] token of the member, -1 = none
  float* pool_r = smem + 96 + kPool;
  float* pool_s = smem + 96 + 2 * kPool;
  float* pool_m = smem + 96 + 3 * kPool;
  int32_t* pool_picked = reinterpret_cast<int32_t*>(smem + 96 + 4 * kPool);
  int32_t* pend_l = reinterpret_cast<int32_t*>(smem + 96 + 5 * kPool);        // [32] pool slots picked this epoch
  float* pend_r = smem + 96 + 5 * kPool + 32;                                  // [32] their inverse norms
  int32_t* order_l = reinterpret_cast<int32_t*>(smem + 96 + 5 * kPool + 64);
  const int bcap = (a.b + 63) & ~63;                             // rows of the pick lists
  float* gain_l = smem + 96 + 5 * kPool + 64 + bcap;
  int32_t* idxs_l = reinterpret_cast<int32_t*>(smem + 96 + 5 * kPool + 64 + 2 * bcap);
  char* prow = reinterpret_cast<char*>(smem + Cfg::kFixedFloats + 3 * bcap);   // [P][272 B] pool rows
  char* uni = prow + kPool * kPoolPitch;
  float* tri = reinterpret_cast<float*>(uni);                    // packed P x P cosine triangle (race) ...
  // ... or the per-wave row stages of the pass over V ...
  int32_t* flag = reinterpret_cast<int32_t*>(uni);               // ... or, at the end, [n padded] pick flags for the ascending read-out
  constexpr int SR = Cfg::kRegSlots;                             // token slots whose state lives in registers
  constexpr int SL = S - SR;                                     // ... and in LDS, [slot - SR][thread]
  float* sX = reinterpret_cast<float*>(uni + Cfg::kUnion);
  float* mX = sX + SL * NT;
  float* rX = mX + SL * NT;
  int32_t* pX = reinterpret_cast<int32_t*>(rX + SL * NT);

  const int h = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = a.n;
  // the head's own budget: its picks are the first b picks of a run for a.b (the rows of the
  // outputs per head), so the epochs stop there
  const int b = BUD ? min(max(a.b_h[blockIdx.x], 0), a.b) : a.b;      // a scalar load: the index is uniform
  const long long head_off = h * a.stride_head * 2;             // bytes
  const char* Vh = a.V + head_off;
  const int base = w * TPW;
  char* stage = uni + w * Cfg::kWaveStage;
  float* scratch = reinterpret_cast<float*>(stage + CH * kPoolPitch);
  float* norm_x = scratch + 256;                                 // [64] squared norms of the wave's current 64 tokens

  float s[SR], m[SR], r[SR];
  int pslot[SR];                 // pool slot of this token in the current epoch, or -1
  // slot k of this lane: a register for k < SR, this thread's LDS column otherwise (k is a constant
  // wherever these are used: the loops over the slots are unrolled)
  const int tidx = threadIdx.x;
  auto get_s = [&](int k) -> float { return k < SR ? s[k < SR ? k : 0] : sX[(k - SR) * NT + tidx]; };
  auto get_m = [&](int k) -> float { return k < SR ? m[k < SR ? k : 0] : mX[(k - SR) * NT + tidx]; };
  auto get_r = [&](int k) -> float { return k < SR ? r[k < SR ? k : 0] : rX[(k - SR) * NT + tidx]; };
  auto get_p = [&](int k) -> int { return k < SR ? pslot[k < SR ? k : 0] : pX[(k - SR) * NT + tidx]; };
  auto set_s = [&](int k, float v) { if (k < SR) s[k < SR ? k : 0] = v; else sX[(k - SR) * NT + tidx] = v; };
  auto set_m = [&](int k, float v) { if (k < SR) m[k < SR ? k : 0] = v; else mX[(k - SR) * NT + tidx] = v; };
  auto set_r = [&](int k, float v) { if (k < SR) r[k < SR ? k : 0] = v; else rX[(k - SR) * NT + tidx] = v; };
  auto set_p = [&](int k, int v) { if (k < SR) pslot[k < SR ? k : 0] = v; else pX[(k - SR) * NT + tidx] = v; };
  auto tok_of = [&](int k) -> int { return base + 64 * k + lane; };
#pragma unroll
  for (int k = 0; k < S; ++k) {
    set_s(k, tok_of(k) < n ? a.s_in[static_cast<long long>(h) * n + tok_of(k)] : -INFINITY);
    set_m(k, 0.f);
    set_r(k, 0.f);
    set_p(k, -1);
  }
  const float nlam = -a.lambda;
  int par = 0;
  int t = 0;
  int kbits = kSelBits;          // leading key bits the pool choice looks at (uniform)
  bool starved = false;

  auto wg_argmax = [&](const float (&av)[S], float& gbest, int& ibest) {
    float best = av[0];
#pragma unroll
    for (int k = 1; k < S; ++k) best = hw_max(best, av[k]);
    const float amax_w = wave_max_uniform(best);
    int i_w = -1;
#pragma unroll
    for (int k = S - 1; k >= 0; --k) {
      const unsigned long long eq = __ballot(av[k] == amax_w);
      if (eq) i_w = base + 64 * k + (__ffsll(static_cast<long long>(eq)) - 1);
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
    float gmax; int i;
    float sa[S];
#pragma unroll
    for (int k = 0; k < S; ++k) sa[k] = get_s(k);
    wg_argmax(sa, gmax, i);
    if (!(gmax > -INFINITY)) starved = true;
    else { if (tid == 0) { order_l[0] = i; gain_l[0] = gmax; } t = 1; }
  } else {
    // Inverse norms (Eq. 1) are not taken in a pass of their own: the first epoch needs them for
    // its pool members only, which get them while their rows are gathered, and every other token
    // gets its norm in the first epoch's pass over V, which reads the row anyway.  Until then
    // r = 0 (it is only ever used for pool members and in that pass).
    bool have_r = false;
    // Exact candidate reduction (as in the kernels for short heads): while fewer than b tokens are
    // selected one of the b best-scored is free and gains at least s_(b) - lambda, and a token gains
    // at most its score, so a token with s_j < s_(b) - lambda never wins Eq. 3.  Such tokens get the
    // score -inf (they are never a pool member or a pick, so the picks are unchanged) and their rows
    // are not read in the passes over V.  With scores that spread by more than lambda most of a long
    // head goes; with scores far below lambda nothing does.
    // Nothing can go when the finite scores spread by less than lambda (then s_(b) - lambda is below
    // all of them); one workgroup-wide min/max settles that before the search for s_(b).
    unsigned long long alive[PRUNE ? S : 1];         // per slot: which lanes' tokens still count (wave-uniform)
    bool wide = false;
    if constexpr (PRUNE) {
    {
      float hi = -INFINITY, lo = INFINITY;
#pragma unroll
      for (int k = 0; k < S; ++k) {
        const float sk = get_s(k);
        if (sk > -INFINITY && sk < INFINITY) { hi = hw_max(hi, sk); lo = fminf(lo, sk); }
      }
      hi = wave_max_uniform(hi);
      lo = -wave_max_uniform(-lo);
      if (lane == 0) { slot_gain[par * 16 + w] = hi; slot_gain[32 + w] = lo; }   // (smem 32.. is slot_idx: free until the first argmax)
      lds_barrier();
      float ghi = -INFINITY, glo = INFINITY;
#pragma unroll
      for (int u = 0; u < W; ++u) { ghi = hw_max(ghi, slot_gain[par * 16 + u]); glo = fminf(glo, slot_gain[32 + u]); }
      par ^= 1;
      wide = __builtin_amdgcn_readfirstlane(ghi - glo > a.lambda ? 1 : 0) != 0;   // false also when no score is finite
      lds_barrier();                                 // the min/max slots are rewritten below
    }
    if (!wide) {
#pragma unroll
      for (int k = 0; k < S; ++k) alive[k] = __ballot(!(get_s(k) == -INFINITY));
    } else {
      uint32_t key[S];
#pragma unroll
      for (int k = 0; k < S; ++k) key[k] = tok_of(k) < n ? ordered_key(get_s(k) + 0.0f) : 0u;
      uint32_t T = 0;                                // s_(b) from the leading 16 bits: at most s_(b), the bound only loosens
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
      for (int k = 0; k < S; ++k) {
        const float sk = get_s(k);
        if (sk < thr) set_s(k, -INFINITY);           // (a NaN threshold or score leaves the token in)
        alive[k] = __ballot(!(sk < thr) && !(sk == -INFINITY));
      }
    }
    }
    auto sum_sq = [](const uint4& x) -> float {
      const float e[8] = {bf16_lo(x.x), bf16_hi(x.x), bf16_lo(x.y), bf16_hi(x.y),
                          bf16_lo(x.z), bf16_hi(x.z), bf16_lo(x.w), bf16_hi(x.w)};
      float ss = 0.f;
#pragma unroll
      for (int q = 0; q < 8; ++q) ss = fmaf(e[q], e[q], ss);
      return group16_sum(ss);                        // the 16 lanes of a row hold its 16-byte chunks
    };

    while (t < b) {
      // ================= 1. pool = the best Q unselected tokens of every wave =================
      float g[S];
      uint32_t key[S];
#pragma unroll
      // Keys are cut to their leading kbits bits: the pool only has to be a good guess (the
      // race against the exact outside bound keeps the picks exact), and the search is shorter.
      // When the cut keys cannot tell a wave's best tokens apart the best one may be left outside
      // and the epoch ends without a pick; it is then repeated on the full keys, where the best
      // token of every wave is a member (equal values join in token order).
      for (int k = 0; k < S; ++k) { g[k] = fmaf(nlam, get_m(k), get_s(k)); key[k] = ordered_key(g[k]) >> (32 - kbits); }
      uint32_t tau = 0;                              // largest key value with at least Q keys >= it
      for (int bit = kbits - 1; bit >= 0; --bit) {
        const uint32_t cand = tau | (1u << bit);
        int c = 0;
#pragma unroll
        for (int k = 0; k < S; ++k) c += __popcll(__ballot(key[k] >= cand));
        if (c >= Q) tau = cand;
      }
      int taken = 0;                                 // members with key > tau come first, ties in token order
#pragma unroll
      for (int k = 0; k < S; ++k) taken += __popcll(__ballot(key[k] > tau));
      int need_eq = Q - taken;                       // how many of the key == tau tokens join
      int rank_base = 0;
      float go[S];                                   // gains of the tokens left outside
#pragma unroll
      for (int k = 0; k < S; ++k) {
        const bool above = key[k] > tau, equal = key[k] == tau;
        const unsigned long long eqm = __ballot(equal);
        const int eq_before = __popcll(eqm & ((1ull << lane) - 1ull));
        const bool in = above || (equal && eq_before < need_eq);
        const unsigned long long inm = __ballot(in);
        const int slot = w * Q + kvr_ix_if(in, rank_base + __popcll(inm & ((1ull << lane) - 1ull)), Q, 201);   // 201: a member's place in the wave's share
        set_p(k, in ? slot : -1);
        if (in) {
          pool_tok[slot] = tok_of(k) < n ? tok_of(k) : -1;
          pool_r[slot] = get_r(k);
          pool_s[slot] = get_s(k);
          pool_m[slot] = get_m(k);
          pool_picked[slot] = 0;
        }
        go[k] = in ? -INFINITY : g[k];
        rank_base += __popcll(inm);
        const int eq_in = __popcll(eqm);
        need_eq -= eq_in < need_eq ? eq_in : need_eq;
      }
      float gout; int jout;
      wg_argmax(go, gout, jout);                     // barrier inside: the pool tables are complete
      // ================= 2. pool rows -> LDS, cosine triangle on MFMA =================
      {
        // all row loads of a thread are issued before the first one is stored: with the loads
        // and stores interleaved, every load waits for the one before it
        constexpr int kGat = kPool * 16 / NT;          // rows per thread
        uint4 x[kGat];
#pragma unroll
        for (int k = 0; k < kGat; ++k) {
          const int tk = pool_tok[k * (NT / 16) + (tid >> 4)];
          const int tkc = kvr_ix(tk < 0 ? 0 : tk, n, 203);   // an empty slot reads row 0 and stores zeros (203: token of a pool member)
          x[k] = *reinterpret_cast<const uint4*>(Vh + (static_cast<long long>(tkc) * a.stride_tok + (tid & 15) * 8) * 2);
        }
#pragma unroll
        for (int k = 0; k < kGat; ++k) {
          const int slot = k * (NT / 16) + (tid >> 4);
          if (pool_tok[slot] < 0) x[k] = make_uint4(0u, 0u, 0u, 0u);   // (only here: a select between the loads would make each wait for the one before)
          *reinterpret_cast<uint4*>(prow + slot * kPoolPitch + (tid & 15) * 16) = x[k];
        }
        if (!have_r) {
#pragma unroll
          for (int k = 0; k < kGat; ++k) {
            const int slot = k * (NT / 16) + (tid >> 4);
            const float ss = sum_sq(x[k]);
            if ((tid & 15) == 0) pool_r[slot] = pool_tok[slot] < 0 ? 0.f : 1.0f / (sqrtf(ss) + a.eps);
          }
        }
      }
      lds_barrier();
      {
        const int hf = lane >> 5;
        for (int tile = w; tile < 10; tile += W) {   // lower-triangular 32x32 tiles of the 128 x 128 matrix
          int I = 0;
          while ((I + 1) * (I + 2) / 2 <= tile) ++I;
          const int J = tile - I * (I + 1) / 2;
          f32x16 acc = {0};
          const char* pa = prow + (I * 32 + (lane & 31)) * kPoolPitch + hf * 16;
          const char* pb = prow + (J * 32 + (lane & 31)) * kPoolPitch + hf * 16;
#pragma unroll
          for (int ks = 0; ks < 8; ++ks)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(pa + ks * 32),
                                                          *reinterpret_cast<const bf16x8*>(pb + ks * 32), acc, 0, 0, 0);
          write_cos_tile(tri, pool_r, acc, I, J, lane);   // the diagonal holds +inf: the row of a pick retires it
        }
      }
      lds_barrier();
      // ================= 3. Algorithm 1 inside the pool, against the outside bound =================
      if (w == 0) {
        // Pool slots lane and lane + 64 live in lane `lane` (slots are in token order, so the lowest
        // slot is the lowest token; the mapping keeps the triangle reads free of bank conflicts).  A pick
        // is parked in lane np of two registers; the pick lists and the pending-row tables are written
        // once, after the loop.
        const int p0 = lane, p1 = lane + 64;
        const float s0 = pool_s[p0], s1 = pool_s[p1];
        float m0 = pool_m[p0], m1 = pool_m[p1];
        typedef __attribute__((address_space(3))) const float* lds_fp;
        const int tri0 = static_cast<int>(reinterpret_cast<uintptr_t>(
            (__attribute__((address_space(3))) const char*)reinterpret_cast<const char*>(tri)));
        const int ja0 = p0 * 4 + tri0, ja1 = p1 * 4 + tri0;
        const int tja0 = p0 * (p0 + 1) * 2 + tri0, tja1 = p1 * (p1 + 1) * 2 + tri0;
        const int jb = __builtin_amdgcn_readfirstlane(jout < 0 ? 0x7fffffff : jout);
        const float gout_u = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(gout)));
        const bool no_out = __builtin_amdgcn_readfirstlane(jout) < 0;
        const int room = __builtin_amdgcn_readfirstlane(min(b - t, kPoolMaxPend));
        int np = 0, stop = 0;                        // stop: 1 = bound wins, 2 = nothing finite left
        int rec_i = 0, rec_g = 0;
        while (np < room) {
          const float a0 = fmaf(nlam, m0, s0), a1 = fmaf(nlam, m1, s1);
          const float amax = wave_max_uniform(hw_max(a0, a1));
          const unsigned long long e0 = __ballot(a0 == amax), e1 = __ballot(a1 == amax);
          const unsigned long long e01[2] = {e0, e1};
          const int i = first_of_slots<2>(e01);
          if (!(amax > gout_u)) {                    // rare: the bound wins, a tie with it, or nothing finite
            if (!(amax > -INFINITY)) { stop = no_out ? 2 : 1; break; }
            const int ti = __builtin_amdgcn_readfirstlane(pool_tok[i < 0 ? 0 : i]);
            if (!(amax == gout_u && ti < jb)) { stop = 1; break; }
          }
          write_lane2(rec_i, rec_g, i, __float_as_int(amax), np);
          np = __builtin_amdgcn_readfirstlane(np + 1);   // keeps the loop control on the scalar unit
          // element (i,j) of the triangle sits at max(T(i)+j, T(j)+i); the diagonal (+inf) retires i
          const int ti4 = i * (i + 1) * 2, i4 = i * 4;
          const int x00 = ti4 + ja0, x01 = tja0 + i4, x10 = ti4 + ja1, x11 = tja1 + i4;
          const float c0 = *reinterpret_cast<lds_fp>(static_cast<uintptr_t>(static_cast<unsigned>(x00 > x01 ? x00 : x01)));
          const float c1 = *reinterpret_cast<lds_fp>(static_cast<uintptr_t>(static_cast<unsigned>(x10 > x11 ? x10 : x11)));
          m0 = hw_max(m0, c0);
          m1 = hw_max(m1, c1);
        }
        pool_m[p0] = m0; pool_m[p1] = m1;            // the pool's m is authoritative
        if (lane < np) {
          const int ri = kvr_ix(rec_i, kPool, 206);      // 206: pool slot of a pick
          const int tp = kvr_ix(t + lane, bcap, 207);    // 207: number of a pick
          order_l[tp] = pool_tok[ri]; gain_l[tp] = __int_as_float(rec_g);
          const int pl = kvr_ix(lane, kPoolMaxPend, 208);   // 208: picks of one epoch
          pend_l[pl] = ri; pend_r[pl] = pool_r[ri]; pool_picked[ri] = 1;
        }
        t += np;
        if (lane == 0) { shared_i[0] = np; shared_i[1] = t; shared_i[2] = stop; }
      }
      lds_barrier();
      const int np = shared_i[0];
      t = shared_i[1];
      const int stop = shared_i[2];
      // pool members: m from the race, picked members leave
#pragma unroll
      for (int k = 0; k < S; ++k) {
        const int ps = get_p(k);
        if (ps >= 0) {
          set_m(k, pool_m[ps]);
          if (!have_r) set_r(k, pool_r[ps]);
          if (pool_picked[ps]) set_s(k, -INFINITY);
        }
      }
      if (t >= b) break;
      if (stop == 2 || (np == 0 && !(gout > -INFINITY))) { starved = true; break; }
      if (np == 0 && t + 1 == b) {                   // the outside token wins the last pick: no row needed
        if (tid == 0) { order_l[t] = jout; gain_l[t] = gout; }
#pragma unroll
        for (int k = 0; k < S; ++k) { if (tok_of(k) == jout) set_s(k, -INFINITY); }
        ++t;
        break;
      }
      if (np == 0) {
        if (kbits == 32) { starved = true; break; }  // cannot happen on finite input: the best token was in the pool
        kbits = 32;                                  // the outside bound won on cut keys: full keys from here on
#pragma unroll
        for (int k = 0; k < S; ++k) set_p(k, -1);
        lds_barrier();                               // the pool tables are rewritten next
        continue;
      }
      lds_barrier();                               // everyone is done with the triangle (the stages alias it)
      // ================= 4. one pass over V: the epoch's picks against every outside token =================
      if (np > 0) {
        const int kg = lane >> 4;
        const int tiles = (np + 15) >> 4;            // 1 or 2 A operands of 16 picked rows
        bf16x8 af[2][4];
        float pr[2][4];
#pragma unroll
        for (int at = 0; at < 2; ++at) {
          const int pi = at * 16 + (lane & 15);
          const int ps = pi < np ? kvr_ix(pend_l[pi], kPool, 209) : -1;   // 209: pool slot of a pending row
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) {
            uint4 x = make_uint4(0u, 0u, 0u, 0u);
            if (ps >= 0) x = *reinterpret_cast<const uint4*>(prow + ps * kPoolPitch + ks * 64 + kg * 16);
            af[at][ks] = *reinterpret_cast<bf16x8*>(&x);
          }
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int ri = at * 16 + 4 * kg + i;     // result row i of this lane belongs to pick ri
            pr[at][i] = ri < np ? pend_r[ri] : 0.f;
          }
        }
        // Two 64-token groups of this wave are in flight: the registers of a 16-token sub-block
        // are refilled for the group after next as soon as they have been written to the stage.
        // Rows past n are clamped to the last row (their results belong to padding tokens, whose
        // scores are -inf), so the loads are straight-line code.
        // (one group with eight slots per lane: two do not fit the register file there)
        constexpr int kDepth = S >= 8 ? 1 : 2;
        uint4 preA[4][LPC], preB[4][LPC];              // even and odd groups
        auto fetch = [&](int kk, int sub, int slot) {
          int row0 = base + (lane >> 4);
          asm volatile("" : "+v"(row0));             // keep the unrolled pass from hoarding addresses
          if (PRUNE && wide) {                       // (uniform: heads without dropped tokens take the plain loads)
            asm volatile("" ::: "memory");           // keeps this a branch: folded into selects it costs every head four VALU instructions a load
            const uint32_t on16 = static_cast<uint32_t>(alive[PRUNE ? kk : 0] >> (sub * CH)) & 0xffffu;   // the sub-block's live rows
#pragma unroll
            for (int q = 0; q < LPC; ++q) {
              const int row = min(row0 + (kk * 4 + sub) * CH + 4 * q, n - 1);
              // a row nobody can pick any more is not read: its lanes re-read the wave's first row (a cache
              // hit; what they compute belongs to a token that never counts again)
              const int rowc = ((on16 >> ((lane >> 4) + 4 * q)) & 1u) ? row : min(base, n - 1);
              const uint4 x = *reinterpret_cast<const uint4*>(Vh + (static_cast<long long>(rowc) * a.stride_tok + (lane & 15) * 8) * 2);
              if (slot == 0) preA[sub][q] = x; else preB[sub][q] = x;
            }
          } else {
#pragma unroll
            for (int q = 0; q < LPC; ++q) {
              const int row = min(row0 + (kk * 4 + sub) * CH + 4 * q, n - 1);
              const uint4 x = *reinterpret_cast<const uint4*>(Vh + (static_cast<long long>(row) * a.stride_tok + (lane & 15) * 8) * 2);
              if (slot == 0) preA[sub][q] = x; else preB[sub][q] = x;
            }
          }
        };
#pragma unroll
        for (int g = 0; g < kDepth; ++g)
#pragma unroll
          for (int sub = 0; sub < 4; ++sub)
            if (g < S) fetch(g, sub, g);
#pragma unroll
        for (int k = 0; k < S; ++k) {
          float part[4];                             // per 16-token sub-block: max over my four picked rows
#pragma unroll
          for (int sub = 0; sub < 4; ++sub) {
            wave_lds_sync();
#pragma unroll
            for (int q = 0; q < LPC; ++q) {
              const uint4 x = (k % kDepth == 0) ? preA[sub][q] : preB[sub][q];
              *reinterpret_cast<uint4*>(stage + ((lane >> 4) + 4 * q) * kPoolPitch + (lane & 15) * 16) = x;
              if (!have_r) {                         // row (lane >> 4) + 4q of the sub-block belongs to lane 16*sub + row
                const float ss = sum_sq(x);
                if ((lane & 15) == 0) norm_x[sub * 16 + (lane >> 4) + 4 * q] = ss;
              }
            }
            if (k + kDepth < S) fetch(k + kDepth, sub, k % kDepth);
            wave_lds_sync();
            const char* fp = stage + (lane & 15) * kPoolPitch + kg * 16;
            bf16x8 bfr[4];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bfr[ks] = *reinterpret_cast<const bf16x8*>(fp + ks * 64);
            f32x4 acc0 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[0][ks], bfr[ks], acc0, 0, 0, 0);
            float pm = hw_max(hw_max(acc0[0] * pr[0][0], acc0[1] * pr[0][1]),
                                   hw_max(acc0[2] * pr[0][2], acc0[3] * pr[0][3]));
            if (tiles > 1) {
              f32x4 acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
              for (int ks = 0; ks < 4; ++ks) acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[1][ks], bfr[ks], acc1, 0, 0, 0);
              const float pm1 = hw_max(hw_max(acc1[0] * pr[1][0], acc1[1] * pr[1][1]),
                                            hw_max(acc1[2] * pr[1][2], acc1[3] * pr[1][3]));
              pm = hw_max(pm, pm1);
            }
            part[sub] = pm;
          }
          // lane (col, kg) holds partial maxima of token col of sub-block 0..3; the owner of token
          // (sub, col) is lane (col, kg = sub).  Exchange through the wave's scratch: [sub][kg][col].
          wave_lds_sync();
#pragma unroll
          for (int sub = 0; sub < 4; ++sub) scratch[sub * 64 + kg * 16 + (lane & 15)] = part[sub];
          wave_lds_sync();
          const float* sp = scratch + kg * 64 + (lane & 15);
          const float mx = hw_max(hw_max(sp[0], sp[16]), hw_max(sp[32], sp[48]));
          const int ps = get_p(k);
          float rk = get_r(k);
          if (!have_r && ps < 0) { rk = tok_of(k) < n ? 1.0f / (sqrtf(norm_x[lane]) + a.eps) : 0.f; set_r(k, rk); }
          if (ps < 0) set_m(k, hw_max(get_m(k), mx * rk));
        }
      }
      have_r = true;
#pragma unroll
      for (int k = 0; k < S; ++k) set_p(k, -1);
      lds_barrier();                               // stages are dead: the next epoch reuses the area
    }
  }

  // ---- sort(S): flag the picked tokens, ascending indices by prefix counts
  lds_barrier();
#pragma unroll
  for (int k = 0; k < S; ++k) flag[base + 64 * k + lane] = 0;
  lds_barrier();
  for (int u = tid; u < t; u += NT) flag[kvr_ix(order_l[u], 64 * S * W, 212)] = 1;   // 212: token of a pick
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
        const int rank = off + __popcll(sel[k] & ((1ull << lane) - 1ull));
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
  if ((a.K_out || a.V_out) && (!BUD || b > 0))
    compact_rows<(NT >= 512 ? 2 : 4)>(a.K, a.V, a.K_out, a.V_out, head_off, a.stride_tok, idxs_l, n, b, ob, tid, NT);
}

KVR_BOUNDS_TU(pool)

bool pool_supported(const Layout& lay, int b) {
  return lay.dtype == DT_BF16 && lay.n > 256 && lay.n <= 8192 && b <= kPoolMaxB;
}

hipError_t launch_select_pool(const void* K, const void* V, const float* s, const Layout& lay, int b,
                              float lambda, float eps, int32_t* idx_sorted, int32_t* pick_order,
                              float* pick_gain, void* K_out, void* V_out, hipStream_t st, const int32_t* b_h,
                              bool prune) {
  PoolArgs a;
  a.b_h = b_h;
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
  auto by_shape = [&](auto bud, auto pr) -> hipError_t {
    constexpr bool BUD = decltype(bud)::value, PR = decltype(pr)::value;
    if (lay.n <= 512) return go(&select_pool_kernel<2, 4, BUD, PR>, 128, PoolCfg<2, 4>::smem_bytes(b));
    if (lay.n <= 1024) return go(&select_pool_kernel<4, 4, BUD, PR>, 256, PoolCfg<4, 4>::smem_bytes(b));
    if (lay.n <= 2048) return go(&select_pool_kernel<8, 4, BUD, PR>, 512, PoolCfg<8, 4>::smem_bytes(b));
    if (lay.n <= 4096) return go(&select_pool_kernel<8, 8, BUD, PR>, 512, PoolCfg<8, 8>::smem_bytes(b));
    return go(&select_pool_kernel<8, 16, BUD, PR>, 512, PoolCfg<8, 16>::smem_bytes(b));
  };
  if (b_h) return prune ? by_shape(std::true_type{}, std::true_type{}) : by_shape(std::true_type{}, std::false_type{});
  return prune ? by_shape(std::false_type{}, std::true_type{}) : by_shape(std::false_type{}, std::false_type{});
}

}  // namespace kvr
