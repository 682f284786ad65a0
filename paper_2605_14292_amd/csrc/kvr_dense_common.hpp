// Pieces shared by the fused kernels for short heads (n <= 256 bf16 tokens): wave-level
// reductions, the padded LDS row stage and its MFMA fragment reads.
#pragma once
#include "kvr_device.hpp"
#include "kvr_bounds.hpp"
#ifndef KVR_BOUNDS_FILE
#define KVR_BOUNDS_FILE 0   // (a source file that reports its bounds checks defines its number before this header)
#endif

namespace kvr {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kDenseThreads = 256;
constexpr int kRowPitch = 272;   // bytes per staged row: 256 + 16 so that 8 consecutive rows hit distinct banks

__host__ __device__ constexpr int dense_tri_floats(int NT) { return (NT * 32) * (NT * 32 + 1) / 2; }
__host__ __device__ constexpr int dense_region_a(int NT) {
  const int tri = dense_tri_floats(NT) * 4, stage = NT * 32 * kRowPitch;
  return ((tri > stage ? tri : stage) + 15) & ~15;
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
      "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf"
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
// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits until every
// global store of the wave has been acknowledged by memory, which costs microseconds after a
// burst of output rows and is needed by nobody: no wave reads what another one wrote to HBM.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
// max(a, b) as the hardware does it (a NaN operand yields the other one), without
// the canonicalising self-max the compiler adds around fmaxf on loaded values
__device__ __forceinline__ float hw_max(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
// ra[lane ln] = va, rb[lane ln] = vb for wave-uniform va, vb, ln; the other lanes keep their
// values.  The lane select goes through m0 because a VALU instruction reads one SGPR only.
__device__ __forceinline__ void write_lane2(int& ra, int& rb, int va, int vb, int ln) {
  va = __builtin_amdgcn_readfirstlane(va);             // no-ops when the compiler knows them uniform
  vb = __builtin_amdgcn_readfirstlane(vb);
  ln = __builtin_amdgcn_readfirstlane(ln);
  asm("s_mov_b32 m0, %4\n\tv_writelane_b32 %0, %2, m0\n\tv_writelane_b32 %1, %3, m0"
      : "+v"(ra), "+v"(rb)
      : "s"(va), "s"(vb), "s"(ln)
      : "m0");
}
// Index of the winning token when token lane + 64*q lives in slot q of lane `lane`: e[q] are the lanes
// whose slot-q token equals the maximum.  The lowest token wins: the lowest non-empty slot, and the
// lowest lane within it.  Negative or meaningless (but below 64*NQ) when all masks are empty.
// (Why lane + 64*q and not NQ*lane + q: the race reads element (i, j) of the packed triangle for every j
// at once, at T(i) + j for j < i and at T(j) + i for j > i, T(j) = j(j+1)/2.  With consecutive j across the
// lanes the first is a stride-1 read and the second hits T(j) mod 64, and the triangular numbers of 64
// consecutive j are a complete residue system mod 64: neither has a bank conflict.  With j = NQ*lane + q
// the lanes read stride NQ and T(NQ*lane) mod 64, which collide.)
template <int NQ>
__device__ __forceinline__ int first_of_slots(const unsigned long long (&e)[NQ]) {
  if constexpr (NQ == 2) {
    // five scalar instructions, four of them in a chain (the race's time is its instruction count);
    // with both masks empty (only a NaN maximum does that) the result is 63, which callers never use
    int i, L;
    unsigned long long m;
    asm("s_cmp_lg_u64 %3, 0\n\t"
        "s_cselect_b64 %1, %3, %4\n\t"
        "s_cselect_b32 %0, 0, 64\n\t"
        "s_ff1_i32_b64 %2, %1\n\t"
        "s_add_i32 %0, %0, %2"
        : "=&s"(i), "=&s"(m), "=&s"(L)
        : "s"(e[0]), "s"(e[1])
        : "scc");
    return i;
  } else {
    // slot q's first winner is token ff1(e[q]) | 64*q; an empty mask gives all ones, which is huge as an
    // unsigned number, so the unsigned minimum over the slots is the answer (-1 when all are empty)
    unsigned best = 0xffffffffu;
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      int L;
      asm("s_ff1_i32_b64 %0, %1" : "=s"(L) : "s"(e[q]));   // -1 for an empty mask
      const unsigned cand = static_cast<unsigned>(L) | static_cast<unsigned>(64 * q);
      best = cand < best ? cand : best;
    }
    return static_cast<int>(best);
  }
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

// Scales one 32x32 tile of raw dot products to cosines and writes it into the packed
// triangle (element (i,j), j <= i, at i(i+1)/2 + j).  The diagonal entry holds +inf: reading
// the row of a pick drives the pick's own m to +inf and its gain to -inf, which is how a
// selected token leaves the race.
__device__ __forceinline__ void write_cos_tile(float* tri, const float* rinv, const f32x16& acc,
                                               int I, int J, int lane) {
  const int hf = lane >> 5;
  const int j = J * 32 + (lane & 31);
  const float rc = rinv[j];
  int i = I * 32 + hf * 4;                            // first of this lane's rows in the tile
  int off = i * (i + 1) / 2 + j;
  float4 rr4[4];                                      // the rows' inverse norms, all requested before the first use
#pragma unroll
  for (int R = 0; R < 4; ++R) rr4[R] = *reinterpret_cast<const float4*>(rinv + i + 8 * R);
  if (I != J) {                                       // two code paths: no per-element predicate off the diagonal
#pragma unroll
    for (int R = 0; R < 4; ++R) {
      const float rrow[4] = {rr4[R].x, rr4[R].y, rr4[R].z, rr4[R].w};
      int o = off;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        tri[o] = acc[R * 4 + q] * rrow[q] * rc;
        o += i + q + 1;
      }
      off += 8 * i + 36;                              // T(i+8) - T(i)
      i += 8;
    }
  } else {
#pragma unroll
    for (int R = 0; R < 4; ++R) {
      const float rrow[4] = {rr4[R].x, rr4[R].y, rr4[R].z, rr4[R].w};
      int o = off;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float c = j == i + q ? INFINITY : acc[R * 4 + q] * rrow[q] * rc;
        if (j <= i + q) tri[o] = c;
        o += i + q + 1;
      }
      off += 8 * i + 36;
      i += 8;
    }
  }
}

// Algorithm 1's pick chain (Eq. 2-3) on one wave, for a head whose cosines sit in the packed
// triangle `tri` (element (i,j), j <= i, at i(i+1)/2 + j, +inf on the diagonal) and whose scores
// sit in s_l (-inf for padding).  A single wave issues one instruction every few cycles, so the
// time of a pick is its instruction count: tokens lane, lane + 64, .. live in lane `lane` (see
// first_of_slots); pick u of a
// 64-pick chunk is parked in lane u of two registers (v_writelane) and the chunk is written to
// order_l / gain_l once; nothing is checked per pick.  Non-finite input is detected afterwards
// from the logged gains: the picks before the first one without a finite gain are kept and the
// list is filled up with the lowest tokens < n_live not yet in it.  `diverse` false is the
// lambda = 0 branch (top-b, the triangle is not read).  Returns the gain of the last pick.
template <int NQ, bool DIVERSE>
__device__ __forceinline__ float pick_chain_impl(const float* s_l, const float* tri, int32_t* order_l, float* gain_l,
                                                 int n_live, int b, float lambda, int lane) {
  typedef __attribute__((address_space(3))) const float* lds_fp;
  const int tri0 = static_cast<int>(reinterpret_cast<uintptr_t>(
      (__attribute__((address_space(3))) const char*)reinterpret_cast<const char*>(tri)));
  float sreg[NQ], mreg[NQ];
  int ja[NQ], tja[NQ];
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int j = lane + 64 * q;
    sreg[q] = s_l[j];
    mreg[q] = 0.f;
    ja[q] = j * 4 + tri0;                              // column offset of the token
    tja[q] = j * (j + 1) * 2 + tri0;                   // start of its row
  }
  const float nlam = -lambda;
  int bad_t = b;                                       // first pick without a finite gain
  float last_g = -INFINITY;
  for (int c0 = 0; c0 < b; c0 += 64) {
    const int cnt = __builtin_amdgcn_readfirstlane(b - c0 < 64 ? b - c0 : 64);
    int rec_i = 0, rec_g = 0;
    for (int u = 0; u < cnt; ++u) {
      float av[NQ];
#pragma unroll
      for (int q = 0; q < NQ; ++q) av[q] = fmaf(nlam, mreg[q], sreg[q]);
      float best = av[0];
#pragma unroll
      for (int q = 1; q < NQ; ++q) best = hw_max(best, av[q]);
      const float amax = wave_max_uniform(best);
      unsigned long long e[NQ];
#pragma unroll
      for (int q = 0; q < NQ; ++q) e[q] = __ballot(av[q] == amax);
      const int i = first_of_slots<NQ>(e);             // negative when nothing compares equal (NaN)
      write_lane2(rec_i, rec_g, i, __float_as_int(amax), u);
      if constexpr (DIVERSE) {
        // element (i,j) sits at max(T(i)+j, T(j)+i); the diagonal entry (+inf) retires the pick.
        // For any i in [-1, 64*NQ) both addresses stay inside the triangle.
        const int ti4 = i * (i + 1) * 2, i4 = i * 4;
        float c[NQ];
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
          const int a0 = ti4 + ja[q], a1 = tja[q] + i4;
          c[q] = *reinterpret_cast<lds_fp>(static_cast<uintptr_t>(static_cast<unsigned>(a0 > a1 ? a0 : a1)));
        }
#pragma unroll
        for (int q = 0; q < NQ; ++q) mreg[q] = hw_max(mreg[q], c[q]);
      } else {
#pragma unroll
        for (int q = 0; q < NQ; ++q) sreg[q] = (lane + 64 * q == i) ? -INFINITY : sreg[q];
      }
    }
    const float g = __int_as_float(rec_g);
    if (lane < cnt) { order_l[c0 + lane] = rec_i; gain_l[c0 + lane] = g; }
    last_g = __int_as_float(__builtin_amdgcn_readlane(rec_g, cnt - 1));
    const unsigned long long bad = __ballot(lane < cnt && !(g > -INFINITY));
    if (bad && bad_t == b) bad_t = c0 + __ffsll(static_cast<long long>(bad)) - 1;
  }
  if (bad_t < b) {
    wave_lds_sync();
    for (int t = bad_t; t < b; ++t) {
      int i = -1;
#pragma unroll
      for (int q = NQ - 1; q >= 0; --q) {
        const int j = lane + 64 * q;
        bool free_tok = j < n_live;
        for (int u = 0; u < t; ++u) free_tok = free_tok && order_l[u] != j;
        const unsigned long long al = __ballot(free_tok);
        if (al) i = (__ffsll(static_cast<long long>(al)) - 1) + 64 * q;
      }
      if (lane == 0) { order_l[t] = i; gain_l[t] = -INFINITY; }
      wave_lds_sync();
    }
    last_g = -INFINITY;
  }
  return last_g;
}

template <int NQ>
__device__ __forceinline__ float pick_chain(const float* s_l, const float* tri, int32_t* order_l, float* gain_l,
                                            int n_live, int b, float lambda, bool diverse, int lane) {
  return diverse ? pick_chain_impl<NQ, true>(s_l, tri, order_l, gain_l, n_live, b, lambda, lane)
                 : pick_chain_impl<NQ, false>(s_l, tri, order_l, gain_l, n_live, b, lambda, lane);
}

// sort(S) on one wave: flags the b picks of order_l (indices < 64*NQ), writes them in ascending
// order to idx_l by prefix popcounts.  With a map (ascending in its argument), idx_l and
// order_l are translated through it.  `flag` is scratch for 64*NQ ints.
template <int NQ>
__device__ __forceinline__ void sort_picks(int32_t* order_l, int32_t* idx_l, int32_t* flag, int b, int lane,
                                           const int32_t* map) {
#pragma unroll
  for (int q = 0; q < NQ; ++q) flag[lane + 64 * q] = 0;
  wave_lds_sync();                                     // order_l was written by other lanes
  for (int u = lane; u < b; u += kWave) flag[min(max(order_l[u], 0), 64 * NQ - 1)] = 1;
  wave_lds_sync();                                     // flags are set by other lanes
  int off = 0;
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int j = lane + 64 * q;
    const bool picked = flag[j] != 0;
    const unsigned long long sel = __ballot(picked);
    if (picked) idx_l[off + __popcll(sel & ((1ull << lane) - 1ull))] = map ? map[j] : j;
    off += __popcll(sel);
  }
  if (map)
    for (int u = lane; u < b; u += kWave) order_l[u] = map[min(max(order_l[u], 0), 64 * NQ - 1)];
}

// Cache update for one head: rows il[t], t < b, of K and V go to rows ob + t of the dense
// outputs, bit for bit, by the nthr threads t0 = 0..nthr-1 (nthr a multiple of 16; 16 threads
// per row).  BATCH rows per thread are loaded by straight-line code before the first store (row
// numbers past b are clamped rather than branched around): with branches between them the
// compiler loses count of what is in flight and waits for everything, acknowledged stores
// included, before each store.  Indices are clamped into [0, n) so that nothing is read
// outside the head whatever the scores were.
template <int BATCH>
__device__ __forceinline__ void compact_rows(const char* K, const char* V, char* K_out, char* V_out,
                                             long long head_off_bytes, long long stride_tok,
                                             const int32_t* il, int n, int b, long long ob, int t0, int nthr) {
  const int chunk = t0 & 15, g = t0 >> 4, G = nthr >> 4;
  const long long base = head_off_bytes + chunk * 16;
  for (int first = 0; first < b; first += BATCH * G) {
    uint4 kr[BATCH], vr[BATCH];
    if (K_out && V_out) {
#pragma unroll
      for (int k = 0; k < BATCH; ++k) {
        const int t = min(first + g + k * G, b - 1);
        const long long src = base + min(max(kvr_ix(il[t], n, KVR_BOUNDS_FILE * 100 + 90), 0), n - 1) * stride_tok * 2;   // (x90: kept token)
        kr[k] = *reinterpret_cast<const uint4*>(K + src);
        vr[k] = *reinterpret_cast<const uint4*>(V + src);
      }
    } else {
#pragma unroll
      for (int k = 0; k < BATCH; ++k) {
        const int t = min(first + g + k * G, b - 1);
        const long long src = base + min(max(kvr_ix(il[t], n, KVR_BOUNDS_FILE * 100 + 90), 0), n - 1) * stride_tok * 2;   // (x90: kept token)
        kr[k] = vr[k] = make_uint4(0u, 0u, 0u, 0u);
        if (K_out) kr[k] = *reinterpret_cast<const uint4*>(K + src);
        if (V_out) vr[k] = *reinterpret_cast<const uint4*>(V + src);
      }
    }
#pragma unroll
    for (int k = 0; k < BATCH; ++k) {
      const int t = first + g + k * G;
      if (t < b) {
        const long long dst = ((ob + t) * kD + chunk * 8) * 2;
        if (K_out) *reinterpret_cast<uint4*>(K_out + dst) = kr[k];
        if (V_out) *reinterpret_cast<uint4*>(V_out + dst) = vr[k];
      }
    }
  }
}

// One head's [n,128] bf16 rows: coalesced 16-byte loads into registers (rows beyond n read
// as zero, so MFMA fragments of padded blocks are zero), then into the padded LDS stage.
template <int NT>
__device__ __forceinline__ void load_rows(const char* __restrict__ src, long long stride_tok, int n,
                                          int tid, uint4 (&reg)[NT * 32 * 16 / kDenseThreads]) {
  constexpr int kIters = NT * 32 * 16 / kDenseThreads;
  const int chunk = tid & 15, r0 = tid >> 4;
#pragma unroll
  for (int k = 0; k < kIters; ++k) {
    const int row = r0 + 16 * k;
    reg[k] = make_uint4(0u, 0u, 0u, 0u);
    if (row < n) reg[k] = *reinterpret_cast<const uint4*>(src + (row * stride_tok + chunk * 8) * 2);
  }
}
template <int NT>
__device__ __forceinline__ void store_rows(char* stage, int tid,
                                           const uint4 (&reg)[NT * 32 * 16 / kDenseThreads]) {
  constexpr int kIters = NT * 32 * 16 / kDenseThreads;
  const int chunk = tid & 15, r0 = tid >> 4;
#pragma unroll
  for (int k = 0; k < kIters; ++k)
    *reinterpret_cast<uint4*>(stage + (r0 + 16 * k) * kRowPitch + chunk * 16) = reg[k];
}

__device__ __forceinline__ bf16x8 frag_at(const char* stage, int block, int ks, int lane) {
  const int row = block * 32 + (lane & 31), hf = lane >> 5;
  return *reinterpret_cast<const bf16x8*>(stage + row * kRowPitch + ks * 32 + hf * 16);
}

}  // namespace kvr
