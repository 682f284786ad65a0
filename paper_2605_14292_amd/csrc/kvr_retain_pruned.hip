// Fused retention step for bf16 heads with 128 < n <= 256 tokens whose scores are
// given, after an exact reduction of the candidate set.
//
// Reduction.  Let s_(b) be the b-th largest score of the head.  While fewer than
// b tokens are selected, one of the b best-scored tokens is still unselected, and
// its marginal gain s_i - lambda * max(0, max cos) (paper Eq. 2) is at least
// s_(b) - lambda because a cosine never exceeds 1.  The greedy argmax (Eq. 3)
// therefore never falls on a token with s_j < s_(b) - lambda: its gain is at most
// s_j.  Such tokens are dropped before anything of V is read; the survivors keep
// their token order, so "lowest index wins a tie" is unchanged, and Algorithm 1
// runs on them exactly as it would on the whole head.  A small safety margin
// covers the rounding of the fp32 cosines (which can exceed 1 by a few ulp).
//
// When at most 128 tokens survive, the head needs a 128-token cosine triangle
// (33 KB of LDS) instead of a 192- or 256-token one, and four workgroups instead
// of two or one share a CU, which is what bounds the throughput of the b
// dependent picks.  Heads with more survivors are marked (idx_sorted[h*b] = -1)
// and left to the full-size kernel, which runs afterwards on marked heads only.
//
// Waves are specialised: wave 0 runs the pick chain of head h while waves 1-3
// find the survivors of the workgroup's next head and start its row gather.
#include "kvr_dense_common.hpp"
#include "kvr_kernels.hpp"

namespace kvr {

constexpr int kPrN = 128;                    // survivors a workgroup can hold
constexpr int kPrLoaders = 192;              // threads of waves 1-3
constexpr int kPrRowsPerIter = kPrLoaders / 16;
constexpr int kPrIters = (kPrN + kPrRowsPerIter - 1) / kPrRowsPerIter;

struct PrunedArgs {
  const char* K; const char* V; const float* s;
  int32_t* idx_sorted; int32_t* pick_order; float* pick_gain;
  char* K_out; char* V_out;
  long long stride_head, stride_tok;         // elements
  int n, b, heads;
  float lambda, eps;
  const int32_t* b_h;                        // per-head budgets <= b (output rows stay b apart), or null
};

constexpr int pruned_region_a() { return dense_region_a(4); }
constexpr int pruned_smem_bytes() {
  // region A | s_c[2][128] | tok_c[2][128] | rinv[128] | idx_l[2][128] | order_l[2][128] | gain_l[2][128] | meta[16: head, survivors, best left-out score, redo flag, picks to run, budget; two of each]
  return pruned_region_a() + 2 * kPrN * 4 * 2 + kPrN * 4 + 2 * kPrN * 4 * 3 + 64;
}

__global__ __launch_bounds__(kDenseThreads, 4) void retain_pruned_kernel(PrunedArgs a) {
  extern __shared__ __align__(16) char smem[];
  char* stage = smem;                                 // gathered rows ...
  float* tri = reinterpret_cast<float*>(smem);        // ... later the packed cosine triangle
  float* s_c = reinterpret_cast<float*>(smem + pruned_region_a());   // [2][128] survivor scores
  int32_t* tok_c = reinterpret_cast<int32_t*>(s_c + 2 * kPrN);       // [2][128] survivor tokens
  float* rinv = reinterpret_cast<float*>(tok_c + 2 * kPrN);
  int32_t* idx_l2 = reinterpret_cast<int32_t*>(rinv + kPrN);          // [2][128] each: the lists of head h
  int32_t* order_l2 = idx_l2 + 2 * kPrN;                             // are written out while head h+1 is
  float* gain_l2 = reinterpret_cast<float*>(order_l2 + 2 * kPrN);     // in its pick chain
  int32_t* meta = reinterpret_cast<int32_t*>(gain_l2 + 2 * kPrN);         // [buf] head, [2+buf] survivors

  const int tid0 = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid0 >> 6);
  const int n = a.n, b = a.b;

  uint4 vpre[kPrIters];                               // gathered rows of the head in preparation (waves 1-3)

  // Waves 1-3, each on its own: survivors of the first head hh, hh + gridDim.x, ... that
  // fits, then the gather of their V rows into registers.  The three waves compute the same
  // survivor list (each needs it for its share of the rows); wave 1 publishes it.
  float s_pre[4];                                     // scores of head s_pre_h, fetched ahead of time
  int s_pre_h = -1;
  auto load_scores = [&](int hh, int lane, float (&dst)[4]) {
    const float* sp = a.s + static_cast<long long>(hh) * n;
#pragma unroll
    for (int q = 0; q < 4; ++q) dst[q] = lane + 64 * q < n ? sp[lane + 64 * q] : -INFINITY;
  };
  auto survivors = [&](int hh, int buf, int tid, int& ns_out) -> int {
    const int lane = tid & 63;
    float sv[4];
    unsigned long long keep[4];
    int ns = 0;
    int bq = b, bt = b;                               // budget of the head: its picks are the first bq of a run for b
    float excl = -INFINITY;                           // best score among the candidates left out
    for (; hh < a.heads; hh += gridDim.x) {
      if (hh == s_pre_h) {
#pragma unroll
        for (int q = 0; q < 4; ++q) sv[q] = s_pre[q];
      } else {
        load_scores(hh, lane, sv);
      }
      bt = a.b_h ? __builtin_amdgcn_readfirstlane(min(max(a.b_h[hh], 0), b)) : b;
      bq = bt < 1 ? 1 : bt;                          // a head with budget 0 still runs one pick; nothing of it is written
      uint32_t key[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) key[q] = lane + 64 * q < n ? ordered_key(sv[q] + 0.0f) : 0u;
      // Bit-wise search for the b-th largest key, leading 16 bits only: the result is at most
      // s_(b), so the bound below stays valid and is looser by less than one part in 128.
      uint32_t T = 0;
      for (int bit = 31; bit >= 16; --bit) {
        const uint32_t cand = T | (1u << bit);
        int cnt = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) cnt += __popcll(__ballot(key[q] >= cand));
        if (cnt >= bq) T = cand;
      }
      const float sb = key_to_float(T);
      const float thr = sb - a.lambda * 1.00001f - 1e-5f * fabsf(sb);
      ns = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        keep[q] = __ballot(lane + 64 * q < n && !(sv[q] < thr));
        ns += __popcll(keep[q]);
      }
      excl = -INFINITY;
      if (ns <= kPrN) break;
      // More candidates than fit: keep the best-scored kPrN of them (fewer when scores tie at
      // the cut) and remember the best score left out; the pick chain is then valid if that
      // score stays below the gain of every pick, which is checked once the chain is done.
      uint32_t T2 = 0;
      for (int bit = 31; bit >= 0; --bit) {
        const uint32_t cand = T2 | (1u << bit);
        int cnt = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) cnt += __popcll(__ballot(key[q] >= cand));
        if (cnt >= kPrN) T2 = cand;
      }
      int cnt_ge = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) cnt_ge += __popcll(__ballot(key[q] >= T2));
      const uint32_t cut = cnt_ge == kPrN ? T2 : T2 + 1u;   // T2 < 0xffffffff here: kPrN < n tokens reach it
      ns = 0;
      float out_best = -INFINITY;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const bool valid = lane + 64 * q < n;
        keep[q] = __ballot(valid && key[q] >= cut);
        ns += __popcll(keep[q]);
        if (valid && key[q] < cut) out_best = fmaxf(out_best, sv[q]);
      }
      excl = wave_max_uniform(out_best);
      // The cut can only be verified if the last pick's gain stays above the best score left out.
      // That gain is at most s_(b) and in practice a good part of lambda below it (the later picks
      // of a head carry a penalty), so when the score left out is within a quarter of lambda of
      // s_(b) the chain would be run in vain and then run again by the full-size kernel: such a
      // head goes there at once.  (A guess about speed only: either way the picks are exact.)
      const bool hopeless = !(excl < sb - 0.25f * a.lambda);
      if (ns >= bq && ns <= kPrN && !hopeless) break;
      if (wave == 1 && lane == 0) a.idx_sorted[static_cast<long long>(hh) * b] = -1;
    }
    if (hh < a.heads) {
      float* sc = s_c + buf * kPrN;
      int32_t* tc = tok_c + buf * kPrN;
      int base = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if ((keep[q] >> lane) & 1ull) {
          const int c = base + __popcll(keep[q] & ((1ull << lane) - 1ull));
          tc[c] = lane + 64 * q;                      // the same value from each of the three waves
          if (wave == 1) sc[c] = sv[q];
        }
        base += __popcll(keep[q]);
      }
      if (wave == 1)
        for (int c = ns + lane; c < kPrN; c += kWave) sc[c] = -INFINITY;   // padding never competes
    }
    if (wave == 1 && lane == 0) {
      meta[buf] = hh < a.heads ? hh : a.heads;
      meta[2 + buf] = ns;
      meta[4 + buf] = __float_as_int(excl);
      meta[8 + buf] = bq;
      meta[10 + buf] = bt;
    }
    s_pre_h = hh < a.heads ? hh + static_cast<int>(gridDim.x) : -1;
    if (s_pre_h >= 0 && s_pre_h < a.heads) load_scores(s_pre_h, lane, s_pre);
    ns_out = ns;
    return hh;
  };
  // Rows of the survivors of head hh (list in buffer buf) into registers.
  auto gather = [&](int hh, int buf, int ns, int tid) {
#pragma unroll
    for (int k = 0; k < kPrIters; ++k) vpre[k] = make_uint4(0u, 0u, 0u, 0u);   // rows past the survivors read as zero
    if (hh < a.heads) {
      const int32_t* tc = tok_c + buf * kPrN;
      wave_lds_sync();                                // tc[] was written by this wave's own lanes
      const int tl = tid - kWave, r0 = tl >> 4, chunk = tl & 15;
      const char* vb = a.V + hh * a.stride_head * 2 + chunk * 16;
#pragma unroll
      for (int k = 0; k < kPrIters; ++k) {
        const int c = r0 + kPrRowsPerIter * k;
        if (c < ns) vpre[k] = *reinterpret_cast<const uint4*>(vb + tc[c] * a.stride_tok * 2);
      }
    }
  };

  // Inverse norms 1/(||V_c|| + eps) of the gathered rows (Eq. 1): eight elements per lane, the
  // sixteen lanes of a row form one DPP row whose last lane ends up with the total.  Runs while
  // wave 0 is still in its chain, once the rows have landed.
  float rn[kPrIters];
  auto norms = [&]() {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
#pragma unroll
    for (int k = 0; k < kPrIters; ++k) {
      const uint32_t wds[4] = {vpre[k].x, vpre[k].y, vpre[k].z, vpre[k].w};
      float ss = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bf16x2 x = __builtin_bit_cast(bf16x2, wds[e]);
        ss = __builtin_amdgcn_fdot2_f32_bf16(x, x, ss, false);
      }
      KVR_DPP_ADD(ss, 0x111, 0xf) KVR_DPP_ADD(ss, 0x112, 0xf) KVR_DPP_ADD(ss, 0x114, 0xf)
      KVR_DPP_ADD(ss, 0x118, 0xf)
      rn[k] = 1.0f / (sqrtf(ss) + a.eps);
      __builtin_amdgcn_sched_barrier(0);              // one row at a time: no registers for eleven in flight
    }
  };

  // Results of head hh (lists in buffer lb) to HBM and the compaction of its kept rows, by the
  // nthr threads t0 = 0..nthr-1 (nthr a multiple of 16).  Rows move in batches of kOutBatch per
  // 16-thread group.  The loads of a batch are straight-line code (row indices past b are
  // clamped, not branched around): with branches in between the compiler loses count of what is
  // in flight and waits for everything, acknowledged stores included, before each store.
  constexpr int kOutBatch = 6;
  auto out_lists = [&](int hh, int lb, int t0, int nthr, int bq) {
    const long long ob = static_cast<long long>(hh) * b;
    const bool redo = meta[6 + lb] != 0;                 // the head is left to the full-size kernel
    for (int t = t0; t < b; t += nthr) {                 // entries past the head's budget are padding
      a.idx_sorted[ob + t] = ((redo && t == 0) || t >= bq) ? -1 : idx_l2[lb * kPrN + t];
      if (a.pick_order) a.pick_order[ob + t] = t < bq ? order_l2[lb * kPrN + t] : -1;
      if (a.pick_gain) a.pick_gain[ob + t] = t < bq ? gain_l2[lb * kPrN + t] : -INFINITY;
    }
  };
  uint4 kr[kOutBatch], vr[kOutBatch];
  const bool copy_both = a.K_out && a.V_out;
  auto out_load = [&](int hh, int lb, int t0, int nthr, int first, int bq) {
    const int32_t* il = idx_l2 + lb * kPrN;
    const long long head_off = hh * a.stride_head * 2 + (t0 & 15) * 16;   // bytes
    if (copy_both) {
#pragma unroll
      for (int k = 0; k < kOutBatch; ++k) {
        const int t = min(first + (t0 >> 4) + k * (nthr >> 4), bq - 1);
        const int it = min(max(il[t], 0), n - 1);        // never read outside the head, whatever the scores were
        const long long src = head_off + it * a.stride_tok * 2;
        kr[k] = *reinterpret_cast<const uint4*>(a.K + src);
        vr[k] = *reinterpret_cast<const uint4*>(a.V + src);
      }
    } else {
#pragma unroll
      for (int k = 0; k < kOutBatch; ++k) {
        const int t = min(first + (t0 >> 4) + k * (nthr >> 4), bq - 1);
        const int it = min(max(il[t], 0), n - 1);
        const long long src = head_off + it * a.stride_tok * 2;
        kr[k] = vr[k] = make_uint4(0u, 0u, 0u, 0u);
        if (a.K_out) kr[k] = *reinterpret_cast<const uint4*>(a.K + src);
        if (a.V_out) vr[k] = *reinterpret_cast<const uint4*>(a.V + src);
      }
    }
  };
  auto out_store = [&](int hh, int t0, int nthr, int first, int bq) {
    const long long ob = static_cast<long long>(hh) * b;
#pragma unroll
    for (int k = 0; k < kOutBatch; ++k) {
      const int t = first + (t0 >> 4) + k * (nthr >> 4);
      if (t < bq) {
        const long long dst = ((ob + t) * kD + (t0 & 15) * 8) * 2;
        if (a.K_out) *reinterpret_cast<uint4*>(a.K_out + dst) = kr[k];
        if (a.V_out) *reinterpret_cast<uint4*>(a.V_out + dst) = vr[k];
      }
    }
  };

  int buf = 0;
  int hprev = -1;                                     // head whose results are still in LDS
  int bprev = b;                                      // and its budget
  if (wave != 0) {
    int ns0;
    const int h0 = survivors(blockIdx.x, 0, tid0, ns0);
    gather(h0, 0, ns0, tid0);
    norms();
  }
  lds_barrier();
  int h = __builtin_amdgcn_readfirstlane(meta[0]);
  while (h < a.heads) {
    // The thread index is made opaque once per head so that per-lane LDS addresses are not
    // hoisted out of the head loop into registers.
    int tid = tid0;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, hf = lane >> 5;
    const int ns = __builtin_amdgcn_readfirstlane(meta[2 + buf]);
    const int bh = __builtin_amdgcn_readfirstlane(meta[8 + buf]);
    const int bout = __builtin_amdgcn_readfirstlane(meta[10 + buf]);
    const float* s_cur = s_c + buf * kPrN;
    const int32_t* tok_cur = tok_c + buf * kPrN;
    int32_t* idx_l = idx_l2 + buf * kPrN;
    int32_t* order_l = order_l2 + buf * kPrN;
    float* gain_l = gain_l2 + buf * kPrN;

    if (wave != 0) {
      const int tl = tid - kWave, r0 = tl >> 4, chunk = tl & 15;
#pragma unroll
      for (int k = 0; k < kPrIters; ++k) {
        const int c = r0 + kPrRowsPerIter * k;
        if (c < kPrN) {
          *reinterpret_cast<uint4*>(stage + c * kRowPitch + chunk * 16) = vpre[k];
          if (chunk == 15) rinv[c] = rn[k];
        }
      }
    }
    lds_barrier();

    // ------------------------------------------------ Gram -> packed cosines
    // Ten lower-triangular 32x32 tiles over four waves; tile rows that hold no survivor are
    // skipped.  wave 0: (3,3) (0,0); wave 1: (3,0..2); wave 2: (2,0..2); wave 3: (1,0..1).
    f32x16 acc[3];
    const int nblk = (ns + 31) >> 5;                  // token blocks in use
    const int rowI = wave == 0 ? 3 : 4 - wave;
    const int ntile = (wave == 0 || wave == 3) ? 2 : 3;
    auto tile_of = [&](int sl, int& I, int& J) -> bool {
      if (wave == 0) { I = sl == 0 ? 3 : 0; J = I; }
      else { I = rowI; J = sl; }
      return sl < ntile && I < nblk;
    };
#pragma unroll
    for (int sl = 0; sl < 3; ++sl) {
      int I, J;
      acc[sl] = f32x16{0};
      if (tile_of(sl, I, J)) {
        // both fragments come from LDS at every k-step: with four workgroups on a CU there are
        // no registers to keep a row block resident
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
          acc[sl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_at(stage, I, ks, lane),
                                                            frag_at(stage, J, ks, lane), acc[sl], 0, 0, 0);
      }
    }
    lds_barrier();                                  // gathered rows are dead from here on
#pragma unroll
    for (int sl = 0; sl < 3; ++sl) {
      int I, J;
      if (tile_of(sl, I, J)) write_cos_tile(tri, rinv, acc[sl], I, J, lane);
    }
    lds_barrier();

    if (wave != 0) {
      // the previous head's kept rows start their trip first, the next head's survivor search
      // runs while they are in flight
      const int tl = tid - kWave;
      constexpr int kStep = kOutBatch * (kPrLoaders / 16);
#pragma unroll
      for (int k = 0; k < kOutBatch; ++k) {            // nothing of the previous head's rows is carried over
        kr[k] = vr[k] = make_uint4(0u, 0u, 0u, 0u);
      }
      if (hprev >= 0) out_load(hprev, buf ^ 1, tl, kPrLoaders, 0, bprev);
      int ns_n;
      const int h_n = survivors(h + gridDim.x, buf ^ 1, tid, ns_n);
      gather(h_n, buf ^ 1, ns_n, tid);   // in flight from here to the end of wave 0's chain
      if (hprev >= 0) {
        out_lists(hprev, buf ^ 1, tl, kPrLoaders, bprev);
        out_store(hprev, tl, kPrLoaders, 0, bprev);
        for (int first = kStep; first < bprev; first += kStep) {
          out_load(hprev, buf ^ 1, tl, kPrLoaders, first, bprev);
          out_store(hprev, tl, kPrLoaders, first, bprev);
        }
      }
      norms();
    } else {
      // ---------------------------------------------------------------- greedy
      __builtin_amdgcn_s_setprio(3);                   // the chain goes first when it shares a SIMD with loader waves
      const float last_g = pick_chain<2>(s_cur, tri, order_l, gain_l, ns, bh, a.lambda, true, lane);
      __builtin_amdgcn_s_setprio(0);
      {
        // Candidates that were left out for lack of room must lie below every pick's gain (the
        // last pick's is the smallest); otherwise the head goes to the full-size kernel.
        const float excl = __int_as_float(meta[4 + buf]);
        const bool ok = excl < last_g - 1e-5f * (fabsf(last_g) + a.lambda);
        if (lane == 0) meta[6 + buf] = (ok || excl == -INFINITY) ? 0 : 1;
      }
      // back to token indices: the survivor list is ascending in the token index
      sort_picks<2>(order_l, idx_l, reinterpret_cast<int32_t*>(rinv), bh, lane, tok_cur);
      // Wave 0 never holds gathered rows.  Saying so (no instruction is emitted) keeps the row
      // registers of the other branch from being carried, as far as the compiler can tell,
      // through this branch and with it through the whole loop body.
#pragma unroll
      for (int k = 0; k < kPrIters; ++k) {
        asm volatile("" : "=v"(vpre[k].x), "=v"(vpre[k].y), "=v"(vpre[k].z), "=v"(vpre[k].w), "=v"(rn[k]));
      }
    }
    lds_barrier();

    hprev = h;
    bprev = bout;
    h = __builtin_amdgcn_readfirstlane(meta[buf ^ 1]);   // published before the barrier above
    buf ^= 1;
  }
  if (hprev >= 0) {
    constexpr int kStep = kOutBatch * (kDenseThreads / 16);
    out_lists(hprev, buf ^ 1, tid0, kDenseThreads, bprev);
    for (int first = 0; first < bprev; first += kStep) {
      out_load(hprev, buf ^ 1, tid0, kDenseThreads, first, bprev);
      out_store(hprev, tid0, kDenseThreads, first, bprev);
    }
  }
}

bool pruned_supported(const Layout& lay, int b, float lambda, bool has_q) {
  return lay.dtype == DT_BF16 && !has_q && lay.n > kPrN && lay.n <= 256 && b > 1 && b <= kPrN &&
         lambda > 0.0f;
}

hipError_t launch_retain_pruned(const void* K, const void* V, const float* s, const Layout& lay, int b,
                                float lambda, float eps, int32_t* idx_sorted, int32_t* pick_order,
                                float* pick_gain, void* K_out, void* V_out, hipStream_t st, const int32_t* b_h) {
  PrunedArgs a;
  a.b_h = b_h;
  a.K = static_cast<const char*>(K); a.V = static_cast<const char*>(V); a.s = s;
  a.idx_sorted = idx_sorted; a.pick_order = pick_order; a.pick_gain = pick_gain;
  a.K_out = static_cast<char*>(K_out); a.V_out = static_cast<char*>(V_out);
  a.stride_head = lay.stride_head; a.stride_tok = lay.stride_tok;
  a.n = lay.n; a.b = b; a.heads = lay.heads; a.lambda = lambda; a.eps = eps;
  const int cus = cu_count();
  constexpr int smem = pruned_smem_bytes();
  static_assert(4 * smem <= 160 * 1024, "four workgroups must share a CU's LDS");
  const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&retain_pruned_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  if (e != hipSuccess) return e;
  const int blocks = lay.heads < cus * 4 ? lay.heads : cus * 4;
  hipLaunchKernelGGL(retain_pruned_kernel, dim3(blocks), dim3(kDenseThreads), smem, st, a);
  return hipGetLastError();
}

}  // namespace kvr
