/*
 * kvr -- per-compression-event KV retention step of the alpha selector on one
 * MI355X (gfx950).  C ABI; every pointer below marked "device" is HIP device
 * memory owned by the caller, everything else is a plain host value.
 *
 * One "head" is one independent selection problem: the n cached tokens of one
 * (sequence, layer, KV-head), with that head's own K rows, V rows and base
 * scores.  The library runs all `heads` problems of a call in one launch
 * sequence on the caller's stream.
 *
 * The method (paper Sec. 4.1 "Method: A V-Space Diversity Penalty"):
 *   - V-signature  v_i = V_i / (||V_i||_2 + eps)                    (Eq. 1,
 *     one layer and one head per problem)
 *   - marginal gain  s_i - lambda * max(0, max_{j in S} v_i . v_j)  (Eq. 2)
 *   - greedy fill: first pick argmax s, then argmax of the marginal gain over
 *     unselected tokens, b-1 times                                  (Eq. 3,
 *     Algorithm 1; b is the paper's k)
 *   - lambda == 0 returns top-b(s) through an explicit branch that never
 *     touches V                                                     (Alg. 1)
 *   - the cache keeps the selected rows in ascending token order    (Alg. 1
 *     returns sort(S); Sec. 1)
 * Every argmax breaks ties towards the lowest token index.
 *
 * Common rules
 *   - Calls enqueue work on `stream` (a hipStream_t passed as void*, NULL =
 *     the default stream) and return without synchronising (the kvr_debug_*
 *     calls say where they differ).
 *   - Inputs are read-only; outputs must not alias inputs or each other,
 *     except where a call says otherwise (kvr_compact_inplace, kvr_score_prior).
 *   - The library allocates no device memory (kvr_retain_budgeted_static
 *     brings a static device array along instead).  `workspace` is reserved for
 *     future kernels: every entry point
 *     accepts NULL / 0 as long as kvr_workspace_bytes() reports 0 for the
 *     same arguments.
 *   - Return value: KVR_OK or a negative kvr_status.  Argument errors are
 *     detected on the host before anything is launched.  Non-finite scores or
 *     rows give unspecified picks (but never out-of-range indices).
 *   - Device pointers must be 16-byte aligned; d must be 128: every kernel
 *     maps the 256 bytes of a bf16 row (512 of an fp32 row) onto fixed lane
 *     groups and MFMA k-steps, and 128 is the head dimension of every model
 *     the paper evaluates and of every benchmark configuration; another d is
 *     KVR_ERR_UNSUPPORTED, never a wrong result.  Strides are in elements,
 *     stride_tok >= d and a multiple of 8, stride_head >= n*stride_tok and a
 *     multiple of 8.
 *   - The library keeps no state between calls apart from the device's
 *     compute-unit count, read once.
 */
#ifndef KVR_H_
#define KVR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  KVR_OK = 0,
  KVR_ERR_ARG = -1,        /* NULL pointer, bad size, b<1, b>n, lambda<0/NaN, G<1, misaligned */
  KVR_ERR_UNSUPPORTED = -2,/* d != 128, unknown dtype, n or G above the limits below */
  KVR_ERR_WORKSPACE = -3,  /* workspace smaller than kvr_workspace_bytes() */
  KVR_ERR_HIP = -4,        /* a HIP launch or runtime call failed */
  KVR_ERR_NONFINITE = -5   /* kvr_debug_validate_finite found a NaN or an infinity */
} kvr_status;

typedef enum { KVR_F32 = 0, KVR_BF16 = 1 } kvr_dtype;

#define KVR_MAX_N 8192     /* candidates per head */
#define KVR_MAX_G 256      /* queries per KV head (observation window x grouped heads) */

/* Layout of a [heads, n, d] tensor of cached rows; d is contiguous. */
typedef struct {
  int32_t heads;           /* sequences * layers * kv_heads, flattened */
  int32_t n;               /* candidate tokens per head, 1..KVR_MAX_N */
  int32_t d;               /* head dimension (128) */
  int32_t dtype;           /* kvr_dtype of K, V, Q and of the compacted rows */
  int64_t stride_head;     /* elements between consecutive heads */
  int64_t stride_tok;      /* elements between consecutive tokens */
} kvr_layout;

int kvr_version(void);
const char* kvr_strerror(int status);

/* Debug aid for the builds of this library, not part of the paper's method.
 * The library can be built with bounds checks (-DKVR_BOUNDS, libkvr_bounds.so):
 * the kernels for heads of more than 256 tokens then pass every index they
 * compute from the data (pool slots, list positions, token indices read back
 * from tables, triangle addresses, kept tokens) through a range check that
 * records a failure and clamps the index instead of trapping.
 *   worst_id (host pointer, required): receives the largest id of a check that
 *     failed since the last call, 0 when none did.  The ids are listed in the
 *     kernels' sources (file number * 100 + site).  The product build has no
 *     checks and always stores 0.
 * Synchronises the device and clears the record.  Returns KVR_OK, KVR_ERR_ARG
 * for a NULL pointer, KVR_ERR_HIP when the record could not be read. */
int kvr_debug_bounds_violation(uint32_t* worst_id);

/* Shows that the record of kvr_debug_bounds_violation works: enqueues one
 * thread that passes the index 5 with the limit 3 through the range check
 * (id 199) without accessing memory through it, and stores the checked index
 * in out[0] (device pointer to one int32, required): 2 in the build with
 * bounds checks, whose next kvr_debug_bounds_violation then reports 199, and 5
 * in the product build.  Returns KVR_OK, KVR_ERR_ARG, KVR_ERR_HIP. */
int kvr_debug_bounds_selftest(int32_t* out, void* stream);

/* Optional validator of an event's inputs, for debugging: Algorithm 1 (Sec. 4.1)
 * is stated for finite scores and rows, and the selection calls promise only
 * distinct, in-range indices for anything else.  Scans K and V ([heads, n, d] in
 * `lay`; either may be NULL), Q ([heads, G, d] dense, of lay's dtype; NULL with
 * G = 0: none) and s ([heads, n] fp32; NULL: none) for NaN and +-inf.
 * Unlike every other call it synchronises `stream` (and reads one flag back).
 * Returns KVR_OK when every value is finite, KVR_ERR_NONFINITE otherwise;
 * KVR_ERR_ARG / KVR_ERR_UNSUPPORTED for a bad layout, misaligned pointers, all
 * four pointers NULL, or Q with G outside [1, KVR_MAX_G]; KVR_ERR_HIP. */
int kvr_debug_validate_finite(const void* K, const void* V, const void* Q, int G, const float* s,
                              const kvr_layout* lay, void* stream);

/* Bytes of caller-provided device workspace the calls below need for these
 * arguments (currently always 0).  Host-only; returns a kvr_status. */
int kvr_workspace_bytes(const kvr_layout* lay, int b, int G, size_t* bytes_out);

/*
 * Base scores, the stand-in for the paper's external scorer (Sec. 4.1 takes s
 * as given): s_i = (1/G) sum_g softmax_i(q_g . k_i / sqrt(d)), the softmax
 * taken over the n tokens of the head, no mask.
 *   K      device, [heads, n, d] per `lay`
 *   Q      device, dense [heads, G, d], same dtype as K
 *   s_out  device, dense float32 [heads, n]
 */
int kvr_score(const void* K, const void* Q, int G, const kvr_layout* lay,
              float* s_out, void* stream);

/*
 * Algorithm 1 for every head: greedy selection of b tokens under the V-space
 * redundancy penalty (Eq. 2-3); lambda == 0 is top-b of s and reads no V.
 *   V           device, [heads, n, d] per `lay` (may be NULL iff lambda == 0)
 *   s           device, dense float32 [heads, n]
 *   idx_sorted  device, int32 [heads, b], ascending token indices (sort(S))
 *   pick_order  device, int32 [heads, b] or NULL: picks in the order made
 *   pick_gain   device, float32 [heads, b] or NULL: marginal gain of each pick
 *               when it was made (pick_gain[0] = max s; with lambda == 0 the
 *               t-th largest score)
 */
int kvr_select_greedy(const void* V, const float* s, const kvr_layout* lay,
                      int b, float lambda, float eps,
                      int32_t* idx_sorted, int32_t* pick_order, float* pick_gain,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * Cache update (Sec. 1: the cache keeps a budget-bounded subset of its tokens;
 * Algorithm 1 returns sort(S), the rows kept, in token order):
 * K_out[h,t,:] = K[h, idx[h,t], :] and the same for V, copied bit for bit.
 * Either of K / V (with its output) may be NULL to skip it.
 *   idx           device, int32 [heads, b], every entry in [0, n)
 *   K_out, V_out  device, dense [heads, b, d], dtype of `lay`
 * An index outside [0, n) is clamped into range rather than read out of
 * bounds (the output row is then meaningless).
 */
int kvr_compact(const void* K, const void* V, const kvr_layout* lay,
                const int32_t* idx, int b, void* K_out, void* V_out, void* stream);

/*
 * The whole per-compression-event step of Sec. 4.1 in one call: base scores
 * (when Q is given; the paper's scorer is external, the stand-in is kvr_score's)
 * -> Algorithm 1 (Eq. 1-3) -> the cache update with sort(S).
 * Exactly one of (Q, G >= 1) and s_in must be provided:
 *   Q != NULL: scores are computed as in kvr_score; s_out (device, dense
 *              float32 [heads, n], required) receives them.
 *   Q == NULL: s_in (device, dense float32 [heads, n]) is used; G is ignored.
 * Outputs as in kvr_select_greedy and kvr_compact; pick_order and pick_gain
 * may be NULL.
 */
int kvr_retain(const void* K, const void* V, const void* Q, int G, const float* s_in,
               const kvr_layout* lay, int b, float lambda, float eps,
               float* s_out, int32_t* idx_sorted, int32_t* pick_order, float* pick_gain,
               void* K_out, void* V_out,
               void* workspace, size_t workspace_bytes, void* stream);

/*
 * Flat-signature mode: Eq. 1 as printed averages V over all layers and heads of
 * a sequence, u_i = (1/(L*H)) sum_{l,h} V_i^(l,h), v_i = u_i/(||u_i|| + eps);
 * one selection per sequence from one score vector, and every layer and head
 * of the sequence keeps the same token set (paper Sec. 4.1, Eq. 1-3; the
 * limitations paragraph names the per-head signature used by the calls above
 * as a variant).  In the [heads, n, d] tensors the L*H heads of a sequence are
 * `group` consecutive heads; heads must be a multiple of group.
 *
 * kvr_signature_flat: u_out[q, i, :] = mean over g < group of V[q*group + g, i, :]
 *   V      device, [heads, n, d] per `lay` (bf16 or fp32)
 *   u_out  device, dense float32 [heads/group, n, d]
 * The sum is taken in fp32.  To select on it, call kvr_select_greedy with a
 * KVR_F32 layout of heads/group dense heads and u_out as V.
 */
int kvr_signature_flat(const void* V, const kvr_layout* lay, int group, float* u_out, void* stream);

/*
 * kvr_compact with one index row per sequence:
 * K_out[h, t, :] = K[h, idx[h / group, t], :], and the same for V.
 *   idx  device, int32 [heads/group, b]
 * Other arguments and rules as in kvr_compact.
 */
int kvr_compact_shared(const void* K, const void* V, const kvr_layout* lay, int group,
                       const int32_t* idx, int b, void* K_out, void* V_out, void* stream);

/*
 * Token-axis pooling of the base scores, the smoothing step of the
 * observation-window scorers the paper builds on and compares against (Sec. 2;
 * Sec. 4.1 takes s as given and the paper does not restate the step):
 *   s_out[h,i] = max (KVR_POOL_MAX) or mean (KVR_POOL_MEAN) of s_in[h,j] over
 *   |j - i| <= kernel/2.
 * Window positions outside [0, n) are skipped by the maximum and count as zeros
 * in the mean, whose divisor is always `kernel` (this library's reading).
 *   s_in, s_out  device, dense float32 [heads, n]; must not be the same buffer
 *   kernel       odd, 1 <= kernel <= KVR_MAX_POOL; heads <= 65535 per call
 */
#define KVR_POOL_MAX 0
#define KVR_POOL_MEAN 1
#define KVR_MAX_POOL 63
int kvr_score_pool(const float* s_in, int heads, int n, int kernel, int mode, float* s_out, void* stream);

/*
 * The one-term modular scoring variant the paper tested and rejected (table of
 * negative gates, scoring family, "variant_b"; Sec. 5 discusses why a modular
 * term cannot do what the set-conditioned penalty does): a prior added to the
 * base score, the cosine of the token's value row with the head's mean value
 * direction,
 *   s_out[h,i] = s_in[h,i] + lambda_p * (V_i . dir) / ((||V_i|| + eps) (||dir|| + eps)),
 *   dir = (1/n) sum_j V[h,j,:]
 * (the paper gives the term as lambda cos(V, dir) only; the mean over the head's
 * n candidate rows and the eps of Eq. 1 in both norms are this library's
 * reading).  Top-b of s_out, kvr_select_greedy with lambda = 0, is that variant;
 * passing s_out to Algorithm 1 composes the two.
 *   V      device, [heads, n, d] per `lay`
 *   s_in   device, dense float32 [heads, n]
 *   s_out  device, dense float32 [heads, n]; may be s_in
 *   lambda_p  any finite weight (negative weights favour rows unlike the mean)
 */
int kvr_score_prior(const void* V, const kvr_layout* lay, const float* s_in, float lambda_p, float eps,
                    float* s_out, void* stream);

/*
 * The cache update of Algorithm 1's return value done inside the cache's own
 * storage, as an eviction step of a serving loop does it (the paper's method
 * returns sort(S) and leaves the storage to the caller):
 *   K[h, t, :] = K[h, idx[h / group, t], :] for t < b, the same for V and for
 *   pos[h, t] = pos[h, idx[h / group, t]]; rows t >= b keep their old contents.
 *   K, V  device, [heads, n, d] per `lay`, updated in place; either may be NULL
 *   idx   device, int32 [heads/group, b].  Each row must be strictly ascending
 *         over its entries >= 0 (idx_sorted of the calls above is) and entry t,
 *         when >= 0, must be >= t; entries < 0 (the padding kvr_retain_budgeted
 *         writes past a head's own budget) move nothing.  A row that is not
 *         ascending gives unspecified (in-bounds) contents.
 *   pos   device, dense int32 [heads, n] or NULL
 * Overlapping calls on the same tensors race.
 */
int kvr_compact_inplace(void* K, void* V, const kvr_layout* lay, int group,
                        const int32_t* idx, int b, int32_t* pos, void* stream);

/*
 * The whole flat-mode event: signature -> select (one problem per sequence) ->
 * compaction of every head of the sequence with the shared index set.
 *   s           device, dense float32 [heads/group, n]: one score vector per sequence
 *   u_out       device, dense float32 [heads/group, n, d]: receives the signature
 *               rows (required unless lambda == 0, which reads no V).  Rows of
 *               tokens that Algorithm 1 cannot select are not computed and read
 *               zero: those with s_j < s_(b) - lambda, s_(b) the b-th largest score
 *               of the sequence (one of the b best-scored tokens is always free
 *               and gains at least s_(b) - lambda; a token gains at most s_j)
 *   idx_sorted, pick_order, pick_gain   [heads/group, b], as in kvr_select_greedy
 *   K_out, V_out  device, dense [heads, b, d], dtype of `lay`
 */
int kvr_retain_flat(const void* K, const void* V, const float* s, const kvr_layout* lay, int group,
                    int b, float lambda, float eps, float* u_out,
                    int32_t* idx_sorted, int32_t* pick_order, float* pick_gain,
                    void* K_out, void* V_out, void* stream);

/*
 * The event inside a budget allocator's frame (the paper names stacking the
 * selector inside per-head / per-layer budget allocators as a composition,
 * Sec. 2 and the limitations paragraph; protected tokens are this library's
 * reading, the paper is silent on them):
 *   n_h   device, int32 [heads] or NULL: only tokens j < n_h[h] are candidates
 *         (NULL: all n)
 *   b_h   device, int32 [heads] or NULL: budget of head h, 0 <= b_h[h] <= b_max
 *         and <= n_h[h] (NULL: b_max everywhere); a budget of 0 keeps nothing
 *   keep  device, uint8 [heads, n] or NULL: non-zero marks protected tokens
 *         (sinks, a recent window).  They are members of S from the start, count
 *         towards b_h and penalise similar tokens through Eq. 2 like any other
 *         member; the greedy fill of Eq. 3 continues from there.  More protected
 *         tokens than b_h gives an unspecified subset of them.
 *   pos_in / pos_out  device, int32 [heads, n] / [heads, b_max] or NULL: position
 *         ids carried along with the kept rows
 *   lambda_h  device, float32 [heads] or NULL: per-head penalty weights, all > 0
 *         (the paper lists a lambda schedule among its untested extensions).  Head h
 *         is selected with lambda_h[h]; `lambda` must then be > 0 and only sets the
 *         scale the kernels run at (argmax of s - lambda_h m = argmax of
 *         (lambda/lambda_h) s - lambda m); pick_gain is reported for lambda_h[h]
 *   s_work  device, float32 [heads, n], required: receives the scores the
 *         selection ran on (computed from Q when Q is given, masked to -inf past
 *         n_h, protected tokens raised by a per-head offset)
 *   idx_sorted, pick_order (required), pick_gain   [heads, b_max]: the first
 *         b_h[h] entries are valid, the rest are -1 (-inf for gains).  In
 *         pick_order the protected tokens come first, in no particular order,
 *         with pick_gain +inf.
 *   K_out, V_out  device, dense [heads, b_max, d] or NULL: rows t < b_h[h] are
 *         written, the others are left as they were
 * Exactly one of (Q, G) and s_in, as in kvr_retain.  The picks for budget b_h
 * are the first b_h picks of a run for b_max (a pick depends on the earlier ones
 * only); the fused kernels stop at the head's own budget, the general path runs
 * b_max picks per head and keeps the first b_h.
 */
int kvr_retain_budgeted(const void* K, const void* V, const void* Q, int G, const float* s_in,
                        const kvr_layout* lay, const int32_t* n_h, const int32_t* b_h, int b_max,
                        const uint8_t* keep, const int32_t* pos_in, const float* lambda_h, float lambda,
                        float eps, float* s_work, int32_t* idx_sorted, int32_t* pick_order, float* pick_gain,
                        void* K_out, void* V_out, int32_t* pos_out, void* stream);

/*
 * kvr_retain_budgeted for callers that cannot hand over (or allocate) the
 * s_work buffer: code under HIP graph capture, tight serving loops, harnesses
 * that forbid allocation.  Same arguments without s_work, same results: the
 * adjusted scores live in a static device array of the library,
 * KVR_STATIC_SCRATCH_FLOATS floats (32 MiB) on every GPU the library runs on,
 * held until the process ends.  The call allocates nothing.
 *   - heads * n > KVR_STATIC_SCRATCH_FLOATS returns KVR_ERR_WORKSPACE before
 *     anything is launched.
 *   - Every call on a GPU uses that GPU's one array (each call rewrites the part
 *     it reads, nothing has to be cleared): calls that overlap on one GPU, on
 *     different streams or from different threads, race; calls on one stream
 *     are ordered like any other work.
 *   - The scores the selection ran on are not returned.
 */
#define KVR_STATIC_SCRATCH_FLOATS (8u << 20)
int kvr_retain_budgeted_static(const void* K, const void* V, const void* Q, int G, const float* s_in,
                               const kvr_layout* lay, const int32_t* n_h, const int32_t* b_h, int b_max,
                               const uint8_t* keep, const int32_t* pos_in, const float* lambda_h, float lambda,
                               float eps, int32_t* idx_sorted, int32_t* pick_order, float* pick_gain,
                               void* K_out, void* V_out, int32_t* pos_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* KVR_H_ */
