/* Host-side walk through the argument validation of every entry point of
 * include/kvr.h.  Built by tests/test_host_sanitizers.py together with the
 * library's host code under AddressSanitizer and UndefinedBehaviorSanitizer and
 * run on the CPU: every call below must be refused before anything is launched,
 * so no GPU is needed and no pointer is ever dereferenced. */
#include <math.h>
#include <stdio.h>
#include <string.h>

#include "../include/kvr.h"

static int failures = 0;
#define EXPECT(call, want)                                                            \
  do {                                                                                \
    const int got_ = (call);                                                          \
    if (got_ != (want)) { printf("line %d: got %d, want %d\n", __LINE__, got_, (want)); ++failures; } \
  } while (0)

int main(void) {
  void* fake = (void*)0x1000;
  void* other = (void*)0x2000;
  void* odd = (void*)0x1004;
  kvr_layout lay = {2, 64, 128, KVR_BF16, 64 * 128, 128};
  kvr_layout bad_d = lay; bad_d.d = 64;
  kvr_layout big_n = lay; big_n.n = KVR_MAX_N + 1;
  kvr_layout short_tok = lay; short_tok.stride_tok = 64;
  kvr_layout overlap = lay; overlap.stride_head = 100;
  kvr_layout bad_dt = lay; bad_dt.dtype = 5;
  kvr_layout six = lay; six.heads = 6;
  kvr_layout huge = {2049, 4096, 128, KVR_BF16, 4096 * 128, 128};
  size_t ws = 7;

  EXPECT(kvr_version() >= 1 ? 0 : 1, 0);
  for (int c = -6; c <= 0; ++c) EXPECT(strlen(kvr_strerror(c)) > 0 ? 0 : 1, 0);
  EXPECT(kvr_workspace_bytes(&lay, 16, 4, &ws), KVR_OK);
  EXPECT((int)ws, 0);
  EXPECT(kvr_workspace_bytes(NULL, 16, 4, &ws), KVR_ERR_ARG);
  EXPECT(kvr_workspace_bytes(&lay, 16, 4, NULL), KVR_ERR_ARG);
  EXPECT(kvr_workspace_bytes(&lay, 65, 4, &ws), KVR_ERR_ARG);

  EXPECT(kvr_score(fake, fake, 1, &bad_d, fake, NULL), KVR_ERR_UNSUPPORTED);
  EXPECT(kvr_score(fake, fake, 1, &big_n, fake, NULL), KVR_ERR_UNSUPPORTED);
  EXPECT(kvr_score(fake, fake, 0, &lay, fake, NULL), KVR_ERR_ARG);
  EXPECT(kvr_score(fake, fake, KVR_MAX_G + 1, &lay, fake, NULL), KVR_ERR_UNSUPPORTED);
  EXPECT(kvr_score(NULL, fake, 1, &lay, fake, NULL), KVR_ERR_ARG);
  EXPECT(kvr_score(odd, fake, 1, &lay, fake, NULL), KVR_ERR_ARG);

  EXPECT(kvr_select_greedy(fake, fake, &lay, 0, 0.5f, 1e-6f, fake, NULL, NULL, NULL, 0, NULL), KVR_ERR_ARG);
  EXPECT(kvr_select_greedy(fake, fake, &lay, 65, 0.5f, 1e-6f, fake, NULL, NULL, NULL, 0, NULL), KVR_ERR_ARG);
  EXPECT(kvr_select_greedy(fake, fake, &lay, 8, -0.1f, 1e-6f, fake, NULL, NULL, NULL, 0, NULL), KVR_ERR_ARG);
  EXPECT(kvr_select_greedy(fake, fake, &lay, 8, NAN, 1e-6f, fake, NULL, NULL, NULL, 0, NULL), KVR_ERR_ARG);
  EXPECT(kvr_select_greedy(fake, fake, &lay, 8, INFINITY, 1e-6f, fake, NULL, NULL, NULL, 0, NULL), KVR_ERR_ARG);
  EXPECT(kvr_select_greedy(fake, fake, &lay, 8, 0.5f, -1.0f, fake, NULL, NULL, NULL, 0, NULL), KVR_ERR_ARG);
  EXPECT(kvr_select_greedy(NULL, fake, &lay, 8, 0.5f, 1e-6f, fake, NULL, NULL, NULL, 0, NULL), KVR_ERR_ARG);
  EXPECT(kvr_select_greedy(fake, fake, &lay, 8, 0.5f, 1e-6f, NULL, NULL, NULL, NULL, 0, NULL), KVR_ERR_ARG);
  EXPECT(kvr_select_greedy(fake, fake, &short_tok, 8, 0.5f, 1e-6f, fake, NULL, NULL, NULL, 0, NULL), KVR_ERR_ARG);
  EXPECT(kvr_select_greedy(fake, fake, &overlap, 8, 0.5f, 1e-6f, fake, NULL, NULL, NULL, 0, NULL), KVR_ERR_ARG);
  EXPECT(kvr_select_greedy(fake, fake, &bad_dt, 8, 0.5f, 1e-6f, fake, NULL, NULL, NULL, 0, NULL), KVR_ERR_UNSUPPORTED);

  EXPECT(kvr_compact(fake, fake, &lay, NULL, 8, fake, fake, NULL), KVR_ERR_ARG);
  EXPECT(kvr_compact(fake, NULL, &lay, fake, 8, fake, fake, NULL), KVR_ERR_ARG);
  EXPECT(kvr_compact(NULL, NULL, &lay, fake, 8, NULL, NULL, NULL), KVR_ERR_ARG);
  EXPECT(kvr_compact(fake, fake, &lay, fake, 65, fake, fake, NULL), KVR_ERR_ARG);

  EXPECT(kvr_retain(fake, fake, fake, 1, fake, &lay, 8, 0.5f, 1e-6f, fake, fake, NULL, NULL, fake, fake, NULL, 0, NULL), KVR_ERR_ARG);
  EXPECT(kvr_retain(fake, fake, NULL, 0, NULL, &lay, 8, 0.5f, 1e-6f, fake, fake, NULL, NULL, fake, fake, NULL, 0, NULL), KVR_ERR_ARG);
  EXPECT(kvr_retain(fake, fake, NULL, 0, fake, &lay, 80, 0.5f, 1e-6f, NULL, fake, NULL, NULL, fake, fake, NULL, 0, NULL), KVR_ERR_ARG);
  EXPECT(kvr_retain(fake, fake, fake, 1, NULL, &lay, 8, 0.5f, 1e-6f, NULL, fake, NULL, NULL, fake, fake, NULL, 0, NULL), KVR_ERR_ARG);

  EXPECT(kvr_signature_flat(fake, &six, 4, fake, NULL), KVR_ERR_ARG);
  EXPECT(kvr_signature_flat(fake, &six, 0, fake, NULL), KVR_ERR_ARG);
  EXPECT(kvr_signature_flat(NULL, &six, 3, fake, NULL), KVR_ERR_ARG);
  EXPECT(kvr_compact_shared(fake, fake, &six, 4, fake, 8, fake, fake, NULL), KVR_ERR_ARG);
  EXPECT(kvr_compact_shared(fake, fake, &six, 3, NULL, 8, fake, fake, NULL), KVR_ERR_ARG);
  EXPECT(kvr_score_pool(fake, 4, 64, 7, KVR_POOL_MAX, fake, NULL), KVR_ERR_ARG);
  EXPECT(kvr_score_pool(fake, 4, 64, 6, KVR_POOL_MAX, other, NULL), KVR_ERR_ARG);
  EXPECT(kvr_score_pool(fake, 4, 64, KVR_MAX_POOL + 2, KVR_POOL_MAX, other, NULL), KVR_ERR_ARG);
  EXPECT(kvr_score_pool(fake, 4, 64, 7, 2, other, NULL), KVR_ERR_ARG);
  EXPECT(kvr_score_pool(fake, 0, 64, 7, KVR_POOL_MEAN, other, NULL), KVR_ERR_ARG);
  EXPECT(kvr_score_pool(NULL, 4, 64, 7, KVR_POOL_MEAN, other, NULL), KVR_ERR_ARG);
  EXPECT(kvr_score_prior(NULL, &six, fake, 0.5f, 1e-6f, fake, NULL), KVR_ERR_ARG);
  EXPECT(kvr_score_prior(fake, &six, NULL, 0.5f, 1e-6f, fake, NULL), KVR_ERR_ARG);
  EXPECT(kvr_score_prior(fake, &six, fake, NAN, 1e-6f, fake, NULL), KVR_ERR_ARG);
  EXPECT(kvr_score_prior(fake, &six, fake, 0.5f, -1.0f, fake, NULL), KVR_ERR_ARG);
  EXPECT(kvr_compact_inplace(fake, fake, &six, 4, fake, 8, NULL, NULL), KVR_ERR_ARG);
  EXPECT(kvr_compact_inplace(fake, fake, &six, 1, NULL, 8, NULL, NULL), KVR_ERR_ARG);
  EXPECT(kvr_compact_inplace(NULL, NULL, &six, 1, fake, 8, NULL, NULL), KVR_ERR_ARG);
  EXPECT(kvr_compact_inplace(fake, fake, &six, 1, fake, 65, NULL, NULL), KVR_ERR_ARG);
  EXPECT(kvr_compact_inplace(odd, fake, &six, 1, fake, 8, NULL, NULL), KVR_ERR_ARG);
  EXPECT(kvr_retain_flat(fake, fake, fake, &six, 3, 8, 0.5f, 1e-6f, NULL, fake, NULL, NULL, fake, fake, NULL), KVR_ERR_ARG);
  EXPECT(kvr_retain_flat(fake, fake, fake, &six, 4, 8, 0.5f, 1e-6f, fake, fake, NULL, NULL, fake, fake, NULL), KVR_ERR_ARG);
  EXPECT(kvr_retain_flat(fake, fake, fake, &six, 3, 65, 0.5f, 1e-6f, fake, fake, NULL, NULL, fake, fake, NULL), KVR_ERR_ARG);
  EXPECT(kvr_retain_flat(fake, fake, NULL, &six, 3, 8, 0.5f, 1e-6f, fake, fake, NULL, NULL, fake, fake, NULL), KVR_ERR_ARG);

  EXPECT(kvr_retain_budgeted(fake, fake, NULL, 0, fake, &lay, NULL, NULL, 65, NULL, NULL, NULL, 0.5f, 1e-6f, fake, fake, fake, fake, fake, fake, NULL, NULL), KVR_ERR_ARG);
  EXPECT(kvr_retain_budgeted(fake, fake, NULL, 0, NULL, &lay, NULL, NULL, 8, NULL, NULL, NULL, 0.5f, 1e-6f, fake, fake, fake, fake, fake, fake, NULL, NULL), KVR_ERR_ARG);
  EXPECT(kvr_retain_budgeted(fake, fake, NULL, 0, fake, &lay, NULL, NULL, 8, NULL, NULL, NULL, 0.5f, 1e-6f, NULL, fake, fake, fake, fake, fake, NULL, NULL), KVR_ERR_ARG);
  EXPECT(kvr_retain_budgeted(fake, fake, NULL, 0, fake, &lay, NULL, NULL, 8, NULL, NULL, NULL, 0.5f, 1e-6f, fake, fake, NULL, fake, fake, fake, NULL, NULL), KVR_ERR_ARG);
  EXPECT(kvr_retain_budgeted(fake, fake, NULL, 0, fake, &lay, NULL, NULL, 8, NULL, NULL, NULL, 0.5f, 1e-6f, fake, fake, fake, fake, fake, fake, fake, NULL), KVR_ERR_ARG);
  EXPECT(kvr_retain_budgeted(fake, fake, NULL, 0, fake, &lay, NULL, NULL, 8, NULL, NULL, fake, 0.0f, 1e-6f, fake, fake, fake, fake, fake, fake, NULL, NULL), KVR_ERR_ARG);
  /* the entry point with the static scratch: too large a call is refused before the array is even looked up */
  EXPECT(kvr_retain_budgeted_static(fake, fake, NULL, 0, fake, &huge, NULL, NULL, 16, NULL, NULL, NULL, 0.5f, 1e-6f, fake, fake, fake, NULL, NULL, NULL, NULL), KVR_ERR_WORKSPACE);
  EXPECT(kvr_retain_budgeted_static(fake, fake, NULL, 0, fake, &lay, NULL, NULL, 65, NULL, NULL, NULL, 0.5f, 1e-6f, fake, fake, fake, NULL, NULL, NULL, NULL), KVR_ERR_ARG);

  if (failures) { printf("%d host checks failed\n", failures); return 1; }
  printf("host checks ok\n");
  return 0;
}
