/* Calls the argument-check paths of the C-ABI from plain C.  Built with AddressSanitizer and
 * UndefinedBehaviorSanitizer (host code only) and linked against a library whose api.hip host code was built the
 * same way; tests/test_host_sanitizers.py runs it.  Every call here returns before anything is launched, so the
 * program needs no GPU.  Exit status 0 = every call returned what it should. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "modse.h"

static int failures = 0;
#define EXPECT(call, want)                                                                        \
  do {                                                                                            \
    modse_status got_ = (call);                                                                   \
    if (got_ != (want)) {                                                                         \
      fprintf(stderr, "line %d: %s returned %d (%s), expected %d\n", __LINE__, #call, (int)got_,  \
              modse_status_string(got_), (int)(want));                                            \
      ++failures;                                                                                 \
    }                                                                                             \
  } while (0)

int main(void) {
  /* d_ff lives in a heap block of exactly n_experts entries: a read past it is an error the sanitizer reports */
  const int n = 8;
  int32_t* d_ff = (int32_t*)malloc(sizeof(int32_t) * n);
  const int32_t widths[8] = {128, 384, 192, 320, 224, 288, 256, 256};
  memcpy(d_ff, widths, sizeof widths);
  modse_desc desc = {256, n, 2, d_ff, MODSE_BF16};
  size_t bytes = 0, saved = 0;
  char dummy[64];

  for (int which = MODSE_WS_FWD; which <= MODSE_WS_FWD_SAVED; ++which) {
    EXPECT(modse_workspace_size(&desc, 512, which, &bytes), MODSE_OK);
    if (bytes == 0) { fprintf(stderr, "workspace size 0 (which = %d)\n", which); ++failures; }
  }
  EXPECT(modse_workspace_size(&desc, 64, MODSE_WS_FWD, &bytes), MODSE_OK);       /* decode-sized: split-K slabs */
  EXPECT(modse_workspace_size(&desc, 0, MODSE_WS_FWD, &bytes), MODSE_OK);
  EXPECT(modse_workspace_size(&desc, ((int64_t)1 << 40), MODSE_WS_BWD, &bytes), MODSE_ERR_UNSUPPORTED);  /* 32-bit row offsets */
  EXPECT(modse_workspace_size(&desc, -1, MODSE_WS_FWD, &bytes), MODSE_ERR_INVALID_ARG);
  EXPECT(modse_workspace_size(&desc, 512, 3, &bytes), MODSE_ERR_INVALID_ARG);
  EXPECT(modse_workspace_size(&desc, 512, MODSE_WS_FWD, NULL), MODSE_ERR_INVALID_ARG);
  EXPECT(modse_workspace_size(NULL, 512, MODSE_WS_FWD, &bytes), MODSE_ERR_INVALID_ARG);
  EXPECT(modse_saved_size(&desc, 512, &saved), MODSE_OK);

  /* descriptors that must be refused */
  {
    modse_desc b = desc;
    b.n_experts = 0;
    EXPECT(modse_workspace_size(&b, 512, MODSE_WS_FWD, &bytes), MODSE_ERR_INVALID_ARG);
    b = desc; b.n_experts = 65;  /* (d_ff has 8 entries: must be refused before it is read) */
    EXPECT(modse_workspace_size(&b, 512, MODSE_WS_FWD, &bytes), MODSE_ERR_UNSUPPORTED);
    b = desc; b.top_k = 3;
    EXPECT(modse_workspace_size(&b, 512, MODSE_WS_FWD, &bytes), MODSE_ERR_UNSUPPORTED);
    b = desc; b.top_k = 0;
    EXPECT(modse_workspace_size(&b, 512, MODSE_WS_FWD, &bytes), MODSE_ERR_INVALID_ARG);
    b = desc; b.d_model = 100;
    EXPECT(modse_workspace_size(&b, 512, MODSE_WS_FWD, &bytes), MODSE_ERR_INVALID_ARG);
    b = desc; b.d_ff = NULL;
    EXPECT(modse_workspace_size(&b, 512, MODSE_WS_FWD, &bytes), MODSE_ERR_INVALID_ARG);
    b = desc; b.dtype = (modse_dtype)7;
    EXPECT(modse_workspace_size(&b, 512, MODSE_WS_FWD, &bytes), MODSE_ERR_UNSUPPORTED);
    d_ff[3] = -32;
    EXPECT(modse_workspace_size(&desc, 512, MODSE_WS_FWD, &bytes), MODSE_ERR_INVALID_ARG);
    d_ff[3] = 100;
    EXPECT(modse_workspace_size(&desc, 512, MODSE_WS_FWD, &bytes), MODSE_ERR_INVALID_ARG);
    d_ff[3] = 320;
  }

  /* calls: null pointers, a workspace that is too small, no tokens */
  modse_routing r;
  memset(&r, 0, sizeof r);
  EXPECT(modse_route(&desc, 512, NULL, dummy, NULL, &r, dummy, 1u << 30, NULL), MODSE_ERR_INVALID_ARG);
  EXPECT(modse_route(&desc, 512, dummy, dummy, NULL, NULL, dummy, 1u << 30, NULL), MODSE_ERR_INVALID_ARG);
  EXPECT(modse_route(&desc, 512, dummy, dummy, NULL, &r, dummy, 1u << 30, NULL), MODSE_ERR_INVALID_ARG); /* null outputs */
  EXPECT(modse_route_static(&desc, 512, dummy, dummy, NULL, &r, NULL), MODSE_ERR_INVALID_ARG);
  EXPECT(modse_layer_fwd(&desc, 512, dummy, dummy, NULL, dummy, dummy, dummy, NULL, NULL, NULL, dummy, 1u << 30, NULL),
         MODSE_ERR_INVALID_ARG);
  EXPECT(modse_layer_fwd(&desc, 512, dummy, dummy, NULL, dummy, dummy, dummy, dummy, NULL, NULL, dummy, 16, NULL),
         MODSE_ERR_WORKSPACE);
  EXPECT(modse_layer_fwd(&desc, 0, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL), MODSE_OK);
  EXPECT(modse_layer_bwd(&desc, 512, dummy, dummy, dummy, dummy, dummy, &r, dummy, dummy, dummy, NULL, NULL, NULL, NULL, 0,
                         dummy, 16, NULL),
         MODSE_ERR_INVALID_ARG);
  {
    int32_t* idx = (int32_t*)dummy;
    modse_routing full = {idx, (float*)dummy, idx, idx, idx, idx, idx};
    /* more tokens than the fixed scratch array serves: refused by size alone */
    EXPECT(modse_route_static(&desc, (int64_t)1 << 22, dummy, dummy, NULL, &full, NULL), MODSE_ERR_WORKSPACE);
    EXPECT(modse_route(&desc, 512, dummy, dummy, NULL, &full, dummy, 16, NULL), MODSE_ERR_WORKSPACE);
    EXPECT(modse_routing_stats(&desc, 512, &full, NULL, NULL, NULL), MODSE_ERR_INVALID_ARG);
  }
  {
    modse_gate_ext g;
    memset(&g, 0, sizeof g);
    g.eps = -1.f;
    g.W_noise = dummy;
    modse_routing full = {(int32_t*)dummy, (float*)dummy, (int32_t*)dummy, (int32_t*)dummy, (int32_t*)dummy,
                          (int32_t*)dummy, (int32_t*)dummy};
    EXPECT(modse_route_ext(&desc, 512, dummy, dummy, NULL, &g, &full, dummy, 1u << 30, NULL), MODSE_ERR_INVALID_ARG);
  }
  for (int s = -1; s < 8; ++s)
    if (modse_status_string((modse_status)s) == NULL) { fprintf(stderr, "no string for status %d\n", s); ++failures; }
  float ms[MODSE_N_STAGES];
  EXPECT(modse_stage_times(ms), MODSE_OK);
  EXPECT(modse_stage_times(NULL), MODSE_ERR_INVALID_ARG);

  free(d_ff);
  if (failures) fprintf(stderr, "%d check(s) failed\n", failures);
  else printf("host ABI driver: all checks passed\n");
  return failures ? 1 : 0;
}
