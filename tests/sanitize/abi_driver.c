/* Calls the host-side validation of the C ABI (no GPU work: every call below is refused
 * before anything is launched) in a library whose host code was built with
 * -fsanitize=address,undefined, from a driver built the same way.  The pointers handed in
 * are real host allocations of the sizes the interface promises to read on the host
 * (cu_seqlens_host), so an overrun in the validation itself ends the run. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "fmha_varlen.h"

#define EXPECT(call, code)                                                                       \
  do {                                                                                           \
    const int rc_ = (call);                                                                      \
    if (rc_ != (code)) {                                                                         \
      fprintf(stderr, "%s:%d: %s returned %d (%s), expected %d\n", __FILE__, __LINE__, #call, rc_, \
              fmha_last_error(), (code));                                                        \
      return 1;                                                                                  \
    }                                                                                            \
    if ((code) != FMHA_OK && !fmha_last_error()[0]) {                                            \
      fprintf(stderr, "%s:%d: no error message\n", __FILE__, __LINE__);                          \
      return 1;                                                                                  \
    }                                                                                            \
  } while (0)

int main(void) {
  /* stand-ins for device pointers: aligned host memory that no refused call touches */
  void* dev = aligned_alloc(256, 1 << 16);
  int32_t* cu_host = malloc(sizeof(int32_t) * 4);  /* exactly batch + 1 entries */
  cu_host[0] = 0, cu_host[1] = 5, cu_host[2] = 5, cu_host[3] = 12;
  fmha_varlen_params_t p;
  memset(&p, 0, sizeof(p));
  p.batch = 3, p.total_tokens = 12, p.heads = 2, p.head_dim = 64, p.dtype = FMHA_F16, p.scale = 0.125f;
  p.cu_seqlens = dev, p.cu_seqlens_host = cu_host, p.workspace = dev, p.workspace_bytes = 1 << 16;

  if (fmha_varlen_workspace_size(3, 12, 2, 0) == 0 || fmha_varlen_workspace_size(3, 12, 2, 1) == 0 ||
      fmha_varlen_workspace_size(-1, 12, 2, 0) != 0 || fmha_varlen_workspace_size(3, 12, 0, 1) != 0) {
    fprintf(stderr, "workspace size arithmetic\n");
    return 1;
  }
  EXPECT(fmha_varlen_fwd(NULL, dev, dev, dev, dev, dev, NULL), FMHA_ERR_INVALID_ARG);
  EXPECT(fmha_varlen_fwd(&p, NULL, dev, dev, dev, dev, NULL), FMHA_ERR_INVALID_ARG);
  EXPECT(fmha_varlen_fwd(&p, (char*)dev + 2, dev, dev, dev, dev, NULL), FMHA_ERR_INVALID_ARG);
  {
    fmha_varlen_params_t x = p;
    x.head_dim = 128;
    EXPECT(fmha_varlen_fwd(&x, dev, dev, dev, dev, dev, NULL), FMHA_ERR_UNSUPPORTED);
    x = p, x.dtype = 7;
    EXPECT(fmha_varlen_fwd(&x, dev, dev, dev, dev, dev, NULL), FMHA_ERR_UNSUPPORTED);
    x = p, x.q_stride = 100;
    EXPECT(fmha_varlen_fwd(&x, dev, dev, dev, dev, dev, NULL), FMHA_ERR_INVALID_ARG);
    x = p, x.workspace_bytes = 16;
    EXPECT(fmha_varlen_fwd(&x, dev, dev, dev, dev, dev, NULL), FMHA_ERR_WORKSPACE);
    x = p, x.workspace = NULL;
    EXPECT(fmha_varlen_fwd(&x, dev, dev, dev, dev, dev, NULL), FMHA_ERR_WORKSPACE);
    x = p, x.total_tokens = 13; /* disagrees with cu_seqlens_host[batch] */
    EXPECT(fmha_varlen_fwd(&x, dev, dev, dev, dev, dev, NULL), FMHA_ERR_INVALID_ARG);
    x = p, x.max_seqlen = 4;    /* shorter than a sequence of the host copy */
    EXPECT(fmha_varlen_fwd(&x, dev, dev, dev, dev, dev, NULL), FMHA_ERR_INVALID_ARG);
    cu_host[2] = 3;             /* decreasing prefix sums */
    EXPECT(fmha_varlen_fwd(&p, dev, dev, dev, dev, dev, NULL), FMHA_ERR_INVALID_ARG);
    cu_host[2] = 5;
    x = p, x.flags = FMHA_FLAG_BWD_ONLY_DQ | FMHA_FLAG_BWD_ONLY_DKV, x.workspace_bytes = (size_t)1 << 30;
    EXPECT(fmha_varlen_bwd(&x, dev, dev, dev, dev, dev, dev, dev, dev, dev, NULL), FMHA_ERR_INVALID_ARG);
    x = p, x.scale = 1.0f / 0.0f;
    EXPECT(fmha_varlen_fwd(&x, dev, dev, dev, dev, dev, NULL), FMHA_ERR_INVALID_ARG);
    /* the entry point without allocations refuses batches whose tile list outgrows its array */
    x = p, x.cu_seqlens_host = NULL, x.batch = 1 << 20, x.total_tokens = 1 << 20;
    EXPECT(fmha_varlen_fwd_static(&x, dev, dev, dev, dev, dev, NULL), FMHA_ERR_WORKSPACE);
    fmha_dropout_t d = {1.5f, 7};
    EXPECT(fmha_varlen_fwd_dropout(&p, &d, dev, dev, dev, dev, dev, NULL), FMHA_ERR_INVALID_ARG);
    EXPECT(fmha_varlen_fwd_dropout(&p, NULL, dev, dev, dev, dev, dev, NULL), FMHA_ERR_INVALID_ARG);
  }
  /* an empty batch is a success that launches nothing */
  {
    fmha_varlen_params_t x = p;
    x.batch = 0, x.total_tokens = 0, x.cu_seqlens_host = NULL;
    EXPECT(fmha_varlen_fwd(&x, dev, dev, dev, dev, dev, NULL), FMHA_OK);
  }
  free(cu_host);
  free(dev);
  puts("C ABI validation under sanitizers: ok");
  return 0;
}
