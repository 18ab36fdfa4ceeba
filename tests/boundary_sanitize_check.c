/* Driver of the host-side sanitizer leg for the C-ABI library: every entry point of include/hydra_attn.h is
 * called with arguments that the host-side validation must turn into a status code before anything is launched
 * (the addresses are fake and never dereferenced; there is no device).  Linked against a build of the library
 * whose HOST code is instrumented with AddressSanitizer and UndefinedBehaviorSanitizer. */
#include <stdint.h>
#include <stdio.h>

#include "../include/hydra_attn.h"

static int failures = 0;
#define EXPECT(call, want)                                                        \
  do {                                                                            \
    const int got_ = (call);                                                      \
    if (got_ != (want)) {                                                         \
      printf("line %d: got %d, expected %d\n", __LINE__, got_, (int)(want));      \
      failures++;                                                                 \
    }                                                                             \
  } while (0)

int main(void) {
  void* p = (void*)16;
  const int32_t* ip = (const int32_t*)16;
  const int64_t* lp = (const int64_t*)16;
  const size_t ws = 1 << 20;
  /* packed attention: combined call, its two halves, the two-stream and the static-scratch variants */
  EXPECT(hydra_attn_varlen_fwd(NULL, p, p, p, 128, 128, 128, ip, 1, 8, 8, 2, 2, 64, 0, 0.125f, p, ws, NULL), HYDRA_ERR_INVALID_ARG);
  EXPECT(hydra_attn_varlen_fwd(p, p, p, p, 128, 128, 128, ip, 1, 8, 8, 2, 2, 96, 0, 0.125f, p, ws, NULL), HYDRA_ERR_UNSUPPORTED);
  EXPECT(hydra_attn_varlen_fwd(p, p, p, p, 128, 128, 128, ip, 1, 8, 8, 2, 2, 64, 0, 0.125f, p, 8, NULL), HYDRA_ERR_WORKSPACE);
  EXPECT(hydra_attn_varlen_fwd(p, p, p, p, 128, 2048, 128, ip, 1, 1 << 20, 1 << 20, 2, 2, 64, 0, 0.125f, p, (size_t)1 << 30, NULL), HYDRA_ERR_UNSUPPORTED);
  EXPECT(hydra_attn_varlen_fwd(NULL, NULL, NULL, NULL, 128, 128, 128, NULL, 0, 0, 0, 2, 2, 64, 0, 0.125f, NULL, 0, NULL), HYDRA_OK);
  EXPECT(hydra_attn_build_worklist(NULL, 1, 8, 8, 2, 2, 64, 1, p, ws, NULL), HYDRA_ERR_INVALID_ARG);
  EXPECT(hydra_attn_build_worklist(ip, 1, 8, 8, 2, 2, 64, 1, NULL, ws, NULL), HYDRA_ERR_WORKSPACE);
  EXPECT(hydra_attn_varlen_fwd_prebuilt(p, p, p, p, 128, 128, 132, ip, 1, 8, 8, 2, 2, 64, 0, 0.125f, p, ws, NULL), HYDRA_ERR_INVALID_ARG);
  EXPECT(hydra_attn_varlen_fwd_shared(p, p, p, p, 128, 128, 128, ip, 1, 8, 8, 2, 2, 64, 0, 0.125f, p, ws, 0, NULL), HYDRA_ERR_INVALID_ARG);
  EXPECT(hydra_attn_varlen_fwd_static(p, p, p, p, 4096, 1024, 1024, ip, 4096, 1 << 20, 4096, 32, 8, 128, 1, 0.125f, NULL), HYDRA_ERR_WORKSPACE);
  EXPECT(hydra_attn_varlen_fwd_static(p, p, p, p, 128, 128, 128, ip, 1, 8, 8, 3, 2, 64, 1, 0.125f, NULL), HYDRA_ERR_INVALID_ARG);
  if (hydra_attn_workspace_bytes(48, 30000, 1312, 28, 4, 128) == 0 || hydra_attn_workspace_bytes(4, 438, 257, 3, 2, 64) != 0) failures++;
  /* paged KV write, attention over the paged cache, paged image cache */
  EXPECT(hydra_kv_cache_write(p, p, 128, 128, p, NULL, lp, 4, 2, 64, 16, 4, NULL), HYDRA_ERR_INVALID_ARG);
  EXPECT(hydra_kv_cache_write(p, p, 128, 128, p, p, lp, 4, 1, 60, 16, 4, NULL), HYDRA_ERR_UNSUPPORTED);
  EXPECT(hydra_kv_cache_write(NULL, NULL, 128, 128, NULL, NULL, NULL, 0, 2, 64, 16, 4, NULL), HYDRA_OK);
  EXPECT(hydra_attn_paged_fwd(p, p, 128, p, p, ip, 4, ip, ip, 2, 2, 1, 2, 2, 64, 12, 8, 0.125f, NULL, 0, NULL), HYDRA_ERR_UNSUPPORTED);
  EXPECT(hydra_attn_paged_fwd(p, NULL, 128, p, p, ip, 4, ip, ip, 2, 2, 1, 2, 2, 64, 16, 8, 0.125f, NULL, 0, NULL), HYDRA_ERR_INVALID_ARG);
  EXPECT(hydra_attn_paged_fwd(p, p, 128, p, p, ip, 4, ip, ip, 2, 2, 1, 2, 2, 64, 16, 8, 0.125f, NULL, 64, NULL), HYDRA_ERR_WORKSPACE);
  if (hydra_attn_paged_workspace_bytes(8, 4, 128, 1024, 16) == 0 || hydra_attn_paged_workspace_bytes(0, 4, 128, 1024, 16) != 0) failures++;
  EXPECT(hydra_page_cache_write(p, 4096, p, lp, 8, 4100, 64, NULL), HYDRA_ERR_UNSUPPORTED);
  EXPECT(hydra_page_cache_gather(p, lp, NULL, 4096, 8, 4096, 64, NULL), HYDRA_ERR_INVALID_ARG);
  EXPECT(hydra_page_cache_gather(NULL, NULL, NULL, 4096, 0, 4096, 64, NULL), HYDRA_OK);
  for (int s = -1; s < 7; s++)
    if (!hydra_status_string(s) || !hydra_status_string(s)[0]) failures++;
  printf("%s\n", failures ? "MISMATCH" : "all statuses as expected");
  return failures != 0;
}
