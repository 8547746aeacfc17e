/* Host-side exercise of the C ABI for an AddressSanitizer / UBSan build of the library's HOST code (no GPU needed):
 * shape validation, workspace sizing over many shapes, and the argument checks that return before any launch.
 * Built and run by tests/test_host_sanitizers.py.  Prints "ok <number of calls>" on success. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../include/nsa_sel.h"

#define CHECK(cond)                                                     \
  do {                                                                  \
    if (!(cond)) {                                                      \
      fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); \
      return 1;                                                         \
    }                                                                   \
  } while (0)

int main(void) {
  long calls = 0;
  const int tokens[] = {0, 1, 63, 64, 65, 1000, 4096, 65536, 262144, 870000, 2000000, 1 << 30};
  const int heads[][2] = {{1, 1}, {4, 1}, {7, 1}, {8, 1}, {32, 8}, {28, 4}, {64, 8}, {16, 16}, {9, 1}, {8, 3}, {0, 0}};
  const int blocks[] = {64, 128, 32, 0};
  const int topks[] = {1, 8, 16, 32, 33, 0, -1};
  for (size_t a = 0; a < sizeof tokens / sizeof *tokens; ++a)
    for (size_t b = 0; b < sizeof heads / sizeof *heads; ++b)
      for (size_t c = 0; c < sizeof blocks / sizeof *blocks; ++c)
        for (size_t d = 0; d < sizeof topks / sizeof *topks; ++d)
          for (int nseq = 0; nseq <= 9; nseq += 3)
            for (int dense = -2; dense <= 2; ++dense) {
              nsa_sel_shape s;
              memset(&s, 0, sizeof s);
              s.total_tokens = tokens[a];
              s.nseq = nseq;
              s.hq = heads[b][0];
              s.hkv = heads[b][1];
              s.d = 128;
              s.block = blocks[c];
              s.topk = topks[d];
              s.causal = 1;
              s.window = (int)(a % 3) * 200;
              s.unit = (d % 2) ? 512 : 0;
              s.dense = dense;
              size_t f = 0, bw = 0, ix = 0, fm = 0, bm = 0;
              const int rc = nsa_sel_workspace_bytes(&s, &f, &bw, &ix);
              const int rc2 = nsa_sel_workspace_bytes_min(&s, &fm, &bm);
              calls += 2;
              CHECK(rc == rc2);
              CHECK(rc == NSA_SEL_OK || rc == NSA_SEL_EINVAL || rc == NSA_SEL_EUNSUPPORTED);
              CHECK(nsa_sel_strerror(rc) != NULL);
              if (rc == NSA_SEL_OK) {
                CHECK(fm <= f && bm <= bw);
                CHECK(ix >= 64);
                /* pointer checks come before any GPU call: null, misaligned, missing cu_seqlens, small workspaces */
                void* p = (void*)(uintptr_t)4096;
                void* odd = (void*)(uintptr_t)4098;
                if (s.total_tokens > 0) {
                  CHECK(nsa_sel_build_index(&s, NULL, NULL, p, ix, NULL) == NSA_SEL_EINVAL);
                  CHECK(nsa_sel_fwd(&s, NULL, p, p, p, p, 1, p, ix, p, p, p, f, NULL) == NSA_SEL_EINVAL);
                  CHECK(nsa_sel_fwd(&s, odd, p, p, p, p, 1, p, ix, p, p, p, f, NULL) == NSA_SEL_EINVAL);
                  CHECK(nsa_sel_fwd(&s, p, p, p, p, p, 1, p, ix - 1, p, p, p, f, NULL) == NSA_SEL_EWORKSPACE);
                  CHECK(nsa_sel_fwd(&s, p, p, p, p, p, 1, p, ix, p, p, p, fm - 1, NULL) == NSA_SEL_EWORKSPACE);
                  CHECK(nsa_sel_bwd(&s, p, p, p, p, p, p, p, p, ix, p, p, p, p, bm - 1, NULL) == NSA_SEL_EWORKSPACE);
                  CHECK(nsa_sel_bwd(&s, p, p, p, p, p, NULL, p, p, ix, p, p, p, p, bw, NULL) == NSA_SEL_EINVAL);
                  CHECK(nsa_sel_fwd_gated(&s, p, p, p, p, p, 1, p, ix, p, p, p, p, p, p, f, NULL) == NSA_SEL_EINVAL); /* O_out == O */
                  if (s.nseq > 1) CHECK(nsa_sel_fwd(&s, p, p, p, p, NULL, 1, p, ix, p, p, p, f, NULL) == NSA_SEL_EINVAL);
                  const int st = nsa_sel_fwd_static(&s, NULL, p, p, p, p, 1, p, ix, p, p, NULL);
                  CHECK(st == NSA_SEL_EINVAL || st == NSA_SEL_ESTATIC);
                  calls += 10;
                } else {
                  CHECK(nsa_sel_fwd(&s, NULL, NULL, NULL, NULL, NULL, 1, NULL, 0, NULL, NULL, NULL, 0, NULL) == NSA_SEL_OK);
                  calls += 1;
                }
                const int32_t *cnt, *off, *qent;
                const uint32_t* vm;
                int32_t bcap = -1;
                CHECK(nsa_sel_index_view(&s, p, &cnt, &off, &qent, &vm, &bcap) == NSA_SEL_OK);
                CHECK(bcap == s.total_tokens / s.block + s.nseq);
                ++calls;
              }
            }
  CHECK(nsa_sel_workspace_bytes(NULL, NULL, NULL, NULL) == NSA_SEL_EINVAL);
  CHECK(nsa_sel_select_blocks(NULL, NULL, 0, NULL, 0, 0, NULL, NULL) != NSA_SEL_OK);
  CHECK(nsa_sel_profile_collect(0, NULL, NULL, NULL) <= 0);
  for (int code = -8; code <= 1; ++code) CHECK(strlen(nsa_sel_strerror(code)) > 1);
  printf("ok %ld\n", calls);
  return 0;
}
