/* Plain C user of the library's boundary: includes thk.h, links libthk.so, and exercises the
 * entry points that need no GPU (host arithmetic, argument checks that return before any
 * launch).  Built and run by tests/test_abi_host.py with gcc. */
#include <stdio.h>
#include <string.h>

#include "thk.h"

#define CHECK(cond)                                              \
  do {                                                           \
    if (!(cond)) {                                               \
      printf("FAILED line %d: %s\n", __LINE__, #cond);           \
      return 1;                                                  \
    }                                                            \
  } while (0)

int main(void) {
  thk_shape s;
  memset(&s, 0, sizeof s);
  s.L = 32; s.B = 4; s.N_q = 32; s.N_kv = 32; s.D = 128; s.S = 4096; s.S_obs = 32;
  s.T = thk_keep_count(128, 0.4); s.dtype = THK_BF16;
  CHECK(thk_version() > 0);
  CHECK(s.T == 76);
  CHECK(thk_keep_count(128, 0.5) == 64 && thk_keep_count(128, 0.6) == 51 && thk_keep_count(128, 1.0) == -1);
  CHECK(strcmp(thk_status_string(THK_OK), "ok") == 0);
  CHECK(thk_workspace_bytes(&s, THK_OP_PRUNE) > 0);
  CHECK(thk_workspace_bytes(&s, THK_OP_DECODE) == 0 || thk_workspace_bytes(&s, THK_OP_DECODE) >= 16);
  CHECK(thk_workspace_bytes(&s, THK_OP_SCORE_VALUE) > 0);
  CHECK(thk_default_split(&s, THK_OP_DECODE) >= 1);
  CHECK(thk_prune_is_fused(&s) == 2);
  CHECK(thk_decode_on_matrix_cores(&s, 0, 0) == 0);   /* one query head per KV head: the general kernel */
  s.N_kv = 8;
  CHECK(thk_decode_on_matrix_cores(&s, 0, 0) == 1 && thk_decode_on_matrix_cores(&s, 51, 52) == 1);
  s.N_kv = 32;
  /* argument errors come back synchronously, before anything touches a device */
  char fake[64] __attribute__((aligned(16)));
  CHECK(thk_score(NULL, fake, fake, (float *)fake, fake, 64, NULL) == THK_ERR_NULL);
  CHECK(thk_score(&s, NULL, fake, (float *)fake, fake, 64, NULL) == THK_ERR_NULL);
  CHECK(thk_score(&s, fake, fake + 4, (float *)fake, fake, 64, NULL) == THK_ERR_ALIGN);
  CHECK(thk_score(&s, fake, fake, (float *)fake, fake, 64, NULL) == THK_ERR_WORKSPACE);
  s.T = 200;
  CHECK(thk_select_topk(&s, (const float *)fake, (int16_t *)fake, NULL) == THK_ERR_SHAPE);
  s.T = 32; s.D = 64;
  CHECK(thk_decode_attn(&s, fake, fake, (const int16_t *)fake, fake, NULL, NULL, 0, 0, fake, fake, 64, NULL) ==
        THK_ERR_UNSUPPORTED);
  printf("abi host check ok\n");
  return 0;
}
