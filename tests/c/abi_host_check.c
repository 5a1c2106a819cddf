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
  /* every other entry point: a valid shape, then one bad argument each; nothing reaches a device */
  s.T = 76; s.D = 128; s.ld_keep = 0;
  size_t big = (size_t)1 << 40;
  int16_t *i16 = (int16_t *)fake;
  CHECK(thk_prune(&s, fake, fake, NULL, i16, fake, fake, 16, NULL) == THK_ERR_WORKSPACE);
  CHECK(thk_prune(&s, fake, NULL, NULL, i16, fake, fake, big, NULL) == THK_ERR_NULL);
  CHECK(thk_score_magnitude(&s, fake, 3, (float *)fake, fake, big, NULL) == THK_ERR_SHAPE);
  CHECK(thk_score_value(&s, fake, fake, fake, 2, (float *)fake, fake, big, NULL) == THK_ERR_SHAPE);
  CHECK(thk_prune_value(&s, fake, fake, fake, 1, NULL, NULL, fake, fake, big, NULL) == THK_ERR_NULL);
  CHECK(thk_compact_keys(&s, fake, i16, fake + 2, NULL) == THK_ERR_ALIGN);
  CHECK(thk_compact_rows(&s, fake, 64, 60, i16, fake, 0, 8, NULL) == THK_ERR_SHAPE);
  CHECK(thk_copy_rows(&s, fake, 64, 0, fake, 64, 4, 8, NULL) == THK_ERR_SHAPE);   /* upward shift in place */
  CHECK(thk_cache_append(&s, fake, fake, fake, fake, 0, 4, NULL) == THK_ERR_SHAPE); /* value cache full: S_cap == S */
  CHECK(thk_tail_flush(&s, i16, fake, fake, NULL, NULL, 4, 8, 5, NULL) == THK_ERR_SHAPE);
  CHECK(thk_tail_append(&s, fake, fake, fake, fake, 4, 4, NULL) == THK_ERR_SHAPE);
  CHECK(thk_decode_attn(&s, fake, fake, i16, fake, NULL, NULL, 1, 4, fake, fake, big, NULL) == THK_ERR_NULL);
  CHECK(thk_decode_attn_kv(&s, fake, fake, i16, fake, i16, 51, 51, NULL, NULL, 0, 0, fake, fake, big, NULL) ==
        THK_ERR_UNSUPPORTED);
  CHECK(thk_decode_attn_kv(&s, fake, fake, i16, fake, i16, 0, 0, NULL, NULL, 0, 0, fake, fake, big, NULL) ==
        THK_ERR_SHAPE);
  {
    thk_shape huge = s;   /* split partials beyond the static buffer: refused before any device call */
    huge.L = 1; huge.B = 64; huge.N_q = 64; huge.N_kv = 64; huge.S = 1 << 20; huge.n_split = 64;
    CHECK(thk_workspace_bytes(&huge, THK_OP_DECODE) > THK_STATIC_SCRATCH_BYTES);
    CHECK(thk_decode_attn_static(&huge, fake, fake, i16, fake, NULL, NULL, 0, 0, fake, NULL) == THK_ERR_SCRATCH);
  }
  thk_reload_env();
  thk_profile_next(NULL, NULL);
  for (int st = 0; st <= 7; ++st) CHECK(thk_status_string((thk_status)st) != NULL);
  CHECK(thk_last_hip_error() != NULL);
  printf("abi host check ok\n");
  return 0;
}
