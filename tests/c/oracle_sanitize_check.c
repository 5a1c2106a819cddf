/* Memory- and undefined-behaviour check of the CPU oracle: every routine of oracle/thk_oracle.c
 * is called on buffers malloc'ed to EXACTLY the sizes its contract states, for the three element
 * types, on small shapes that include the edge cases (one key, T == D, a full tail, padded
 * pitches, several query heads per KV head).  Built together with thk_oracle.c by
 * tests/test_oracle_pins.py with gcc -fsanitize=address,undefined -fno-sanitize-recover=all: a
 * read or write one element past a buffer, a signed overflow or a misaligned access aborts the
 * program.  Values are not judged here (the pins do that); the outputs are only summed so that
 * nothing is optimised away. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int thko_max_threads(void);
int32_t thko_keep_count(int32_t D, double lambda);
double thko_kv_cache_bytes(double B, double S, double L, double N, double D, double bytes_per_elem);
void thko_score(int dtype, int32_t L, int32_t B, int32_t N_q, int32_t N_kv, int32_t D, int64_t S, int32_t S_obs,
                const void *q_obs, const void *k, double *score);
void thko_score_bruteforce(int dtype, int32_t L, int32_t B, int32_t N_q, int32_t N_kv, int32_t D, int64_t S,
                           int32_t S_obs, const void *q_obs, const void *k, double *score);
void thko_score_magnitude(int dtype, int64_t U, int32_t D, int64_t S, int32_t p, const void *k, double *score);
void thko_select_topk(int64_t U, int32_t D, int32_t T, const double *score, int16_t *idx);
void thko_compact_keys(int dtype, int64_t U, int64_t S, int32_t D, int32_t T, int32_t ld_keep, const void *k,
                       const int16_t *idx, void *k_pruned);
void thko_decode_attn(int dtype, int32_t B, int32_t N_q, int32_t N_kv, int32_t D, int64_t S, int32_t T,
                      int32_t ld_keep, const void *q, const void *k_pruned, const int16_t *idx, const void *v,
                      const void *k_tail, const void *v_tail, int32_t S_tail, int32_t S_tail_cap, double *out);
double thko_objective(int32_t S_q, int64_t S_k, int32_t D, const double *Q, const double *K,
                      const unsigned char *keep);
void thko_score_value(int dtype, int32_t L, int32_t B, int32_t N_q, int32_t N_kv, int32_t D, int64_t S,
                      int32_t S_obs, int32_t causal, const void *q_obs, const void *k, const void *v, double *score);
void thko_decode_attn_kv(int dtype, int32_t B, int32_t N_q, int32_t N_kv, int32_t D, int64_t S, int32_t T,
                         int32_t ld_keep, int32_t T_v, int32_t ld_v, const void *q, const void *k_pruned,
                         const int16_t *idx, const void *v_pruned, const int16_t *idx_v, const void *k_tail,
                         const void *v_tail, int32_t S_tail, int32_t S_tail_cap, double *out);

static uint64_t rng = 0x9e3779b97f4a7c15ull;
static double uniform(void) {   /* in (-1, 1) */
  rng = rng * 6364136223846793005ull + 1442695040888963407ull;
  return (double)(int64_t)(rng >> 11) / (double)(1ll << 52) - 1.0;
}
static size_t esize(int dt) { return dt == 0 ? 4 : dt == 1 ? 2 : 8; }

/* n elements of type dt (0 fp32, 1 bf16, 2 fp64) in a buffer of exactly n elements */
static void *tensor(int dt, size_t n) {
  void *p = malloc(n * esize(dt) ? n * esize(dt) : 1);
  for (size_t i = 0; i < n; ++i) {
    const double x = 2.0 * uniform();
    if (dt == 0) ((float *)p)[i] = (float)x;
    else if (dt == 2) ((double *)p)[i] = x;
    else { float f = (float)x; uint32_t u; memcpy(&u, &f, 4); ((uint16_t *)p)[i] = (uint16_t)(u >> 16); }
  }
  return p;
}
static double sum(const double *x, size_t n) { double s = 0; for (size_t i = 0; i < n; ++i) s += x[i]; return s; }

static double one_shape(int dt, int L, int B, int N_q, int N_kv, int D, int64_t S, int S_obs, int T, int ld, int T_v,
                        int ld_v, int S_tail, int cap) {
  const int64_t U = (int64_t)L * B * N_kv, H = (int64_t)L * B * N_q;
  double acc = 0;
  void *q_obs = tensor(dt, (size_t)H * S_obs * D), *k = tensor(dt, (size_t)U * S * D), *v = tensor(dt, (size_t)U * S * D);
  double *score = malloc(sizeof(double) * U * D), *score2 = malloc(sizeof(double) * U * D);
  thko_score(dt, L, B, N_q, N_kv, D, S, S_obs, q_obs, k, score);
  thko_score_bruteforce(dt, L, B, N_q, N_kv, D, S, S_obs, q_obs, k, score2);
  acc += sum(score, U * D) - sum(score2, U * D);
  thko_score_magnitude(dt, U, D, S, 1, k, score2); acc += sum(score2, U * D);
  thko_score_magnitude(dt, U, D, S, 2, k, score2); acc += sum(score2, U * D);
  int16_t *idx = malloc(sizeof(int16_t) * U * T), *idx_v = malloc(sizeof(int16_t) * U * T_v);
  thko_select_topk(U, D, T, score, idx);
  for (int causal = 0; causal < 2; ++causal) {
    thko_score_value(dt, L, B, N_q, N_kv, D, S, S_obs, causal, q_obs, k, v, score2);
    acc += sum(score2, U * D);
  }
  thko_select_topk(U, D, T_v, score2, idx_v);
  void *kp = malloc((size_t)U * S * ld * esize(dt)), *vp = malloc((size_t)U * S * ld_v * esize(dt));
  thko_compact_keys(dt, U, S, D, T, ld, k, idx, kp);
  thko_compact_keys(dt, U, S, D, T_v, ld_v, v, idx_v, vp);
  /* decode works on one layer: B * N_q heads, B * N_kv units */
  void *q = tensor(dt, (size_t)B * N_q * D), *kt = tensor(dt, (size_t)B * N_kv * (cap ? cap : 1) * D),
       *vt = tensor(dt, (size_t)B * N_kv * (cap ? cap : 1) * D);
  double *out = malloc(sizeof(double) * B * N_q * D);
  thko_decode_attn(dt, B, N_q, N_kv, D, S, T, ld, q, kp, idx, v, cap ? kt : NULL, cap ? vt : NULL, S_tail, cap, out);
  acc += sum(out, (size_t)B * N_q * D);
  thko_decode_attn_kv(dt, B, N_q, N_kv, D, S, T, ld, T_v, ld_v, q, kp, idx, vp, idx_v, cap ? kt : NULL,
                      cap ? vt : NULL, S_tail, cap, out);
  acc += sum(out, (size_t)B * N_q * D);
  free(q_obs); free(k); free(v); free(score); free(score2); free(idx); free(idx_v); free(kp); free(vp);
  free(q); free(kt); free(vt); free(out);
  return acc;
}

int main(void) {
  double acc = 0;
  acc += thko_max_threads() + thko_keep_count(128, 0.4) + thko_keep_count(10, 0.3) + thko_keep_count(1, 0.0);
  acc += thko_kv_cache_bytes(13, 2048, 32, 32, 128, 2);
  for (int dt = 0; dt < 3; ++dt) {
    /*             L  B N_q N_kv   D    S S_obs   T  ld T_v ld_v tail cap */
    acc += one_shape(dt, 1, 1, 1, 1, 128, 1, 1, 128, 128, 128, 128, 0, 0);     /* one key, nothing pruned */
    acc += one_shape(dt, 2, 2, 4, 2, 128, 37, 5, 76, 76, 51, 52, 3, 4);        /* odd sizes, padded value rows */
    acc += one_shape(dt, 1, 3, 8, 2, 16, 9, 9, 1, 3, 15, 16, 2, 2);            /* one kept channel, full tail, S_obs == S */
    acc += one_shape(dt, 1, 1, 6, 6, 8, 64, 32, 7, 7, 8, 8, 0, 5);             /* empty tail with capacity */
  }
  {
    double *Q = tensor(2, 4 * 8), *K = tensor(2, 11 * 8);
    unsigned char keep[8] = {1, 0, 1, 1, 0, 0, 1, 1};
    acc += thko_objective(4, 11, 8, Q, K, keep);
    free(Q); free(K);
  }
  printf("oracle sanitize check ok (%.6g)\n", acc);
  return 0;
}
