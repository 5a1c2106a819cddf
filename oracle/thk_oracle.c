/*
 * thk_oracle.c -- CPU fp64 oracle for the ThinK key-cache channel-pruning path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP library is checked against.  It shares no code, header, table or helper
 * with the HIP path and must never be called from the product path; only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may load it.
 *
 * Every floating-point input element is widened exactly to double before any
 * arithmetic (bf16 and fp32 are subsets of fp64), all sums run in plain index
 * order, and nothing is blocked, fused or reordered.  OpenMP is used only to
 * spread whole independent (layer, batch, head) units over host cores.
 *
 * Tensor layouts (last index contiguous):
 *   K, V      [L][B][N_kv][S][D]
 *   Q_obs     [L][B][N_q ][S_obs][D]      (the last S_obs query rows, Sec. 3.2
 *                                          "Observation Window")
 *   score     [L][B][N_kv][D]             double
 *   idx       [L][B][N_kv][T]             int16, 0-based, ascending
 *   K_pruned  [L][B][N_kv][S][ld_keep]    same element type as K
 * Query head n reads KV head n / G, G = N_q / N_kv.
 *
 * Pins (tests/test_oracle_pins.py): explicit rank-1 Frobenius brute force,
 * closed forms for constant columns, equivariances, numpy stable argsort,
 * numpy.take, the pruning objective's triangle bound and its exact T = D-1
 * case (Sec. 3.2, Eq. 2), textbook attention at T = D and on channel-masked
 * keys, and the paper's KV-size example (Sec. 3.1) and Table 7 memory column.
 * The value-cache routines (tests/test_oracle_pins_value.py): library fp64
 * attention followed by library column norms, the uniform-attention and
 * one-hot closed forms with and without the causal mask, shift / permutation
 * / scaling invariances, and the reduction of the pruned-value decode to the
 * key-only decode on channel-masked values.
 * Parity unpinned by any value printed in the paper: the GQA aggregation
 * (sum over the G query heads of per-head Frobenius norms), the ascending
 * order of the index list, and the attention error metric are conventions of
 * this build; the paper prints no numeric score, index set or output.  The
 * same holds for the value score's optional causal mask and for reading a
 * removed value channel as a zero in the attention output.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { THKO_F32 = 0, THKO_BF16 = 1, THKO_F64 = 2 };

static size_t elem_size(int dtype) {
  return dtype == THKO_F32 ? 4 : dtype == THKO_BF16 ? 2 : 8;
}

/* Exact widening of element i of a typed array to double. */
static double ld(const void *p, int dtype, size_t i) {
  if (dtype == THKO_F32) return (double)((const float *)p)[i];
  if (dtype == THKO_F64) return ((const double *)p)[i];
  /* bf16 is the upper 16 bits of an IEEE fp32 */
  uint32_t bits = (uint32_t)((const uint16_t *)p)[i] << 16;
  float f;
  memcpy(&f, &bits, 4);
  return (double)f;
}

int thko_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* T = floor((1 - lambda) * D)  (Sec. 3.1, below Eq. 1; Eq. 2 constraint).
 * (1 - lambda) * D is evaluated in fp64; a product that lands within a few
 * ulps below an integer (0.4 * 128 style cases are exact, 0.7 * 10 is not) is
 * treated as that integer so that decimal lambdas behave as written. */
int32_t thko_keep_count(int32_t D, double lambda) {
  if (D < 1 || !(lambda >= 0.0) || !(lambda < 1.0)) return -1;
  double x = (1.0 - lambda) * (double)D;
  double r = floor(x + 1e-9);
  return (int32_t)r;
}

/* KV-cache element count 2*B*S*L*N*D (Sec. 1; Sec. 3.1) times bytes/elem. */
double thko_kv_cache_bytes(double B, double S, double L, double N, double D,
                           double bytes_per_elem) {
  return 2.0 * B * S * L * N * D * bytes_per_elem;
}

/*
 * Query-driven channel score (Sec. 3.2, Score_i[j] with the observation
 * window).  The S_obs x S matrix Q[:,c] K[:,c]^T is an outer product of two
 * column vectors, so its Frobenius norm is the product of their 2-norms; this
 * routine writes that product out.  For grouped-query attention the scores of
 * the G query heads that read one KV head are added.
 */
void thko_score(int dtype, int32_t L, int32_t B, int32_t N_q, int32_t N_kv,
                int32_t D, int64_t S, int32_t S_obs, const void *q_obs,
                const void *k, double *score) {
  const int32_t G = N_q / N_kv;
  const int64_t U = (int64_t)L * B * N_kv;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t u = 0; u < U; ++u) {
    const int64_t lb = u / N_kv; /* fused (layer, batch) index */
    const int32_t h = (int32_t)(u % N_kv);
    const size_t kbase = (size_t)u * (size_t)S * D;
    for (int32_t c = 0; c < D; ++c) {
      double kss = 0.0;
      for (int64_t s = 0; s < S; ++s) {
        double x = ld(k, dtype, kbase + (size_t)s * D + c);
        kss += x * x;
      }
      double knorm = sqrt(kss);
      double sc = 0.0;
      for (int32_t g = 0; g < G; ++g) {
        const int64_t n = (int64_t)h * G + g;
        const size_t qbase = (size_t)(lb * N_q + n) * (size_t)S_obs * D;
        double qss = 0.0;
        for (int32_t i = 0; i < S_obs; ++i) {
          double x = ld(q_obs, dtype, qbase + (size_t)i * D + c);
          qss += x * x;
        }
        sc += sqrt(qss) * knorm;
      }
      score[(size_t)u * D + c] = sc;
    }
  }
}

/*
 * The same score from the definition with no identity applied: build every
 * entry of M = Q_obs[:,c] K[:,c]^T and take sqrt(sum M^2).  O(S_obs*S) per
 * channel: tiny inputs only.
 */
void thko_score_bruteforce(int dtype, int32_t L, int32_t B, int32_t N_q,
                           int32_t N_kv, int32_t D, int64_t S, int32_t S_obs,
                           const void *q_obs, const void *k, double *score) {
  const int32_t G = N_q / N_kv;
  const int64_t U = (int64_t)L * B * N_kv;
  for (int64_t u = 0; u < U; ++u) {
    const int64_t lb = u / N_kv;
    const int32_t h = (int32_t)(u % N_kv);
    const size_t kbase = (size_t)u * (size_t)S * D;
    for (int32_t c = 0; c < D; ++c) {
      double sc = 0.0;
      for (int32_t g = 0; g < G; ++g) {
        const int64_t n = (int64_t)h * G + g;
        const size_t qbase = (size_t)(lb * N_q + n) * (size_t)S_obs * D;
        double fro2 = 0.0;
        for (int32_t i = 0; i < S_obs; ++i) {
          double qi = ld(q_obs, dtype, qbase + (size_t)i * D + c);
          for (int64_t s = 0; s < S; ++s) {
            double m = qi * ld(k, dtype, kbase + (size_t)s * D + c);
            fro2 += m * m;
          }
        }
        sc += sqrt(fro2);
      }
      score[(size_t)u * D + c] = sc;
    }
  }
}

/* Magnitude-only criterion M[n,d] = ||K[n,:,d]||_p, p in {1,2} (Eq. 1). */
void thko_score_magnitude(int dtype, int64_t U, int32_t D, int64_t S, int32_t p,
                          const void *k, double *score) {
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t u = 0; u < U; ++u) {
    const size_t kbase = (size_t)u * (size_t)S * D;
    for (int32_t c = 0; c < D; ++c) {
      double acc = 0.0;
      for (int64_t s = 0; s < S; ++s) {
        double x = ld(k, dtype, kbase + (size_t)s * D + c);
        acc += (p == 1) ? fabs(x) : x * x;
      }
      score[(size_t)u * D + c] = (p == 1) ? acc : sqrt(acc);
    }
  }
}

/*
 * Top_T selection (Sec. 3.1 I = Top_T(.,T); Sec. 3.2 I_i).  Channels are
 * ranked by score descending; equal scores rank the lower channel index
 * first.  The T best are written in ascending channel order (what applying a
 * binary keep-mask yields, Fig. 1).  Selection by repeated argmax: T passes,
 * each taking the best remaining channel.
 */
void thko_select_topk(int64_t U, int32_t D, int32_t T, const double *score,
                      int16_t *idx) {
  for (int64_t u = 0; u < U; ++u) {
    const double *sc = score + (size_t)u * D;
    unsigned char *taken = (unsigned char *)calloc((size_t)D, 1);
    for (int32_t t = 0; t < T; ++t) {
      int32_t best = -1;
      for (int32_t c = 0; c < D; ++c) {
        if (taken[c]) continue;
        if (best < 0 || sc[c] > sc[best]) best = c; /* strict >: lower index wins ties */
      }
      taken[best] = 1;
    }
    int32_t t = 0;
    for (int32_t c = 0; c < D; ++c)
      if (taken[c]) idx[(size_t)u * T + t++] = (int16_t)c;
    free(taken);
  }
}

/* K_pruned[s][t] = K[s][idx[t]] -- a byte copy of the kept channels
 * (Fig. 1: the pruned keys are what is stored; Sec. 3.3).  Columns
 * t in [T, ld_keep) of the destination are left untouched. */
void thko_compact_keys(int dtype, int64_t U, int64_t S, int32_t D, int32_t T,
                       int32_t ld_keep, const void *k, const int16_t *idx,
                       void *k_pruned) {
  const size_t e = elem_size(dtype);
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t u = 0; u < U; ++u) {
    const unsigned char *src = (const unsigned char *)k + (size_t)u * S * D * e;
    unsigned char *dst = (unsigned char *)k_pruned + (size_t)u * S * ld_keep * e;
    for (int64_t s = 0; s < S; ++s)
      for (int32_t t = 0; t < T; ++t)
        memcpy(dst + ((size_t)s * ld_keep + t) * e,
               src + ((size_t)s * D + idx[(size_t)u * T + t]) * e, e);
  }
}

/*
 * Decode attention over the two key segments (Sec. 3.3, Fig. 2; attention
 * formula of Sec. 3.2).  For query head n with KV head h = n / G:
 *   z_s     = sum_t q[n][idx[h][t]] * K_pruned[h][s][t] / sqrt(D),  s < S
 *   z_{S+j} = sum_c q[n][c]         * K_tail[h][j][c]   / sqrt(D),  j < S_tail
 * The two logit vectors are concatenated along the key axis, one softmax runs
 * over all S + S_tail entries (max subtracted first), and the output is the
 * weighted sum of the rows of [V ; V_tail].  The divisor is the square root
 * of the ORIGINAL channel count D.
 *   q, out [B][N_q][D]; K_pruned [B][N_kv][S][ld_keep]; V [B][N_kv][S][D];
 *   K_tail, V_tail [B][N_kv][S_tail_cap][D]; idx [B][N_kv][T].  out is double.
 */
void thko_decode_attn(int dtype, int32_t B, int32_t N_q, int32_t N_kv,
                      int32_t D, int64_t S, int32_t T, int32_t ld_keep,
                      const void *q, const void *k_pruned, const int16_t *idx,
                      const void *v, const void *k_tail, const void *v_tail,
                      int32_t S_tail, int32_t S_tail_cap, double *out) {
  const int32_t G = N_q / N_kv;
  const int64_t n_heads = (int64_t)B * N_q;
  const double inv_sqrt_d = 1.0 / sqrt((double)D);
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t bn = 0; bn < n_heads; ++bn) {
    const int64_t b = bn / N_q;
    const int32_t n = (int32_t)(bn % N_q);
    const int64_t u = b * N_kv + n / G; /* (batch, KV head) unit */
    const size_t qb = (size_t)bn * D;
    const int64_t n_keys = S + S_tail;
    double *z = (double *)malloc((size_t)n_keys * sizeof(double));
    for (int64_t s = 0; s < S; ++s) {
      double dot = 0.0;
      for (int32_t t = 0; t < T; ++t)
        dot += ld(q, dtype, qb + (size_t)idx[(size_t)u * T + t]) *
               ld(k_pruned, dtype, ((size_t)u * S + s) * ld_keep + t);
      z[s] = dot * inv_sqrt_d;
    }
    for (int32_t j = 0; j < S_tail; ++j) {
      double dot = 0.0;
      for (int32_t c = 0; c < D; ++c)
        dot += ld(q, dtype, qb + c) *
               ld(k_tail, dtype, ((size_t)u * S_tail_cap + j) * D + c);
      z[S + j] = dot * inv_sqrt_d;
    }
    double zmax = z[0];
    for (int64_t s = 1; s < n_keys; ++s)
      if (z[s] > zmax) zmax = z[s];
    double denom = 0.0;
    for (int64_t s = 0; s < n_keys; ++s) {
      z[s] = exp(z[s] - zmax);
      denom += z[s];
    }
    for (int32_t c = 0; c < D; ++c) {
      double acc = 0.0;
      for (int64_t s = 0; s < S; ++s)
        acc += z[s] * ld(v, dtype, ((size_t)u * S + s) * D + c);
      for (int32_t j = 0; j < S_tail; ++j)
        acc += z[S + j] * ld(v_tail, dtype, ((size_t)u * S_tail_cap + j) * D + c);
      out[qb + c] = acc / denom;
    }
    free(z);
  }
}

/*
 * Pruning objective of Eq. 2 for one head, evaluated from its definition:
 * || Q K^T - Q S K^T ||_F with S = diag(keep), Q [S_q][D], K [S_k][D] in fp64.
 * Used only by the pins that tie the greedy selection back to the objective.
 */
double thko_objective(int32_t S_q, int64_t S_k, int32_t D, const double *Q,
                      const double *K, const unsigned char *keep) {
  double fro2 = 0.0;
  for (int32_t i = 0; i < S_q; ++i)
    for (int64_t s = 0; s < S_k; ++s) {
      double full = 0.0, kept = 0.0;
      for (int32_t c = 0; c < D; ++c) {
        double prod = Q[(size_t)i * D + c] * K[(size_t)s * D + c];
        full += prod;
        if (keep[c]) kept += prod;
      }
      fro2 += (full - kept) * (full - kept);
    }
  return sqrt(fro2);
}

/*
 * Query-driven VALUE channel score (Appendix "Value Cache Pruning",
 * Score_{v,i}[j]).  For one query head: A = softmax(Q_obs K^T / sqrt(D)) is
 * S_obs x S, row-wise; column j of A V is one S_obs-vector and the Frobenius
 * norm of a vector is its 2-norm.  Written out as defined: logits, softmax
 * with the row maximum subtracted, the product with V, then the column norm.
 * K is the un-pruned key cache.  For grouped-query attention the per-head
 * norms of the G query heads that read one KV head are added (the same
 * convention as the key score).
 *
 * causal = 0: the equation as printed, every window row sees all S keys.
 * causal = 1: window row i sits at absolute position S - S_obs + i and sees
 *             keys 0 .. S - S_obs + i only, as in the prefill's own attention
 *             (the paper does not say which is meant; both are offered).
 * Requires S_obs <= S when causal.  score [L][B][N_kv][D], double.
 */
void thko_score_value(int dtype, int32_t L, int32_t B, int32_t N_q,
                      int32_t N_kv, int32_t D, int64_t S, int32_t S_obs,
                      int32_t causal, const void *q_obs, const void *k,
                      const void *v, double *score) {
  const int32_t G = N_q / N_kv;
  const int64_t U = (int64_t)L * B * N_kv;
  const double inv_sqrt_d = 1.0 / sqrt((double)D);
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t u = 0; u < U; ++u) {
    const int64_t lb = u / N_kv;
    const int32_t h = (int32_t)(u % N_kv);
    const size_t kvbase = (size_t)u * (size_t)S * D;
    double *a = (double *)malloc((size_t)S * sizeof(double));
    double *o = (double *)malloc((size_t)S_obs * D * sizeof(double));
    double *sc = score + (size_t)u * D;
    for (int32_t j = 0; j < D; ++j) sc[j] = 0.0;
    for (int32_t g = 0; g < G; ++g) {
      const int64_t n = (int64_t)h * G + g;
      const size_t qbase = (size_t)(lb * N_q + n) * (size_t)S_obs * D;
      for (int32_t i = 0; i < S_obs; ++i) {
        const int64_t n_vis = causal ? (S - S_obs + i + 1) : S;
        for (int64_t s = 0; s < n_vis; ++s) {
          double dot = 0.0;
          for (int32_t c = 0; c < D; ++c)
            dot += ld(q_obs, dtype, qbase + (size_t)i * D + c) *
                   ld(k, dtype, kvbase + (size_t)s * D + c);
          a[s] = dot * inv_sqrt_d;
        }
        double amax = a[0];
        for (int64_t s = 1; s < n_vis; ++s)
          if (a[s] > amax) amax = a[s];
        double denom = 0.0;
        for (int64_t s = 0; s < n_vis; ++s) {
          a[s] = exp(a[s] - amax);
          denom += a[s];
        }
        for (int32_t j = 0; j < D; ++j) {
          double acc = 0.0;
          for (int64_t s = 0; s < n_vis; ++s)
            acc += a[s] * ld(v, dtype, kvbase + (size_t)s * D + j);
          o[(size_t)i * D + j] = acc / denom;
        }
      }
      for (int32_t j = 0; j < D; ++j) {
        double ss = 0.0;
        for (int32_t i = 0; i < S_obs; ++i)
          ss += o[(size_t)i * D + j] * o[(size_t)i * D + j];
        sc[j] += sqrt(ss);
      }
    }
    free(a);
    free(o);
  }
}

/*
 * Decode attention with BOTH caches channel-pruned (Sec. 3.3 for the keys;
 * Appendix "Value Cache Pruning" for the values).  Logits and softmax are
 * those of thko_decode_attn.  The value rows of the pruned segment hold only
 * the T_v kept channels idx_v[0..T_v); a removed value channel contributes
 * nothing, so for output channel c
 *   out[c] = ( sum_s p_s * V_pruned[s][t]  if c == idx_v[t] for some t, else 0
 *            + sum_j p_{S+j} * V_tail[j][c] ) / denom.
 * The un-pruned tail keeps full-width value rows.
 *   V_pruned [B][N_kv][S][ld_v]; idx_v [B][N_kv][T_v]; the rest as in
 *   thko_decode_attn.  out [B][N_q][D], double.
 */
void thko_decode_attn_kv(int dtype, int32_t B, int32_t N_q, int32_t N_kv,
                         int32_t D, int64_t S, int32_t T, int32_t ld_keep,
                         int32_t T_v, int32_t ld_v, const void *q,
                         const void *k_pruned, const int16_t *idx,
                         const void *v_pruned, const int16_t *idx_v,
                         const void *k_tail, const void *v_tail,
                         int32_t S_tail, int32_t S_tail_cap, double *out) {
  const int32_t G = N_q / N_kv;
  const int64_t n_heads = (int64_t)B * N_q;
  const double inv_sqrt_d = 1.0 / sqrt((double)D);
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t bn = 0; bn < n_heads; ++bn) {
    const int64_t b = bn / N_q;
    const int32_t n = (int32_t)(bn % N_q);
    const int64_t u = b * N_kv + n / G;
    const size_t qb = (size_t)bn * D;
    const int64_t n_keys = S + S_tail;
    double *z = (double *)malloc((size_t)n_keys * sizeof(double));
    for (int64_t s = 0; s < S; ++s) {
      double dot = 0.0;
      for (int32_t t = 0; t < T; ++t)
        dot += ld(q, dtype, qb + (size_t)idx[(size_t)u * T + t]) *
               ld(k_pruned, dtype, ((size_t)u * S + s) * ld_keep + t);
      z[s] = dot * inv_sqrt_d;
    }
    for (int32_t j = 0; j < S_tail; ++j) {
      double dot = 0.0;
      for (int32_t c = 0; c < D; ++c)
        dot += ld(q, dtype, qb + c) *
               ld(k_tail, dtype, ((size_t)u * S_tail_cap + j) * D + c);
      z[S + j] = dot * inv_sqrt_d;
    }
    double zmax = z[0];
    for (int64_t s = 1; s < n_keys; ++s)
      if (z[s] > zmax) zmax = z[s];
    double denom = 0.0;
    for (int64_t s = 0; s < n_keys; ++s) {
      z[s] = exp(z[s] - zmax);
      denom += z[s];
    }
    for (int32_t c = 0; c < D; ++c) out[qb + c] = 0.0;
    for (int32_t t = 0; t < T_v; ++t) {
      double acc = 0.0;
      for (int64_t s = 0; s < S; ++s)
        acc += z[s] * ld(v_pruned, dtype, ((size_t)u * S + s) * ld_v + t);
      out[qb + (size_t)idx_v[(size_t)u * T_v + t]] = acc;
    }
    for (int32_t c = 0; c < D; ++c) {
      double acc = out[qb + c];
      for (int32_t j = 0; j < S_tail; ++j)
        acc += z[S + j] * ld(v_tail, dtype, ((size_t)u * S_tail_cap + j) * D + c);
      out[qb + c] = acc / denom;
    }
    free(z);
  }
}
