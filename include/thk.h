/*
 * thk.h -- C ABI of libthk: query-driven key-cache channel pruning (ThinK) and
 * decode attention over the pruned cache, hand-written HIP for gfx950.
 *
 * Conventions that hold for every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller; the library
 *     allocates nothing, frees nothing and never synchronises.  Work is enqueued
 *     on `stream` (a hipStream_t passed as void*; NULL = the default stream).
 *   - Base pointers must be 16-byte aligned (THK_ERR_ALIGN otherwise), and the
 *     16-byte granule that holds a tensor's last element must be readable to its
 *     end (kernels load whole aligned granules; true of any hipMalloc'ed buffer
 *     and of any sub-range of one).
 *   - Argument errors are reported synchronously and enqueue nothing.  A launch
 *     failure is reported as THK_ERR_HIP.
 *   - Dense row-major layouts, last index contiguous:
 *       K         [L][B][N_kv][S][D]         (prefill keys, input of score / compaction)
 *       V         [L][B][N_kv][S_cap][D]     (decode; S_cap = S unless set)
 *       Q_obs     [L][B][N_q ][S_obs][D]
 *       score     [L][B][N_kv][D]            float
 *       idx       [L][B][N_kv][T]            int16, 0-based, ascending
 *       K_pruned  [L][B][N_kv][S_cap][ld_keep]  element type of K; S_cap = S unless set
 *       q, out    [L][B][N_q ][D]
 *       K_tail, V_tail [L][B][N_kv][S_tail_cap][D]
 *     Query head n reads KV head n / (N_q / N_kv).
 *   - Scratch memory comes from the caller: `ws` of at least
 *     thk_workspace_bytes(shape, op) bytes, 16-byte aligned (THK_ERR_WORKSPACE).
 *   - Inputs must be finite; results for NaN/Inf inputs are unspecified.
 *   - Element types: fp32 and bf16.  D must be 128.
 *   - Built for one card: gfx950 code only, and the launch heuristics (default splits,
 *     block sizes of the prune, its graded start) assume an MI355X in SPX mode -- 256
 *     compute units at about 2.4 GHz behind one device, 8 TB/s of HBM.  On another
 *     partitioning the results are the same and the launch shapes are merely not tuned;
 *     the one rule that safety rests on -- thk_prune keeps a unit's rows on chip only if all
 *     of the unit's row blocks can be resident at once, because they wait for each other --
 *     uses the compute-unit count the current device reports (every wait is bounded besides).
 *   - The THK_* environment switches named below are for experiments and tests.  They
 *     are read once per process, on the first call that needs them; thk_reload_env()
 *     reads them again.
 */
#ifndef THK_H
#define THK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  THK_OK = 0,
  THK_ERR_NULL = 1,        /* a required pointer is NULL                       */
  THK_ERR_SHAPE = 2,       /* a size is out of range or inconsistent           */
  THK_ERR_UNSUPPORTED = 3, /* valid in principle, not built (D != 128, dtype)  */
  THK_ERR_ALIGN = 4,       /* a pointer is not 16-byte aligned                 */
  THK_ERR_WORKSPACE = 5,   /* ws is NULL or smaller than thk_workspace_bytes   */
  THK_ERR_HIP = 6,         /* the HIP runtime refused a launch                 */
  THK_ERR_SCRATCH = 7      /* thk_decode_attn_static: the shape needs more than
                              THK_STATIC_SCRATCH_BYTES of scratch                */
} thk_status;

typedef enum { THK_F32 = 0, THK_BF16 = 1 } thk_dtype;

typedef enum {
  THK_OP_SCORE = 0,  /* thk_score                       */
  THK_OP_DECODE = 1, /* thk_decode_attn                 */
  THK_OP_PRUNE = 2,  /* thk_prune                       */
  THK_OP_SCORE_VALUE = 3, /* thk_score_value            */
  THK_OP_PRUNE_VALUE = 4  /* thk_prune_value            */
} thk_op;

/* Problem statement in the paper's B x S x L x N x D terms (Sec. 1). */
typedef struct {
  int32_t L;       /* layers handled by this call, >= 1                          */
  int32_t B;       /* batch, >= 1                                                */
  int32_t N_q;     /* query heads; N_q % N_kv == 0                               */
  int32_t N_kv;    /* key/value heads                                            */
  int32_t D;       /* channels per head; must be 128                             */
  int64_t S;       /* keys in the prunable segment, >= 1                         */
  int32_t S_obs;   /* observation-window queries, 1..S (score / prune only)      */
  int32_t T;       /* channels kept, 1..D                                        */
  int32_t ld_keep; /* row stride of K_pruned in elements, T <= ld_keep <= D; 0 means
                      T (the columns past T are written as zeros and never read) */
  int32_t dtype;   /* thk_dtype of Q, K, V, K_pruned, out                        */
  int32_t n_split; /* pieces the S axis is cut into per unit; 0 = library choice */
  int32_t S_recent;/* prune: the last S_recent of the S scored keys are NOT compacted    */
                   /* (they stay at full width with the caller); 0 <= S_recent < S       */
  int64_t S_cap;   /* rows allocated per unit in K_pruned and V (cache capacity), >= the */
                   /* rows in use; 0 means dense: S (S - S_recent for thk_prune's output)*/
} thk_shape;

/* Library version, major*10000 + minor*100 + patch. */
int32_t thk_version(void);

/* Reads the THK_* environment switches again (they are otherwise read once per process).
 * A hook for tests and experiments; not meant to be called while other threads are inside
 * the library's entry points with a call half planned (each entry point takes one
 * consistent snapshot, so the worst case is a call planned with the previous values). */
void thk_reload_env(void);

/* Static string for a status code. */
const char *thk_status_string(thk_status st);

/* The HIP runtime's message for the launch error behind the calling thread's most recent
 * THK_ERR_HIP ("no error" if there was none).  An entry point that launches first consumes
 * any error the thread's earlier HIP calls left pending, so THK_ERR_HIP is about its own
 * launches only. */
const char *thk_last_hip_error(void);

/*
 * T = floor((1 - lambda) * D): the number of channels kept at pruning ratio
 * lambda (Sec. 3.1, below Eq. 1; constraint of Eq. 2).  Evaluated in fp64; a
 * product within 1e-9 below an integer counts as that integer.  Returns -1 for
 * D < 1 or lambda outside [0, 1).  Host-only arithmetic.
 */
int32_t thk_keep_count(int32_t D, double lambda);

/*
 * Bytes of caller-provided scratch that `op` needs for `shape` (including the
 * shape's n_split; 0 there means the library's own choice, which this function
 * reproduces).  Returns 0 for an invalid shape.  Host-only arithmetic.
 */
size_t thk_workspace_bytes(const thk_shape *shape, int32_t op);

/* The n_split the library would use for `op` when shape->n_split == 0. */
int32_t thk_default_split(const thk_shape *shape, int32_t op);

/* How thk_prune would run `shape`: 2 = one launch that keeps the rows on chip between the
 * score and the compaction (K read once), 1 = one launch that reads the rows twice, 0 = the
 * staged three-kernel form (or an invalid shape).  Host-only. */
int32_t thk_prune_is_fused(const thk_shape *shape);

/* Kernels a thk_prune call on `shape` enqueues: 1 when the rows are held on chip and the call
 * is short -- at most two rounds of resident blocks, three for units of more than 64 blocks (the
 * kernel then initialises its own hand-off state, computes the query norms in a prologue block
 * per unit, and serves blocks whose wait ran out by itself); 3 for longer calls, with
 * THK_PRUNE_LAUNCH=classic, or for blocks that re-read their rows (a kernel in front that
 * clears the state and computes the query norms, one behind that compacts what was left
 * undone); 3 per group of units in the staged form; 0 for an invalid shape.  Host-only. */
int32_t thk_prune_launches(const thk_shape *shape);

/* 1 if thk_decode_attn (T_v == 0) or thk_decode_attn_kv (value rows of T_v kept channels,
 * ld_v elements apart) would run `shape` on the matrix-core kernel k_decode_mq, 0 if on the
 * general kernel k_decode (or the shape is invalid).  Host-only; honours THK_DECODE_MFMA. */
int32_t thk_decode_on_matrix_cores(const thk_shape *shape, int32_t T_v, int32_t ld_v);

/*
 * Query-driven channel score (Sec. 3.2, Score_i[j] = ||Q_i[-S_obs:, j] K_i[:, j]^T||_F).
 * The matrix is an outer product of two columns, so the score is
 * ||Q_obs[:, c]||_2 * ||K[:, c]||_2; with grouped queries the scores of the
 * N_q / N_kv query heads that read one KV head are added.  No 1/sqrt(D), mask
 * or softmax enters.  Squares are summed in fp32 chains of at most 16 terms,
 * merged and square-rooted in fp64, and the product is rounded once to float.
 *   in : q_obs, k (device)           out: score (device, float)
 *   ws : THK_OP_SCORE bytes.
 */
thk_status thk_score(const thk_shape *shape, const void *q_obs, const void *k,
                     float *score, void *ws, size_t ws_bytes, void *stream);

/*
 * Magnitude-only criterion M[n, d] = ||K[n, :, d]||_p, p = 1 or 2 (Eq. 1), in
 * the same layout and precision as thk_score; q_obs is not read.
 */
thk_status thk_score_magnitude(const thk_shape *shape, const void *k, int32_t p,
                               float *score, void *ws, size_t ws_bytes,
                               void *stream);

/*
 * Query-driven VALUE channel score (Appendix "Value Cache Pruning"):
 *   Score_v[j] = || softmax(Q_obs K^T / sqrt(D)) V[:, j] ||_2 ,
 * the norm of channel j of the observation window's attention output, added
 * over the N_q / N_kv query heads that read one KV head.  K is the un-pruned
 * key cache.  causal = 0 is the equation as printed (every window row sees all
 * S keys); causal = 1 lets window row i, the token at position S - S_obs + i,
 * see keys 0 .. S - S_obs + i as in the prefill's own attention.  Logits are
 * accumulated in fp32 on the matrix cores and the softmax runs in fp32.  For
 * bf16 tensors each probability multiplies V as two bf16 terms (hi + lo, within
 * 2^-18 of the fp32 value; the row sum takes the fp32 values); for fp32 tensors
 * every product is fp32.  Column norms are summed in fp64 and rounded once to
 * float.  Scores agree with an fp64 evaluation to about 1e-6 relative.
 * Feed the result to thk_select_topk for the value index list and to
 * thk_compact_keys (which copies channels of any [S][D] cache) for the pruned
 * values.
 *   in : q_obs, k, v (device)        out: score_v (device, float, [L][B][N_kv][D])
 *   ws : THK_OP_SCORE_VALUE bytes.
 */
thk_status thk_score_value(const thk_shape *shape, const void *q_obs, const void *k,
                           const void *v, int32_t causal, float *score_v, void *ws,
                           size_t ws_bytes, void *stream);

/*
 * End-of-prefill prune of the VALUE cache (Appendix "Value Cache Pruning"):
 * thk_score_value + thk_select_topk + thk_compact_keys applied to V in one call.
 * The shape's T, ld_keep, S_recent and S_cap describe the pruned VALUE cache here
 * (T = channels kept, the paper's T for I_i = Top_T(Score_v, T)).  `score_v` may
 * be NULL (then it lives in ws).  Calls of at least 16 rounds of resident blocks
 * (12288 blocks of 512 bf16 rows) compact V with the kernels of thk_prune, the index
 * list given: their hand-off makes the blocks of a unit store together, which the
 * memory takes better than stores scattered between other units' loads; shorter
 * calls use the kernel of thk_compact_keys.  Same bytes either way.
 * Environment (experiments and tests): THK_VALUE_COMPACT = flat | burst.
 *   in : q_obs, k, v (device)   out: score_v (float), idx_v (int16), v_pruned
 *   ws : THK_OP_PRUNE_VALUE bytes.
 */
thk_status thk_prune_value(const thk_shape *shape, const void *q_obs, const void *k,
                           const void *v, int32_t causal, float *score_v, int16_t *idx_v,
                           void *v_pruned, void *ws, size_t ws_bytes, void *stream);

/*
 * Top_T selection (Sec. 3.1 I = Top_T(M, T); Sec. 3.2 I_i): per unit the T
 * channels of largest score, equal scores resolved towards the lower channel
 * index, written in ascending channel order (the order a binary keep-mask
 * yields, Fig. 1).  Scores are compared as floats exactly as given.
 *   in : score (device, float)       out: idx (device, int16)
 */
thk_status thk_select_topk(const thk_shape *shape, const float *score,
                           int16_t *idx, void *stream);

/*
 * K_pruned[s][t] = K[s][idx[t]] -- a bit copy of the kept channels (Fig. 1;
 * Sec. 3.3 "pruned keys with a reduced channel size") for rows s < S - S_recent.
 * Columns [T, ld_keep) of the rows written are set to zero.  idx entries must lie in [0, D).
 */
thk_status thk_compact_keys(const thk_shape *shape, const void *k,
                            const int16_t *idx, void *k_pruned, void *stream);

/*
 * End-of-prefill prune = thk_score + thk_select_topk + thk_compact_keys in one
 * call.  A single kernel does all three steps (alone for short calls, between a
 * small set-up and a small repair kernel for long ones: see thk_prune_launches),
 * for dense or padded rows, any S, any unit pitch: a block takes 512 bf16 or 256 fp32 rows of a unit (256 or 128
 * for calls small enough to stay within two blocks per compute unit), keeps
 * them on chip while the unit's index list is being decided, and compacts them
 * from there, so K is read from memory once.  Units of more blocks than are
 * resident on the chip at once (768 blocks of 512 bf16 rows: S > 393216) take
 * the three kernels one after the other.  Scores agree with thk_score to fp64
 * summation order (the last float bit can differ).  `score` may be NULL (then
 * it lives in ws).
 * Environment (for experiments and tests): THK_PRUNE_LAUNCH = classic (three launches:
 * state and query norms, the main kernel, repair) | solo (one launch; the default for
 * short calls whose rows are held on chip); THK_PRUNE_PATH =
 * staged | fused | reread (the one-kernel form with the rows read twice);
 * THK_PRUNE_BLOCK_ROWS (rows per block; 128, 256 and 512 are held on chip),
 * THK_PRUNE_HOLD_ROWS (largest default block), THK_PRUNE_MAX_BLOCKS (blocks
 * per unit beyond which the staged form is taken), THK_PRUNE_SPIN_LIMIT (polls
 * before a waiting block leaves its rows to the repair kernel or to the unit's
 * finisher; 0 forces that path), THK_PRUNE_STAGGER_NS (spacing of the first round's unit starts; 0 =
 * none), THK_PRUNE_GROUP_MIB (bytes of K per group of units in the staged form),
 * THK_PRUNE_PROLOGUE_DELAY_US (single-launch form: the unit's prologue block starts
 * that late, at most 500 us, so that the row blocks find their arrival counters not
 * yet initialised and have to wait for them -- a path that otherwise needs an
 * unlucky schedule).
 *   ws : THK_OP_PRUNE bytes.
 */
thk_status thk_prune(const thk_shape *shape, const void *q_obs, const void *k,
                     float *score, int16_t *idx, void *k_pruned, void *ws,
                     size_t ws_bytes, void *stream);

/*
 * Decode attention over the two key segments (Sec. 3.3, Fig. 2, with the
 * attention formula of Sec. 3.2).  Per query head n with KV head h:
 *   z_s     = (sum_t q[n][idx[h][t]] * K_pruned[h][s][t]) / sqrt(D),   s < S
 *   z_{S+j} = (sum_c q[n][c] * K_tail[h][j][c]) / sqrt(D),             j < s_tail
 *   out[n]  = softmax(z) . [V ; V_tail]
 * one softmax over all S + s_tail logits; sqrt(D) uses the original D.  fp32
 * arithmetic; out has the input element type (bf16: round to nearest even).
 * k_tail may be NULL iff s_tail == 0; 0 <= s_tail <= s_tail_cap.  v_tail == NULL
 * with s_tail > 0 selects the unified value cache: the tail's value rows are rows
 * [S, S + s_tail) of v (needs S_cap >= S + s_tail).
 * S_obs in the shape is ignored.  With n_split > 1 partial (max, sum, acc[D])
 * states go through ws and are merged in split order, so repeated calls give
 * identical bits: by a second kernel, or -- for small calls (at most 16 pieces, at
 * most two query heads per block, at most two blocks per compute unit) -- inside the
 * one launch by the block that finishes last for a head group (the blocks signal
 * through per-piece flag words in ws that carry a nonce drawn per call; no
 * read-modify-write, nothing in ws has to be cleared beforehand).
 * THK_DECODE_MERGE = kernel | fused in the environment overrides the choice.
 * bf16 caches with N_q / N_kv >= 3 and a key row pitch (ld_keep, or T when rows are
 * dense) that is a multiple of 4 elements run the two products on the matrix cores,
 * here and in thk_decode_attn_kv: four or eight query heads share every key and
 * value byte a block reads (probabilities as two bf16 terms, exact to 2^-16;
 * accumulation in fp32; elements of a padded row past T are masked, whatever they
 * hold).  For T that is not a multiple of 4 (51, 89, ...) a pitch rounded up to one
 * therefore pays with several query heads per KV head. THK_DECODE_MFMA=0 in the environment
 * (for experiments and tests) keeps them on the general kernel.
 *   ws : THK_OP_DECODE bytes.
 */
thk_status thk_decode_attn(const thk_shape *shape, const void *q,
                           const void *k_pruned, const int16_t *idx,
                           const void *v, const void *k_tail,
                           const void *v_tail, int32_t s_tail,
                           int32_t s_tail_cap, void *out, void *ws,
                           size_t ws_bytes, void *stream);

/*
 * Decode attention with the VALUE cache channel-pruned as well (Appendix "Value
 * Cache Pruning"; keys as in thk_decode_attn).  V_pruned [L][B][N_kv][S_cap][ld_v]
 * holds, per row, the T_v channels idx_v[0 .. T_v) of the values (what
 * thk_compact_keys writes from V with the value index list and ld_keep = ld_v).
 * A removed channel contributes nothing:
 *   out[n][c] = ( sum_s p_s V_pruned[h][s][t]   if c == idx_v[h][t], else 0
 *               + sum_j p_{S+j} V_tail[h][j][c] ) / sum p
 * The tail keeps full-width rows (v_tail is required when s_tail > 0).
 * 1 <= T_v <= ld_v <= D; ld_v must be a multiple of 4 (THK_ERR_UNSUPPORTED
 * otherwise); idx_v [L][B][N_kv][T_v] int16, ascending, 16-byte aligned.
 *   ws : THK_OP_DECODE bytes.
 */
thk_status thk_decode_attn_kv(const thk_shape *shape, const void *q, const void *k_pruned,
                              const int16_t *idx, const void *v_pruned,
                              const int16_t *idx_v, int32_t T_v, int32_t ld_v,
                              const void *k_tail, const void *v_tail, int32_t s_tail,
                              int32_t s_tail_cap, void *out, void *ws, size_t ws_bytes,
                              void *stream);

/*
 * thk_decode_attn for callers that cannot allocate or carry a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same kernels, same split and therefore the same bits as thk_decode_attn with
 * n_split as given in the shape (0 = library choice), but the split partials go to a
 * buffer of THK_STATIC_SCRATCH_BYTES that is part of the library's device image (a
 * file-scope device array; each GPU the library runs on holds its own copy until the
 * process ends).  The call allocates nothing and frees nothing.  The array's address on a
 * device is looked up on the first call made with that device current (one runtime query,
 * no allocation; make that first call outside graph capture).
 *   - A shape whose thk_workspace_bytes(shape, THK_OP_DECODE) exceeds
 *     THK_STATIC_SCRATCH_BYTES is rejected with THK_ERR_SCRATCH and nothing is enqueued
 *     (the five workloads of the benchmark need 0.07 - 2.1 MiB).
 *   - All calls on one GPU share that GPU's buffer: calls whose execution may overlap
 *     (different streams, concurrent graphs) race on it and must be ordered by the caller.
 *     Nothing in it needs to start at zero; a call overwrites every record it later reads.
 */
#define THK_STATIC_SCRATCH_BYTES (8u << 20)
thk_status thk_decode_attn_static(const thk_shape *shape, const void *q,
                                  const void *k_pruned, const int16_t *idx,
                                  const void *v, const void *k_tail,
                                  const void *v_tail, int32_t s_tail,
                                  int32_t s_tail_cap, void *out, void *stream);

/*
 * Append one newly decoded token per (layer, batch, KV head) to the unpruned
 * tail segment (Sec. 3.3: new keys stay at full D):
 *   K_tail[..][s_tail][:] = k_new[..][:],  V_tail[..][s_tail][:] = v_new[..][:]
 * k_new, v_new [L][B][N_kv][D].  Requires 0 <= s_tail < s_tail_cap.  The caller
 * then attends with s_tail + 1.
 */
thk_status thk_tail_append(const thk_shape *shape, const void *k_new,
                           const void *v_new, void *k_tail, void *v_tail,
                           int32_t s_tail, int32_t s_tail_cap, void *stream);

/*
 * Cache growth (Sec. 3.3: recent and newly generated keys stay un-pruned; Appendix
 * "Implementation with quantization": a residual buffer of new tokens is pruned
 * with the stored mask and appended once it is full).
 *
 * thk_compact_rows: K_pruned[u][dst_row0 + r][t] = src[u][src_row0 + r][idx[u][t]],
 *   r < n_rows, for every unit u.  src has src_unit_rows rows of D per unit (the
 *   prefill K with src_unit_rows = S, or a tail buffer with src_unit_rows = cap);
 *   K_pruned has S_cap rows per unit (shape->S_cap, 0 = shape->S).  shape->S is
 *   not otherwise used.  Requires dst_row0 + n_rows <= rows per unit of K_pruned.
 * thk_copy_rows: dst[u][dst_row0 + r][:] = src[u][src_row0 + r][:], r < n_rows, rows of
 *   D elements.  src and dst may be the same buffer when dst_row0 <= src_row0.
 * thk_cache_append: K_tail[u][s_tail] = k_new[u]; V[u][S + s_tail] = v_new[u]
 *   (unified value cache, S_cap rows per unit; needs S + s_tail < S_cap).
 * thk_tail_flush: the n_flush oldest tail keys are compacted with the stored index
 *   list into K_pruned rows [S, S + n_flush) and the remaining s_tail - n_flush tail
 *   rows move to the front of the tail.  With a separate value tail (v, v_tail not
 *   NULL) the flushed value rows are copied into V rows [S, S + n_flush) and v_tail
 *   is shifted likewise; with the unified value cache pass v = v_tail = NULL.  The
 *   caller then uses S + n_flush and s_tail - n_flush.
 */
thk_status thk_compact_rows(const thk_shape *shape, const void *src, int64_t src_unit_rows,
                            int64_t src_row0, const int16_t *idx, void *k_pruned,
                            int64_t dst_row0, int64_t n_rows, void *stream);
thk_status thk_copy_rows(const thk_shape *shape, const void *src, int64_t src_unit_rows,
                         int64_t src_row0, void *dst, int64_t dst_unit_rows, int64_t dst_row0,
                         int64_t n_rows, void *stream);
thk_status thk_cache_append(const thk_shape *shape, const void *k_new, const void *v_new,
                            void *k_tail, void *v, int32_t s_tail, int32_t s_tail_cap,
                            void *stream);
thk_status thk_tail_flush(const thk_shape *shape, const int16_t *idx, void *k_pruned,
                          void *k_tail, void *v, void *v_tail, int32_t s_tail,
                          int32_t s_tail_cap, int32_t n_flush, void *stream);

/*
 * Timing hook for benchmarks: the main kernel of the NEXT call made by this host
 * thread (the one-launch prune kernel, or the compaction kernel of the staged
 * form; the attention kernel, not the split merge; the value-score attention
 * kernel) is launched with `ev_start` and `ev_stop` attached to it, so that the
 * interval between the two events is that kernel's own duration -- begin to end
 * of its execution, as a profiler reports it; nothing extra enters the stream.
 * Both are hipEvent_t handles passed as void*, created by the caller with
 * timing enabled; the pair is used once.  Passing NULL for either cancels a
 * pending pair.  Such a launch costs the host about 12 us more than a plain
 * one; do not arm the hook while the stream is being captured into a graph.
 */
void thk_profile_next(void *ev_start, void *ev_stop);

/*
 * Benchmark aid, not part of the method: a kernel that does nothing but stream
 * memory, so that a prune or decode call can be set against what the chip gives
 * a plain read, copy or write of the SAME number of bytes (a launch of a few
 * hundred MB pays its start and its end: the rate of a long stream is not its
 * ceiling).  Each of the n_blocks blocks owns 128 KiB of `src` and w * 4 KiB of
 * `dst` (16 bytes per thread and access, non-temporal like the library's own
 * streams, all of a block's loads in flight at once):
 *   THK_STREAM_READ   reads src (n_blocks * 128 KiB); dst may be NULL, w is ignored
 *   THK_STREAM_COPY   reads src, keeps the block's bytes in registers, then writes
 *                     the first w / 32 of them to dst -- the traffic of a prune
 *                     block with w / 32 = T / D, without the exchange between blocks
 *   THK_STREAM_WRITE  writes dst (n_blocks * w * 4 KiB); src may be NULL
 * src, dst: device pointers, 16-byte aligned, owned by the caller, at least
 * the sizes above; 1 <= n_blocks <= 2^31 - 1, 0 <= w <= 32 (1 <= w for COPY and
 * WRITE).  THK_ERR_NULL / THK_ERR_ALIGN / THK_ERR_SHAPE on misuse (nothing is
 * enqueued then), THK_ERR_HIP if the launch fails.  Enqueues one kernel on `stream`;
 * thk_profile_next applies to it.
 */
enum { THK_STREAM_READ = 0, THK_STREAM_COPY = 1, THK_STREAM_WRITE = 2 };
thk_status thk_bench_stream(int32_t mode, const void *src, void *dst, int64_t n_blocks, int32_t w, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* THK_H */
