// Internal declarations shared by the libthk translation units (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <atomic>

#include "thk.h"

namespace thk {

constexpr int kD = 128;     // channels per head (the only size built)
constexpr int kWave = 64;   // wavefront width on CDNA4
constexpr int kCUs = 256;   // compute units of an MI355X

// 16 bytes as a native vector: register arrays of this type are promoted to VGPRs reliably
// (arrays of the uint4 class type are copied member-wise through memcpy and can end up in scratch).
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// A 16-byte load of data that is read once and never again (the K and V streams): the
// non-temporal hint keeps it from allocating in the L2 and the memory-side cache, which on
// MI355X lifts a pure read stream from ~6.3 to ~7.1 TB/s.
__device__ __forceinline__ u32x4 ld_stream(const u32x4 *p) { return __builtin_nontemporal_load(p); }
// ... and the matching store for data this launch will not read back (a few percent on mixed
// read / write streams).
__device__ __forceinline__ void st_stream(u32x4 *p, u32x4 v) { __builtin_nontemporal_store(v, p); }

// ---- values of the lane 16 or 32 lanes away, without the LDS crossbar ------
// v_permlane16_swap / v_permlane32_swap with both operands x: a = x of the pair's lane in the even
// 16-lane row (in the lower half of the wave), b = x of the other one; both lanes of a pair
// receive the same (a, b), so a + b has the same bits in both.
struct LanePair { float a, b; };
__device__ __forceinline__ LanePair pair16(float x) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return {__uint_as_float(r[0]), __uint_as_float(r[1])};
}
__device__ __forceinline__ LanePair pair32(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return {__uint_as_float(r[0]), __uint_as_float(r[1])};
}
// x + (x of the lane OFF away) for a double, OFF = 16 or 32: the same bits as x + __shfl_xor(x, OFF)
// (the sum of two values does not depend on their order), by four register swaps instead of
// four trips through the LDS crossbar.
template <int OFF>
__device__ __forceinline__ double add_across(double x) {
  static_assert(OFF == 16 || OFF == 32, "one swap instruction exists for each of these distances");
  const unsigned long long bits = (unsigned long long)__double_as_longlong(x);
  const unsigned lo = (unsigned)bits, hi = (unsigned)(bits >> 32);
  unsigned alo, blo, ahi, bhi;
  if constexpr (OFF == 16) {
    const auto rl = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
    const auto rh = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
    alo = rl[0]; blo = rl[1]; ahi = rh[0]; bhi = rh[1];
  } else {
    const auto rl = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
    const auto rh = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
    alo = rl[0]; blo = rl[1]; ahi = rh[0]; bhi = rh[1];
  }
  const double a = __longlong_as_double((long long)(((unsigned long long)ahi << 32) | alo));
  const double b = __longlong_as_double((long long)(((unsigned long long)bhi << 32) | blo));
  return a + b;
}
// A per-lane double summed over the lane groups of LPR lanes each (LPR = 16 or 32) of a wavefront.
template <int LPR>
__device__ __forceinline__ double add_lane_groups(double x) {
  static_assert(LPR == 16 || LPR == 32, "lane groups of a 16-byte-chunk row: 16 (bf16) or 32 (fp32) lanes");
  if constexpr (LPR == 16) x = add_across<16>(x);
  return add_across<32>(x);
}

// ---- element access ------------------------------------------------------
// A 16-byte chunk holds VEC elements; unpack() widens them to float exactly.
template <int DT> struct Elem;
template <> struct Elem<THK_F32> {
  static constexpr int EB = 4, VEC = 4;
  using Bits = uint32_t;
  template <class V4> __device__ static inline void unpack(const V4 &r, float (&f)[4]) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
  __device__ static inline float load1(const void *p, size_t i) { return ((const float *)p)[i]; }
  __device__ static inline void store1(void *p, size_t i, float x) { ((float *)p)[i] = x; }
};
template <> struct Elem<THK_BF16> {
  static constexpr int EB = 2, VEC = 8;
  using Bits = uint16_t;
  template <class V4> __device__ static inline void unpack(const V4 &r, float (&f)[8]) {
    f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
    f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
    f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
    f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
  }
  __device__ static inline float load1(const void *p, size_t i) {
    return __uint_as_float((uint32_t)((const uint16_t *)p)[i] << 16);
  }
  // fp32 -> bf16, round to nearest even (finite inputs)
  __device__ static inline uint16_t round_bf16(float x) {
    uint32_t u = __float_as_uint(x);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
  }
  __device__ static inline void store1(void *p, size_t i, float x) { ((uint16_t *)p)[i] = round_bf16(x); }
};

// ---- one-shot timing hook (thk_profile_next) ----
// The launch of a call's main kernel.  With an event pair pending the kernel goes out through
// hipExtLaunchKernel, which stamps the two events with the kernel's own begin and end (nothing
// extra enters the queue, so the interval is the kernel's duration as a profiler reports it),
// and the pair is consumed; otherwise a plain launch.  `args` as for hipLaunchKernel.
hipError_t launch_main_kernel(const void *fn, dim3 grid, dim3 block, void **args, size_t lds, hipStream_t st);

// hipGetLastError() reports the calling thread's most recent unconsumed error, whoever caused
// it; a launcher consumes whatever is pending first so that what it returns is about its own
// launches only.
inline void clear_stale_hip_error() { (void)hipGetLastError(); }

// ---- environment switches (experiments and tests) ----
// Read from the environment ONCE per process, on first use; thk_reload_env() reads them again.
struct EnvSwitches {
  char prune_path;        // first letter of THK_PRUNE_PATH ('s'taged, 'f'used, 'r'eread), 0 = unset
  long group_mib;         // THK_PRUNE_GROUP_MIB, <= 0 = unset
  long block_rows;        // THK_PRUNE_BLOCK_ROWS, <= 0 = unset
  long hold_rows;         // THK_PRUNE_HOLD_ROWS, <= 0 = unset
  long max_blocks;        // THK_PRUNE_MAX_BLOCKS, < 0 = unset
  long spin_limit;        // THK_PRUNE_SPIN_LIMIT, < 0 = unset
  bool stagger_set;       // THK_PRUNE_STAGGER_NS present
  double stagger_ns;
  bool decode_mfma_off;   // THK_DECODE_MFMA=0
  char prune_launch;      // first letter of THK_PRUNE_LAUNCH ('c'lassic: three launches, 's'olo: one), 0 = unset
  long prologue_delay_us; // THK_PRUNE_PROLOGUE_DELAY_US (test hook of the single-launch prune), <= 0 = none
  char decode_merge;      // first letter of THK_DECODE_MERGE ('k'ernel: a second launch merges the split
                          // records, 'f'used: the last block of a head group merges), 0 = unset
  char value_compact;     // first letter of THK_VALUE_COMPACT ('f'lat: the plain compaction kernel,
                          // 'b'urst: the one-pass prune kernels with the list given), 0 = unset
};
const EnvSwitches &env_switches();

// hipFuncAttributeMaxDynamicSharedMemorySize is set once per kernel and device, not per launch.
// One DynLds object per kernel (a function-local static of the launcher's instantiation).
struct DynLds {
  static constexpr int kDevs = 64;
  std::atomic<int> bytes[kDevs];
};
inline hipError_t ensure_dyn_lds(const void *fn, size_t lds, DynLds &st) {
  if (lds <= 48 * 1024) return hipSuccess;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < DynLds::kDevs;
  if (tracked && st.bytes[dev].load(std::memory_order_acquire) >= (int)lds) return hipSuccess;
  e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e == hipSuccess && tracked) st.bytes[dev].store((int)lds, std::memory_order_release);
  return e;
}

// ---- launchers (one per kernel family; each returns hipGetLastError()) ----
// Column sums of squares (p == 2) or of absolute values (p == 1) of K per
// unit, cut into n_split pieces of rows_per_split rows: partial[U][n_split][D].
hipError_t launch_colsum(int dtype, const void *k, double *partial, int64_t U, int64_t S,
                         int n_split, int64_t rows_per_split, int p, hipStream_t st);

// score (and optionally idx) from the partial sums and Q_obs.
//   mode 0: query-driven (Sec. 3.2); mode 1: magnitude l1; mode 2: magnitude l2.
hipError_t launch_finalize(int dtype, int mode, const double *partial, const void *q_obs,
                           float *score, int16_t *idx /*may be null*/, int64_t U, int G,
                           int S_obs, int n_split, int T, hipStream_t st);

hipError_t launch_select(const float *score, int16_t *idx, int64_t U, int T, hipStream_t st);

// K_pruned[u][dst_row0 + r][t] = src[u][src_row0 + r][idx[u][t]], r < n_rows; src has
// src_unit_rows rows of 128 per unit, K_pruned dst_unit_rows rows of ld_keep per unit.
struct CompactArgs {
  const void *src;
  void *dst;
  const int16_t *idx;
  int64_t src_unit_rows, src_row0, dst_unit_rows, dst_row0, n_rows, rows_per_block;
  int32_t T, ld, blocks_per_unit;
};
hipError_t launch_compact(int dtype, const void *src, int64_t src_unit_rows, int64_t src_row0,
                          const int16_t *idx, void *dst, int64_t dst_unit_rows, int64_t dst_row0,
                          int64_t U, int64_t n_rows, int T, int ld_keep, hipStream_t st);
hipError_t launch_copy_rows(int dtype, const void *src, int64_t src_unit_rows, int64_t src_row0, void *dst,
                            int64_t dst_unit_rows, int64_t dst_row0, int64_t U, int64_t n_rows,
                            hipStream_t st);

// One-launch prune (flat K_pruned layout only).  ws: prune_fused_ws_bytes(U, NB) bytes.
size_t prune_fused_ws_bytes(int64_t U, int NB);
// S rows per unit are scored; rows [0, S_keep) are compacted into K_pruned, whose units are
// kp_unit_rows rows apart.  hold = 0: blocks of RB rows re-read their rows for the compaction;
// hold = 1, 2, 4 (fp32: 1, 2): RB = 128 * hold and the rows stay on chip in between.
// given = 1: idx is an INPUT (the list is known; pass G = 1, S_obs = 0, q_obs = k, score = nullptr):
// the call compacts with the same kernels, whose hand-off then only makes a unit's blocks store
// their rows together.
hipError_t launch_prune_fused(int dtype, const void *q_obs, const void *k, float *score, int16_t *idx,
                              void *kp, void *ws, int64_t U, int64_t S, int64_t S_keep,
                              int64_t kp_unit_rows, int G, int S_obs, int T, int ld, int NB, int64_t RB,
                              int hold, int spin_limit, int given, hipStream_t st);

// The same work in ONE launch (rows held on chip only: hold = 1, 2, 4; fp32: 1, 2): the state is
// initialised and the query norms are computed by a prologue block per unit, and blocks whose
// wait ran out are served by the unit's finisher.  ws: prune_solo_ws_bytes(U, NB) bytes.
size_t prune_solo_ws_bytes(int64_t U, int NB);
hipError_t launch_prune_solo(int dtype, const void *q_obs, const void *k, float *score, int16_t *idx,
                             void *kp, void *ws, int64_t U, int64_t S, int64_t S_keep,
                             int64_t kp_unit_rows, int G, int S_obs, int T, int ld, int NB, int64_t RB,
                             int hold, int spin_limit, hipStream_t st);

struct DecodeArgs {
  const void *q, *kp, *v, *kt, *vt;
  const int16_t *idx;
  void *out;
  float *ws;
  int64_t S, rows_per_split;
  int64_t unit_rows;          // rows between units in K_pruned and V (cache capacity per unit)
  int32_t unified_v;          // tail values continue in v after row S (no separate v_tail)
  int32_t T, ldk, N_q, N_kv, s_tail, s_tail_cap, n_split, dtype;
  int64_t units;              // L * B * N_kv
  float scale_log2;           // log2(e) / sqrt(D)
  double scale_log2_d;        // the same, not rounded to float (logits of fp32 inputs)
  // merge inside the launch: one flag word per (unit, head group, split) behind the split
  // records (nullptr: a second kernel merges), and the call's nonce (64 bits, never 0)
  unsigned long long *arrive;
  unsigned long long nonce;
  // channel-pruned values (T_v > 0): v is V_pruned, rows ld_v elements apart, channels idx_v
  const int16_t *idx_v;
  int32_t T_v, ld_v;
};
hipError_t launch_decode(const DecodeArgs &a, hipStream_t st);
constexpr int kDecodeFuseMaxSplit = 16;   // most pieces per unit the launch merges by itself
// the shape runs on the matrix-core kernel (needs dtype, T, ldk, N_q, N_kv, T_v, ld_v of a)
bool decode_mq_serves(const DecodeArgs &a);
int decode_mq_heads(const DecodeArgs &a);   // query heads per block of that kernel: 4 or 8

hipError_t launch_tail_append(int dtype, const void *k_new, const void *v_new, void *k_dst, void *v_dst,
                              int64_t U, int64_t k_unit_rows, int64_t k_row, int64_t v_unit_rows,
                              int64_t v_row, hipStream_t st);

// ---- plain read / copy / write streams for benchmarks (thk_bench_stream.hip) ----
hipError_t launch_bench_stream(int mode, const void *src, void *dst, int64_t n_blocks, int w, hipStream_t st);

// ---- value-channel score (Appendix "Value Cache Pruning") ----
struct ValueAttnArgs {
  const void *q_obs, *k, *v;
  float *part;                 // partial records, value_part_bytes() bytes
  int64_t S, rows_per_split;   // rows_per_split is a multiple of 128
  int64_t U;                   // units of the call
  int32_t G, S_obs, n_split, causal, n_qblk;
  float scale_log2;            // log2(e) / sqrt(D)
};
int value_attn_qt(int G, int S_obs);   // query tiles of 32 rows carried by one block: 1, 2 or 4
size_t value_part_bytes(int64_t U, int G, int S_obs, int n_split);
hipError_t launch_value_score(int dtype, const void *q_obs, const void *k, const void *v, float *part,
                              float *score, int64_t U, int64_t S, int G, int S_obs, int causal,
                              int n_split, int64_t rows_per_split, hipStream_t st);

}  // namespace thk
