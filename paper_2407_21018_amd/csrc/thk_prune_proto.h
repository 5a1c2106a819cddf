// Shared pieces of the one-launch prune kernels: the argument block, the cross-block publishing
// primitives and the steps that turn a unit's column sums into its index list (gfx950, wave64).
//
// Cross-block traffic.  The L2 caches of the eight XCDs are not coherent with each other, and a
// device-scope release/acquire fence would write back / invalidate a whole L2 per block.
// Instead, everything one block hands to another moves through relaxed device-scope atomic
// loads and stores, which go to the coherence point themselves.  Before it signals through a
// counter a producer waits until what it published has been acknowledged (s_waitcnt vmcnt(0)
// in every wave, then the block barrier): a workgroup-scope release fence compiles to nothing
// here (a block's waves share one L1), and without the wait the counter can overtake the data
// on its way to memory.
#pragma once
#include "thk_prune_device.h"

namespace thk {

constexpr int kMaxGroups = 16;   // groups per unit in the two-level arrival

struct PruneFusedArgs {
  const void *k, *q_obs;
  void *kp;
  float *score;
  int16_t *idx;
  double *partial;        // [U][NB][128]
  double *qn;             // [U][128]   sum_g ||Q_obs,g[:, c]||
  int *arrived;           // [U] blocks (or groups) of the unit that have published their sums
  int *arrived_g;         // [U][kMaxGroups] blocks of a group that have published (two-level form)
  double *gpartial;       // [U][kMaxGroups][128] group sums (two-level form)
  int32_t GS;             // blocks per group; 0 = one level
  // graded start of a launch's first round: block `item` < stagger_blocks of unit u first
  // sleeps (u % stagger_units) * stagger_ticks times 64 cycles
  int32_t stagger_blocks, stagger_units, stagger_ticks;
  uint32_t *idx_pub;      // [U][64]  the index list, two entries per word, for the waiting blocks
  unsigned char *done;    // [U * NB]  three-launch form: row blocks that have been compacted
  // single-launch form only
  unsigned long long *tctr;    // [U] arrival counter of the unit (one level), tagged with the call's nonce
  unsigned long long *tctr_g;  // [U][kMaxGroups] arrival counters of the groups (two levels), tagged
  unsigned long long nonce;    // 48 bits, never 0, different for every call
  unsigned char *undone;       // [U * NB] raised by a block that gave up waiting: its rows are the finisher's
  int *gaveup;                 // [U] tickets: +1 per block that gave up, + kFinisherDone by the finisher
  int32_t prologue_delay;      // test hook: 64-cycle ticks the prologue block sleeps before it starts
  int64_t U;                   // units of the call: blocks 0 .. U-1 are the prologue blocks, the row blocks follow
  int64_t S, RB;          // rows per unit, rows per block
  int64_t S_keep;         // rows [0, S_keep) of every unit are compacted
  int64_t kp_unit_rows;   // rows between units of K_pruned
  int32_t T, ld, G, S_obs, NB, spin_limit;   // ld: elements from row to row of K_pruned
  // 1: the index list in `idx` is the caller's INPUT (compaction of a cache whose list is known,
  // e.g. the value cache).  The blocks of a unit still exchange their column sums, but only as
  // the barrier that makes a unit's rows leave the chip in one burst; no score is written.
  int32_t given;
};

__device__ inline void pub_store_f64(double *p, double v) {
  __hip_atomic_store((unsigned long long *)p, (unsigned long long)__double_as_longlong(v), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline double pub_load_f64(const double *p) {
  return __longlong_as_double((long long)__hip_atomic_load((const unsigned long long *)p, __ATOMIC_RELAXED,
                                                           __HIP_MEMORY_SCOPE_AGENT));
}
// Mark of a published index-list word (channel numbers are below 128, so bit 15 of each half
// is free); k_prune_prep clears the words.
constexpr uint32_t kPubValid = 0x80008000u;

// Every store the block has issued so far has been acknowledged by the memory system (no cache
// maintenance): what a producer needs before it signals through a device-scope atomic.
__device__ inline void block_stores_done() {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
}

// Sum of n partial vectors (128 doubles each, consecutive) for channel tid % 128: the two halves
// of the list are summed by two thread groups (eight loads in flight each) and added, first
// half first.  The result is valid in the threads of the first group.  xch: 128 doubles of LDS.
__device__ __forceinline__ double merge_partials(const double *base, int n, double *xch) {
  const int tid = threadIdx.x;
  const int c = tid & (kD - 1), half = tid >> 7;
  const int b_mid = (n + 1) / 2;
  const int b0 = half ? b_mid : 0, b1 = half ? n : b_mid;
  const double *p = base + c;
  double sum = 0.0;
  for (int b = b0; b < b1; b += 8) {   // a short last batch re-reads its last entry, unused
    double x[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) x[j] = pub_load_f64(p + (size_t)min(b + j, b1 - 1) * kD);
#pragma unroll
    for (int j = 0; j < 8; ++j) sum += (b + j < b1) ? x[j] : 0.0;
  }
  if (half) xch[c] = sum;
  __syncthreads();
  if (!half) sum += xch[c];
  return sum;
}

// One arrival: thread 0 bumps the counter; true in every thread of the block that makes it `full`.
__device__ __forceinline__ bool arrive(int *counter, int full, int *s_flag) {
  if (threadIdx.x == 0) *s_flag = (atomicAdd(counter, 1) == full - 1);
  __syncthreads();
  const bool last = *s_flag != 0;
  __syncthreads();   // everyone has read the flag before it is reused
  return last;
}

// A group's sums as the group's last block publishes them: 64-bit words that carry their own
// validity mark in the lowest mantissa bit (a change of at most 2^-52 relative; k_prune_prep
// clears the words before every call), so that readers need no flag and no ordering.
__device__ inline void pub_store_marked(double *p, double v) {
  __hip_atomic_store((unsigned long long *)p, (unsigned long long)__double_as_longlong(v) | 1ull, __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline unsigned long long pub_load_bits(const double *p) {
  return __hip_atomic_load((const unsigned long long *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Scores of the unit from its column sums (kss, valid in threads < 128) and the index list;
// `writer` also stores both for the caller.
__device__ __forceinline__ void score_and_select(const PruneFusedArgs &a, int64_t u, double qn_c, double kss,
                                                 float *s_sc, int16_t *s_idx, bool writer) {
  const int tid = threadIdx.x;
  if (a.given) {
    if (tid < a.T) s_idx[tid] = a.idx[(size_t)u * a.T + tid];
    __syncthreads();
    return;
  }
  if (tid < kD) {
    const float scf = (float)(qn_c * sqrt(kss));
    if (writer) a.score[(size_t)u * kD + tid] = scf;
    s_sc[tid] = scf;
  }
  __syncthreads();
  select_block(s_sc, a.T, s_idx);
  if (writer && tid < a.T) a.idx[(size_t)u * a.T + tid] = s_idx[tid];
}

}  // namespace thk
