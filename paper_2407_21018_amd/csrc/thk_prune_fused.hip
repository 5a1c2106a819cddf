// One-launch prune: score -> Top_T -> compaction with K read from HBM once
// (Sec. 3.2 selection, Fig. 1 storage) -- gfx950, wave64.
//
// Every 256-thread block owns one (unit, row block) item and does three things:
//   A. column sums of squares of its rows -> partial[item] (fp64), then it
//      announces itself on the unit's arrival counter;
//   B. the block that arrives LAST for a unit merges the unit's partials in
//      row-block order, forms the scores with the pre-computed query norms,
//      runs the Top_T selection, publishes idx and raises the unit's ready
//      flag; the other blocks of the unit wait for that flag (bounded spin);
//   C. every block compacts ITS OWN rows with the published index list.  The
//      rows were streamed moments ago by the same block, so this second read is
//      served by the L2 / memory-side cache instead of HBM.
//
// Waiting is safe: a block only waits for blocks of its own unit, which have
// lower or neighbouring block numbers and are dispatched with it; the wait is
// bounded all the same, and a block that gives up leaves its rows to
// k_prune_repair, which runs afterwards and compacts whatever is not marked
// done.  All sums run in a fixed order: the result does not depend on which
// block arrives last.
//
// Cross-block traffic.  The L2 caches of the eight XCDs are not coherent with
// each other, and a device-scope release/acquire fence would write back /
// invalidate a whole L2 per block.  Instead, everything one block hands to
// another (partial sums, the index list, the counter and the flag) moves through
// relaxed device-scope atomic loads and stores, which go to the coherence point
// themselves; a producer waits until its own stores have been acknowledged
// (s_waitcnt vmcnt(0) in every wave, then the block barrier) before it bumps the
// counter or raises the flag, and a consumer only reads after it has seen the
// counter or flag value.  The wait is written out: a workgroup-scope release
// fence compiles to nothing here (a block's waves share one L1), and without it
// the flag can overtake the data on its way to memory.
#include "thk_prune_device.h"

namespace thk {

struct PruneFusedArgs {
  const void *k, *q_obs;
  void *kp;
  float *score;
  int16_t *idx;
  double *partial;        // [U][NB][128]
  double *qn;             // [U][128]   sum_g ||Q_obs,g[:, c]||
  int *arrived, *ready;   // [U] each
  uint32_t *idx_pub;      // [U][64]  the index list, two entries per word, for the waiting blocks
  unsigned char *done;    // [U * NB]
  int64_t S, RB;          // rows per unit, rows per block
  int64_t S_keep;         // rows [0, S_keep) of every unit are compacted
  int64_t kp_unit_rows;   // rows between units of K_pruned
  int32_t T, G, S_obs, NB, spin_limit;
};

__device__ inline void pub_store_f64(double *p, double v) {
  __hip_atomic_store((unsigned long long *)p, (unsigned long long)__double_as_longlong(v), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline double pub_load_f64(const double *p) {
  return __longlong_as_double((long long)__hip_atomic_load((const unsigned long long *)p, __ATOMIC_RELAXED,
                                                           __HIP_MEMORY_SCOPE_AGENT));
}
// Every store the block has issued so far has been acknowledged by the memory system (no cache
// maintenance): what a producer needs before it signals through a device-scope atomic.
__device__ inline void block_stores_done() {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
}

// Per unit: query norms, and the counters / flags back to zero.
template <int DT>
__global__ __launch_bounds__(512) void k_prune_prep(PruneFusedArgs a) {
  __shared__ double red[kQnHeads][512 / kWave][kD];
  const int64_t u = blockIdx.x;
  const double tot = unit_query_norm<DT, 512>(a.q_obs, u, a.G, a.S_obs, red);
  if (threadIdx.x < kD) a.qn[(size_t)u * kD + threadIdx.x] = tot;
  if (threadIdx.x == 0) { a.arrived[u] = 0; a.ready[u] = 0; }
  for (int i = threadIdx.x; i < a.NB; i += 512) a.done[(size_t)u * a.NB + i] = 0;
}

template <int DT>
__global__ __launch_bounds__(256) void k_prune_fused(PruneFusedArgs a) {
  using E = Elem<DT>;
  extern __shared__ u32x4 smem[];
  uint16_t *tab = (uint16_t *)smem;          // 2 KiB
  u32x4 *tiles = smem + 128;                 // 4 x [32][128] elements
  __shared__ double red[4][kD];
  __shared__ float s_sc[kD];
  __shared__ int s_flag;
  const int tid = threadIdx.x;
  const int64_t item = blockIdx.x;
  const int64_t u = item / a.NB;
  const int blk = (int)(item % a.NB);
  const int64_t s0 = (int64_t)blk * a.RB;
  const int64_t s1 = min(a.S, s0 + a.RB);
  const u32x4 *src = (const u32x4 *)((const char *)a.k + (size_t)u * a.S * kD * E::EB);

  // ---- A. partial column sums, then arrive -----------------------------------
  __shared__ double s_part[kD];
  __shared__ int16_t s_idx[kD];
  colsum_block<DT, 2>(src, s0, s1, s_part, red);
  __syncthreads();
  if (tid < kD) pub_store_f64(a.partial + (size_t)item * kD + tid, s_part[tid]);
  block_stores_done();
  if (tid == 0) s_flag = (atomicAdd(&a.arrived[u], 1) == a.NB - 1);
  __syncthreads();

  if (s_flag) {
    // ---- B. last block of the unit: merge, score, select, publish ------------
    if (tid < kD) {
      const double *p = a.partial + (size_t)u * a.NB * kD + tid;
      double kss = 0.0;
      int b = 0;
      for (; b + 8 <= a.NB; b += 8) {
        double x[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = pub_load_f64(p + (size_t)(b + j) * kD);
#pragma unroll
        for (int j = 0; j < 8; ++j) kss += x[j];
      }
      for (; b < a.NB; ++b) kss += pub_load_f64(p + (size_t)b * kD);
      const float scf = (float)(a.qn[(size_t)u * kD + tid] * sqrt(kss));
      a.score[(size_t)u * kD + tid] = scf;
      s_sc[tid] = scf;
    }
    __syncthreads();
    if (tid < kWave) select_wave(s_sc[tid], s_sc[tid + 64], a.T, s_idx, tid);
    __syncthreads();
    if (tid < a.T) a.idx[(size_t)u * a.T + tid] = s_idx[tid];
    if (tid < kWave) {
      const uint32_t lo = 2 * tid < a.T ? (uint16_t)s_idx[2 * tid] : 0u;
      const uint32_t hi = 2 * tid + 1 < a.T ? (uint16_t)s_idx[2 * tid + 1] : 0u;
      __hip_atomic_store(a.idx_pub + (size_t)u * kWave + tid, lo | (hi << 16), __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
    }
    block_stores_done();
    if (tid == 0) __hip_atomic_store(&a.ready[u], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  } else {
    // ---- wait (bounded) for the unit's index list ----------------------------
    if (tid == 0) {
      int ok = __hip_atomic_load(&a.ready[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      for (int n = 0; ok == 0 && n < a.spin_limit; ++n) {
        __builtin_amdgcn_s_sleep(16);
        ok = __hip_atomic_load(&a.ready[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      s_flag = ok;
    }
    __syncthreads();
    if (s_flag == 0) return;   // whole block leaves; k_prune_repair compacts these rows
    if (tid < kWave) {
      const uint32_t w = __hip_atomic_load(a.idx_pub + (size_t)u * kWave + tid, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
      s_idx[2 * tid] = (int16_t)(w & 0xffffu);
      s_idx[2 * tid + 1] = (int16_t)(w >> 16);
    }
    __syncthreads();
  }

  // ---- C. compact this block's rows -------------------------------------------
  compact_build_tab(tab, s_idx, a.T);
  __syncthreads();
  const int64_t s1c = min(s1, a.S_keep);   // rows past S_keep stay at full width with the caller
  if (s0 < s1c)
    compact_rows<DT>(src, (u32x4 *)((char *)a.kp + (size_t)u * a.kp_unit_rows * a.T * E::EB), s0, s1c, a.T, tab, tiles);
  if (tid == 0) a.done[item] = 1;
}

// One block per unit: compact the row blocks that k_prune_fused left undone.
template <int DT>
__global__ __launch_bounds__(256) void k_prune_repair(PruneFusedArgs a) {
  using E = Elem<DT>;
  extern __shared__ u32x4 smem[];
  uint16_t *tab = (uint16_t *)smem;
  u32x4 *tiles = smem + 128;
  __shared__ int s_any;
  const int64_t u = blockIdx.x;
  const unsigned char *done = a.done + (size_t)u * a.NB;
  if (threadIdx.x == 0) s_any = 0;
  __syncthreads();
  int undone = 0;
  for (int i = threadIdx.x; i < a.NB; i += 256) undone |= (done[i] == 0);
  if (undone) s_any = 1;
  __syncthreads();
  if (s_any == 0) return;
  compact_build_tab(tab, a.idx + (size_t)u * a.T, a.T);
  __syncthreads();
  const u32x4 *src = (const u32x4 *)((const char *)a.k + (size_t)u * a.S * kD * E::EB);
  u32x4 *dst = (u32x4 *)((char *)a.kp + (size_t)u * a.kp_unit_rows * a.T * E::EB);
  for (int blk = 0; blk < a.NB; ++blk) {
    if (done[blk]) continue;   // block-uniform: every thread reads the same byte
    const int64_t s0 = (int64_t)blk * a.RB;
    const int64_t s1c = min(a.S_keep, s0 + a.RB);
    if (s0 < s1c) compact_rows<DT>(src, dst, s0, s1c, a.T, tab, tiles);
  }
}

size_t prune_fused_ws_bytes(int64_t U, int NB) {
  size_t b = (size_t)U * NB * kD * sizeof(double);   // partial
  b += (size_t)U * kD * sizeof(double);              // qn
  b += (size_t)U * 2 * sizeof(int);                  // arrived, ready
  b = (b + 15) & ~(size_t)15;
  b += (size_t)U * kWave * sizeof(uint32_t);         // idx_pub
  b += ((size_t)U * NB + 15) & ~(size_t)15;          // done
  return b;
}

hipError_t launch_prune_fused(int dtype, const void *q_obs, const void *k, float *score, int16_t *idx,
                              void *kp, void *ws, int64_t U, int64_t S, int64_t S_keep,
                              int64_t kp_unit_rows, int G, int S_obs, int T, int NB, int64_t RB,
                              int spin_limit, hipStream_t st) {
  clear_stale_hip_error();
  PruneFusedArgs a;
  a.k = k; a.q_obs = q_obs; a.kp = kp; a.score = score; a.idx = idx;
  char *w = (char *)ws;
  a.partial = (double *)w; w += (size_t)U * NB * kD * sizeof(double);
  a.qn = (double *)w;      w += (size_t)U * kD * sizeof(double);
  a.arrived = (int *)w;    w += (size_t)U * sizeof(int);
  a.ready = (int *)w;      w += (size_t)U * sizeof(int);
  w = (char *)(((uintptr_t)w + 15) & ~(uintptr_t)15);
  a.idx_pub = (uint32_t *)w; w += (size_t)U * kWave * sizeof(uint32_t);
  a.done = (unsigned char *)w;
  a.S = S; a.S_keep = S_keep; a.kp_unit_rows = kp_unit_rows; a.RB = RB; a.T = T; a.G = G; a.S_obs = S_obs; a.NB = NB; a.spin_limit = spin_limit;
  const int eb = dtype == THK_BF16 ? 2 : 4;
  const size_t lds = 2048 + 4 * (size_t)kCompactTileRows * kD * eb;
  const dim3 gu((unsigned)U), gi((unsigned)(U * NB));
  if (dtype == THK_BF16) {
    hipLaunchKernelGGL((k_prune_prep<THK_BF16>), gu, dim3(512), 0, st, a);
    profile_mark(true, st);
    hipLaunchKernelGGL((k_prune_fused<THK_BF16>), gi, dim3(256), lds, st, a);
    profile_mark(false, st);
    hipLaunchKernelGGL((k_prune_repair<THK_BF16>), gu, dim3(256), lds, st, a);
  } else {
    hipError_t e = hipFuncSetAttribute((const void *)k_prune_fused<THK_F32>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void *)k_prune_repair<THK_F32>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((k_prune_prep<THK_F32>), gu, dim3(512), 0, st, a);
    profile_mark(true, st);
    hipLaunchKernelGGL((k_prune_fused<THK_F32>), gi, dim3(256), lds, st, a);
    profile_mark(false, st);
    hipLaunchKernelGGL((k_prune_repair<THK_F32>), gu, dim3(256), lds, st, a);
  }
  return hipGetLastError();
}

}  // namespace thk
