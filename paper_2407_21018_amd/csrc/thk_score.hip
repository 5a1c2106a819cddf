// Channel scoring and Top_T selection kernels (gfx950, wave64).
//
//   k_colsum    streams K once and leaves per-split column sums of squares
//               (Sec. 3.2: the squared 2-norm of every key channel) in fp64.
//   k_finalize  merges the splits, adds the observation-window query norms and
//               writes Score = sum_g ||Q_obs,g[:,c]|| * ||K[:,c]||; optionally
//               runs the selection in the same launch.
//   k_select    Top_T (Sec. 3.1 / 3.2) with one wavefront per unit.
#include "thk_prune_device.h"

namespace thk {

template <int DT, int P>
__global__ __launch_bounds__(256) void k_colsum(const void *__restrict__ k,
                                                double *__restrict__ partial, int64_t S,
                                                int n_split, int64_t rows_per_split) {
  __shared__ double red[4][kD];
  const int64_t u = blockIdx.x / n_split;
  const int sp = (int)(blockIdx.x % n_split);
  const int64_t s0 = (int64_t)sp * rows_per_split;
  const int64_t s1 = min(S, s0 + rows_per_split);
  const u32x4 *base = (const u32x4 *)((const char *)k + (size_t)u * S * kD * Elem<DT>::EB);
  colsum_block<DT, P>(base, s0, s1, partial + (size_t)blockIdx.x * kD, red);
}

__global__ __launch_bounds__(256) void k_select(const float *__restrict__ score,
                                                int16_t *__restrict__ idx, int64_t U, int T) {
  const int lane = threadIdx.x % kWave;
  const int64_t u = (int64_t)blockIdx.x * 4 + threadIdx.x / kWave;
  if (u >= U) return;   // whole wave leaves together
  const float *sc = score + (size_t)u * kD;
  select_wave(sc[lane], sc[lane + 64], T, idx + (size_t)u * T, lane);
}

// ---------------------------------------------------------------------------
// One 512-thread block per unit.
//   1. split merge: thread (sg, c) adds the partial sums of splits sg, sg+4, ..
//      for channel c; the four strands are added in fixed order.
//   2. query norms: the unit's G heads hold G * S_obs contiguous rows of Q_obs;
//      heads are taken four at a time, each thread squares (in fp64) the VEC
//      channels it owns over the rows of its row group, row groups are folded
//      by shuffles inside a wave and through LDS across the 8 waves.
//   3. threads 0..127 form the score of their channel; wave 0 may select.
// All sums run in a fixed order, so repeated calls give identical bits.
// ---------------------------------------------------------------------------
constexpr int kFinThreads = 512;

template <int DT>
__global__ __launch_bounds__(kFinThreads) void k_finalize(int mode, const double *__restrict__ partial,
                                                          const void *__restrict__ q_obs,
                                                          float *__restrict__ score,
                                                          int16_t *__restrict__ idx, int G,
                                                          int S_obs, int n_split, int T) {
  constexpr int NW = kFinThreads / kWave;
  __shared__ double red[kQnHeads][NW][kD];
  __shared__ float s_sc[kD];
  const int tid = threadIdx.x;
  const int64_t u = blockIdx.x;

  // ---- 1. split merge ----------------------------------------------------
  {
    const int c = tid % kD, sg = tid / kD;
    const double *p = partial + (size_t)u * n_split * kD + c;
    double a = 0.0;
    int sp = sg;
    for (; sp + 12 < n_split; sp += 16) {
      const double x0 = p[(size_t)sp * kD], x1 = p[(size_t)(sp + 4) * kD];
      const double x2 = p[(size_t)(sp + 8) * kD], x3 = p[(size_t)(sp + 12) * kD];
      a += x0; a += x1; a += x2; a += x3;
    }
    for (; sp < n_split; sp += 4) a += p[(size_t)sp * kD];
    red[0][sg][c] = a;
  }
  __syncthreads();
  double kacc = 0.0;
  if (tid < kD) kacc = ((red[0][0][tid] + red[0][1][tid]) + red[0][2][tid]) + red[0][3][tid];
  __syncthreads();

  // ---- 2. query norms ------------------------------------------------------
  double tot = 0.0;
  if (mode == 0) tot = unit_query_norm<DT, kFinThreads>(q_obs, u, G, S_obs, red);

  // ---- 3. score, optional selection ----------------------------------------
  if (tid < kD) {
    const double sc = mode == 0 ? tot * sqrt(kacc) : (mode == 1 ? kacc : sqrt(kacc));
    const float scf = (float)sc;
    score[(size_t)u * kD + tid] = scf;
    s_sc[tid] = scf;
  }
  if (idx != nullptr) {
    __syncthreads();
    if (tid < kWave) select_wave(s_sc[tid], s_sc[tid + 64], T, idx + (size_t)u * T, tid);
  }
}

// ---------------------------------------------------------------------------
hipError_t launch_colsum(int dtype, const void *k, double *partial, int64_t U, int64_t S,
                         int n_split, int64_t rows_per_split, int p, hipStream_t st) {
  clear_stale_hip_error();
  const dim3 grid((unsigned)(U * n_split)), block(256);
  if (dtype == THK_BF16) {
    if (p == 2) hipLaunchKernelGGL((k_colsum<THK_BF16, 2>), grid, block, 0, st, k, partial, S, n_split, rows_per_split);
    else        hipLaunchKernelGGL((k_colsum<THK_BF16, 1>), grid, block, 0, st, k, partial, S, n_split, rows_per_split);
  } else {
    if (p == 2) hipLaunchKernelGGL((k_colsum<THK_F32, 2>), grid, block, 0, st, k, partial, S, n_split, rows_per_split);
    else        hipLaunchKernelGGL((k_colsum<THK_F32, 1>), grid, block, 0, st, k, partial, S, n_split, rows_per_split);
  }
  return hipGetLastError();
}

hipError_t launch_finalize(int dtype, int mode, const double *partial, const void *q_obs,
                           float *score, int16_t *idx, int64_t U, int G, int S_obs,
                           int n_split, int T, hipStream_t st) {
  clear_stale_hip_error();
  const dim3 grid((unsigned)U), block(kFinThreads);
  if (dtype == THK_BF16)
    hipLaunchKernelGGL((k_finalize<THK_BF16>), grid, block, 0, st, mode, partial, q_obs, score, idx, G, S_obs, n_split, T);
  else
    hipLaunchKernelGGL((k_finalize<THK_F32>), grid, block, 0, st, mode, partial, q_obs, score, idx, G, S_obs, n_split, T);
  return hipGetLastError();
}

hipError_t launch_select(const float *score, int16_t *idx, int64_t U, int T, hipStream_t st) {
  clear_stale_hip_error();
  const dim3 grid((unsigned)((U + 3) / 4)), block(256);
  hipLaunchKernelGGL(k_select, grid, block, 0, st, score, idx, U, T);
  return hipGetLastError();
}

}  // namespace thk
