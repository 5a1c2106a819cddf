// Channel scoring and Top_T selection kernels (gfx950, wave64).
//
//   k_colsum    streams K once and leaves per-split column sums of squares
//               (Sec. 3.2: the squared 2-norm of every key channel) in fp64.
//   k_finalize  merges the splits, adds the observation-window query norms and
//               writes Score = sum_g ||Q_obs,g[:,c]|| * ||K[:,c]||; optionally
//               runs the selection in the same launch.
//   k_select    Top_T (Sec. 3.1 / 3.2) with one wavefront per unit.
#include "thk_internal.h"

namespace thk {

// ---------------------------------------------------------------------------
// Column reduction of one [rows, 128] slab.  A 16-byte load covers VEC
// channels, so LPR = 128 / VEC lanes cover a row and a 256-thread block covers
// RPB rows per step; each thread keeps the same VEC channels for all its rows.
// Squares of bf16 values are exact in fp32; fp32 chains are UNR terms long and
// are then folded into fp64 accumulators, which carry every later merge.
// ---------------------------------------------------------------------------
template <int DT, int P>
__global__ __launch_bounds__(256) void k_colsum(const void *__restrict__ k,
                                                double *__restrict__ partial, int64_t S,
                                                int n_split, int64_t rows_per_split) {
  using E = Elem<DT>;
  constexpr int VEC = E::VEC, LPR = kD / VEC, RPB = 256 / LPR, UNR = 8;
  const int tid = threadIdx.x;
  const int cl = tid % LPR, rg = tid / LPR;
  const int64_t u = blockIdx.x / n_split;
  const int sp = (int)(blockIdx.x % n_split);
  const int64_t s0 = (int64_t)sp * rows_per_split;
  const int64_t s1 = min(S, s0 + rows_per_split);
  const uint4 *base = (const uint4 *)((const char *)k + (size_t)u * S * kD * E::EB);

  double dacc[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) dacc[v] = 0.0;

  for (int64_t s = s0 + rg; s < s1; s += (int64_t)RPB * UNR) {
    uint4 r[UNR];
#pragma unroll
    for (int j = 0; j < UNR; ++j) {
      const int64_t row = s + (int64_t)j * RPB;
      r[j] = row < s1 ? base[row * LPR + cl] : make_uint4(0, 0, 0, 0);
    }
    float facc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) facc[v] = 0.f;
#pragma unroll
    for (int j = 0; j < UNR; ++j) {
      float f[VEC];
      E::unpack(r[j], f);
#pragma unroll
      for (int v = 0; v < VEC; ++v)
        facc[v] = (P == 2) ? fmaf(f[v], f[v], facc[v]) : facc[v] + fabsf(f[v]);
    }
#pragma unroll
    for (int v = 0; v < VEC; ++v) dacc[v] += (double)facc[v];
  }

  // rows held by the other lane groups of this wave
#pragma unroll
  for (int off = LPR; off < kWave; off <<= 1)
#pragma unroll
    for (int v = 0; v < VEC; ++v) dacc[v] += __shfl_xor(dacc[v], off);

  __shared__ double red[4][kD];
  const int wave = tid / kWave, lane = tid % kWave;
  if (lane < LPR)
#pragma unroll
    for (int v = 0; v < VEC; ++v) red[wave][lane * VEC + v] = dacc[v];
  __syncthreads();
  if (tid < kD)
    partial[(size_t)blockIdx.x * kD + tid] = ((red[0][tid] + red[1][tid]) + red[2][tid]) + red[3][tid];
}

// ---------------------------------------------------------------------------
// Top_T of 128 scores with one wavefront: two keys per lane, bitonic sort of
// 64-bit keys (order-preserving score bits << 32 | 127 - channel, so that equal
// scores rank the lower channel first and all keys are distinct), then every
// lane compares its own keys with the T-th largest and the kept channels are
// emitted in ascending order through ballot + prefix popcount.
// ---------------------------------------------------------------------------
__device__ inline unsigned long long score_key(float s, int c) {
  uint32_t b = __float_as_uint(s);
  b = (b & 0x80000000u) ? ~b : (b | 0x80000000u);   // unsigned order == float order
  return ((unsigned long long)b << 32) | (uint32_t)(kD - 1 - c);
}

__device__ inline void select_wave(float s_lo, float s_hi, int T, int16_t *__restrict__ out, int lane) {
  using u64 = unsigned long long;
  const u64 k0 = score_key(s_lo, lane), k1 = score_key(s_hi, lane + 64);
  u64 a0 = k0, a1 = k1;   // sorted position i = r * 64 + lane holds a_r
#pragma unroll
  for (int k = 2; k <= 128; k <<= 1) {
#pragma unroll
    for (int j = k >> 1; j > 0; j >>= 1) {
      if (j == 64) {   // partner sits in the other register of the same lane
        const u64 hi = a0 > a1 ? a0 : a1, lo = a0 > a1 ? a1 : a0;
        a0 = hi; a1 = lo;
      } else {
        const u64 o0 = __shfl_xor(a0, j), o1 = __shfl_xor(a1, j);
        const bool lower = (lane & j) == 0;
        const bool desc0 = (lane & k) == 0;          // i = lane
        const bool desc1 = ((lane + 64) & k) == 0;   // i = lane + 64
        const u64 mx0 = a0 > o0 ? a0 : o0, mn0 = a0 > o0 ? o0 : a0;
        const u64 mx1 = a1 > o1 ? a1 : o1, mn1 = a1 > o1 ? o1 : a1;
        a0 = (desc0 == lower) ? mx0 : mn0;
        a1 = (desc1 == lower) ? mx1 : mn1;
      }
    }
  }
  const int pos = T - 1;
  const u64 t0 = __shfl(a0, pos & 63), t1 = __shfl(a1, pos & 63);
  const u64 thr = (pos >> 6) ? t1 : t0;
  const bool keep0 = k0 >= thr, keep1 = k1 >= thr;
  const u64 m0 = __ballot(keep0), m1 = __ballot(keep1);
  const u64 below = (1ull << lane) - 1ull;
  if (keep0) out[__popcll(m0 & below)] = (int16_t)lane;
  if (keep1) out[__popcll(m0) + __popcll(m1 & below)] = (int16_t)(lane + 64);
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
  using E = Elem<DT>;
  constexpr int VEC = E::VEC, LPR = kD / VEC, RG = kFinThreads / LPR, NW = kFinThreads / kWave;
  constexpr int GC = 4;   // heads per pass
  __shared__ double red[GC][NW][kD];
  __shared__ float s_sc[kD];
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
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
  if (mode == 0) {
    const int cl = tid % LPR, rg = tid / LPR;
    // unit u = (layer*batch, KV head) reads query heads u * G .. u * G + G - 1
    const uint4 *qbase = (const uint4 *)((const char *)q_obs + (size_t)u * G * S_obs * kD * E::EB);
    for (int g0 = 0; g0 < G; g0 += GC) {
      const int ng = min(GC, G - g0);
      double qa[GC][VEC];
#pragma unroll
      for (int g = 0; g < GC; ++g)
#pragma unroll
        for (int v = 0; v < VEC; ++v) qa[g][v] = 0.0;
      for (int i0 = 0; i0 < S_obs; i0 += RG) {
        uint4 r[GC];
        const int i = i0 + rg;
#pragma unroll
        for (int g = 0; g < GC; ++g)
          r[g] = (g < ng && i < S_obs) ? qbase[((size_t)(g0 + g) * S_obs + i) * LPR + cl]
                                       : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int g = 0; g < GC; ++g) {
          float f[VEC];
          E::unpack(r[g], f);
#pragma unroll
          for (int v = 0; v < VEC; ++v) qa[g][v] += (double)f[v] * (double)f[v];
        }
      }
#pragma unroll
      for (int g = 0; g < GC; ++g) {
#pragma unroll
        for (int off = LPR; off < kWave; off <<= 1)
#pragma unroll
          for (int v = 0; v < VEC; ++v) qa[g][v] += __shfl_xor(qa[g][v], off);
        if (lane < LPR)
#pragma unroll
          for (int v = 0; v < VEC; ++v) red[g][wave][lane * VEC + v] = qa[g][v];
      }
      __syncthreads();
      if (tid < kD)
        for (int g = 0; g < ng; ++g) {
          double qss = 0.0;
#pragma unroll
          for (int w = 0; w < NW; ++w) qss += red[g][w][tid];
          tot += sqrt(qss);
        }
      __syncthreads();
    }
  }

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
  const dim3 grid((unsigned)U), block(kFinThreads);
  if (dtype == THK_BF16)
    hipLaunchKernelGGL((k_finalize<THK_BF16>), grid, block, 0, st, mode, partial, q_obs, score, idx, G, S_obs, n_split, T);
  else
    hipLaunchKernelGGL((k_finalize<THK_F32>), grid, block, 0, st, mode, partial, q_obs, score, idx, G, S_obs, n_split, T);
  return hipGetLastError();
}

hipError_t launch_select(const float *score, int16_t *idx, int64_t U, int T, hipStream_t st) {
  const dim3 grid((unsigned)((U + 3) / 4)), block(256);
  hipLaunchKernelGGL(k_select, grid, block, 0, st, score, idx, U, T);
  return hipGetLastError();
}

}  // namespace thk
