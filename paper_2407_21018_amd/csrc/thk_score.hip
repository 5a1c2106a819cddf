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
// One 128-thread block per unit, thread c owns channel c.
// ---------------------------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(128) void k_finalize(int mode, const double *__restrict__ partial,
                                                  const void *__restrict__ q_obs,
                                                  float *__restrict__ score,
                                                  int16_t *__restrict__ idx, int G,
                                                  int S_obs, int n_split, int T) {
  using E = Elem<DT>;
  const int c = threadIdx.x;
  const int64_t u = blockIdx.x;
  double kacc = 0.0;
  for (int sp = 0; sp < n_split; ++sp) kacc += partial[((size_t)u * n_split + sp) * kD + c];
  double sc;
  if (mode == 0) {
    // unit u = (layer*batch, KV head h) reads query heads u * G .. u * G + G - 1
    double tot = 0.0;
    for (int g = 0; g < G; ++g) {
      const size_t qb = ((size_t)(u * G + g) * S_obs) * kD;
      double qss = 0.0;
      for (int i = 0; i < S_obs; ++i) {
        const double x = (double)E::load1(q_obs, qb + (size_t)i * kD + c);
        qss += x * x;
      }
      tot += sqrt(qss);
    }
    sc = tot * sqrt(kacc);
  } else {
    sc = (mode == 1) ? kacc : sqrt(kacc);
  }
  const float scf = (float)sc;
  score[(size_t)u * kD + c] = scf;
  if (idx != nullptr) {
    __shared__ float s_sc[kD];
    s_sc[c] = scf;
    __syncthreads();
    if (c < kWave) select_wave(s_sc[c], s_sc[c + 64], T, idx + (size_t)u * T, c);
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
  const dim3 grid((unsigned)U), block(128);
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
