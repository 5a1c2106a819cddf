// Key compaction K_pruned[s][t] = K[s][idx[t]] (Fig. 1; Sec. 3.3) and the
// tail append (gfx950, wave64).  Pure byte movement: no arithmetic on values.
#include <type_traits>

#include "thk_prune_device.h"

namespace thk {

// Flat path: K_pruned rows dense (ld_keep == T) and every unit of K_pruned
// starting on a 16-byte boundary, so that a slab of whole rows is a run of whole
// 16-byte chunks (see compact_rows).
template <int DT>
__global__ __launch_bounds__(256) void k_compact_flat(const void *__restrict__ k,
                                                      const int16_t *__restrict__ idx,
                                                      void *__restrict__ kp, int64_t S, int T,
                                                      int blocks_per_unit, int64_t rows_per_block) {
  using E = Elem<DT>;
  extern __shared__ u32x4 smem[];
  uint16_t *tab = (uint16_t *)smem;                       // [8 * T], padded to 2 KiB
  const int64_t u = blockIdx.x / blocks_per_unit;
  const int blk = (int)(blockIdx.x % blocks_per_unit);
  const int64_t s0 = (int64_t)blk * rows_per_block;
  const int64_t s1 = min(S, s0 + rows_per_block);
  compact_build_tab(tab, idx + (size_t)u * T, T);
  __syncthreads();
  compact_rows<DT>((const u32x4 *)((const char *)k + (size_t)u * S * kD * E::EB),
                   (u32x4 *)((char *)kp + (size_t)u * S * T * E::EB), s0, s1, T, tab, smem + 128);
}

// Element-wise path for padded or unaligned K_pruned layouts.
template <int DT>
__global__ __launch_bounds__(256) void k_compact_generic(const void *__restrict__ k,
                                                         const int16_t *__restrict__ idx,
                                                         void *__restrict__ kp, int64_t S, int T,
                                                         int ld, int blocks_per_unit,
                                                         int64_t rows_per_block) {
  using ET = typename std::conditional<DT == THK_BF16, uint16_t, uint32_t>::type;
  const int64_t u = blockIdx.x / blocks_per_unit;
  const int blk = (int)(blockIdx.x % blocks_per_unit);
  const int64_t s0 = (int64_t)blk * rows_per_block;
  const int64_t s1 = min(S, s0 + rows_per_block);
  const ET *src = (const ET *)k + (size_t)u * S * kD;
  ET *dst = (ET *)kp + (size_t)u * S * ld;
  const int16_t *uidx = idx + (size_t)u * T;
  const int64_t n = (s1 - s0) * T;
  for (int64_t e = threadIdx.x; e < n; e += 256) {
    const int64_t s = s0 + e / T;
    const int t = (int)(e % T);
    dst[(size_t)s * ld + t] = src[(size_t)s * kD + uidx[t]];
  }
}

template <int DT>
__global__ __launch_bounds__(256) void k_tail_append(const void *__restrict__ k_new,
                                                     const void *__restrict__ v_new,
                                                     void *__restrict__ k_tail,
                                                     void *__restrict__ v_tail, int64_t U,
                                                     int s_tail, int cap) {
  using E = Elem<DT>;
  constexpr int CPR = kD / E::VEC;   // 16-byte chunks per row
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= U * CPR) return;
  const int64_t u = i / CPR;
  const int c = (int)(i % CPR);
  const size_t d = ((size_t)u * cap + s_tail) * CPR + c;
  ((uint4 *)k_tail)[d] = ((const uint4 *)k_new)[i];
  ((uint4 *)v_tail)[d] = ((const uint4 *)v_new)[i];
}

hipError_t launch_compact(int dtype, const void *k, const int16_t *idx, void *kp, int64_t U,
                          int64_t S, int T, int ld_keep, hipStream_t st) {
  const int eb = dtype == THK_BF16 ? 2 : 4;
  const bool flat = ld_keep == T && ((size_t)S * T * eb) % 16 == 0;
  // 512 rows per block (4 waves x 4 tiles), fewer blocks per unit when S is short
  const int64_t rows_per_block = 512;
  const int bpu = (int)((S + rows_per_block - 1) / rows_per_block);
  const dim3 grid((unsigned)(U * bpu)), block(256);
  if (flat) {
    const size_t lds = 2048 + 4 * (size_t)32 * kD * eb;
    if (dtype == THK_BF16)
      hipLaunchKernelGGL((k_compact_flat<THK_BF16>), grid, block, lds, st, k, idx, kp, S, T, bpu, rows_per_block);
    else
      hipLaunchKernelGGL((k_compact_flat<THK_F32>), grid, block, lds, st, k, idx, kp, S, T, bpu, rows_per_block);
  } else {
    if (dtype == THK_BF16)
      hipLaunchKernelGGL((k_compact_generic<THK_BF16>), grid, block, 0, st, k, idx, kp, S, T, ld_keep, bpu, rows_per_block);
    else
      hipLaunchKernelGGL((k_compact_generic<THK_F32>), grid, block, 0, st, k, idx, kp, S, T, ld_keep, bpu, rows_per_block);
  }
  return hipGetLastError();
}

hipError_t launch_tail_append(int dtype, const void *k_new, const void *v_new, void *k_tail,
                              void *v_tail, int64_t U, int s_tail, int cap, hipStream_t st) {
  const int cpr = dtype == THK_BF16 ? 16 : 32;
  const dim3 grid((unsigned)((U * cpr + 255) / 256)), block(256);
  if (dtype == THK_BF16)
    hipLaunchKernelGGL((k_tail_append<THK_BF16>), grid, block, 0, st, k_new, v_new, k_tail, v_tail, U, s_tail, cap);
  else
    hipLaunchKernelGGL((k_tail_append<THK_F32>), grid, block, 0, st, k_new, v_new, k_tail, v_tail, U, s_tail, cap);
  return hipGetLastError();
}

}  // namespace thk
