// Key compaction K_pruned[s][t] = K[s][idx[t]] (Fig. 1; Sec. 3.3) and the
// tail append (gfx950, wave64).  Pure byte movement: no arithmetic on values.
#include "thk_internal.h"

namespace thk {

// ---------------------------------------------------------------------------
// Flat path.  Used when K_pruned rows are dense (ld_keep == T) and every unit
// of K_pruned starts on a 16-byte boundary, so that a slab of whole rows is a
// run of whole 16-byte chunks.  Each wavefront works alone on tiles of TR rows:
//   1. 16-byte coalesced loads of the full-width rows into its LDS tile;
//   2. for every 16-byte chunk of the OUTPUT slab, a table lookup gives the LDS
//      element offsets of its VEC source elements (the pattern of
//      row * 128 + idx[t] repeats every 8 output rows because 8 * T elements is
//      a whole number of chunks), the elements are gathered from LDS, packed
//      and stored with one 16-byte store.
// ---------------------------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(256) void k_compact_flat(const void *__restrict__ k,
                                                      const int16_t *__restrict__ idx,
                                                      void *__restrict__ kp, int64_t S, int T,
                                                      int blocks_per_unit, int64_t rows_per_block) {
  using E = Elem<DT>;
  constexpr int VEC = E::VEC, CPR = kD / VEC, TR = 32;
  constexpr int NLD = TR * CPR / kWave;   // 16-byte loads per lane per tile
  extern __shared__ uint4 smem[];
  uint16_t *tab = (uint16_t *)smem;                       // [8 * T], padded to 2 KiB
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  uint4 *tile = smem + 128 + wave * (TR * CPR);           // this wave's [TR][128] slab

  const int64_t u = blockIdx.x / blocks_per_unit;
  const int blk = (int)(blockIdx.x % blocks_per_unit);
  const int64_t s0 = (int64_t)blk * rows_per_block;
  const int64_t s1 = min(S, s0 + rows_per_block);

  const int period = 8 * T;
  const int16_t *uidx = idx + (size_t)u * T;
  for (int e = threadIdx.x; e < period; e += 256) {
    const int row = e / T, t = e - row * T;
    tab[e] = (uint16_t)(row * kD + (int)uidx[t]);
  }
  __syncthreads();

  const uint4 *src = (const uint4 *)((const char *)k + (size_t)u * S * kD * E::EB);
  uint4 *dst = (uint4 *)((char *)kp + (size_t)u * S * T * E::EB);

  for (int64_t r0 = s0 + (int64_t)wave * TR; r0 < s1; r0 += 4 * TR) {
    const int nr = (int)min((int64_t)TR, s1 - r0);
    // rows past the end of a ragged last tile re-read its last row (kept in bounds, never gathered)
    uint4 r[NLD];
    const uint4 *tsrc = src + (size_t)r0 * CPR;
    const int cmax = nr * CPR - 1;
#pragma unroll
    for (int j = 0; j < NLD; ++j) r[j] = tsrc[min(j * kWave + lane, cmax)];
#pragma unroll
    for (int j = 0; j < NLD; ++j) tile[j * kWave + lane] = r[j];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    const int nchunks = nr * T / VEC;   // exact: (r0 * T) and (S * T) are multiples of VEC
    uint4 *o = dst + (size_t)r0 * T / VEC;
    for (int c = lane; c < nchunks; c += kWave) {
      const int e0 = c * VEC;
      const int pb = e0 / period;
      const int pe = e0 - pb * period;
      const int rowbase = pb * 8 * kD;
      uint4 w;
      if constexpr (DT == THK_BF16) {
        const uint16_t *tl = (const uint16_t *)tile + rowbase;
        const uint4 offs = *(const uint4 *)(tab + pe);   // 8 offsets
        const uint32_t o0 = offs.x & 0xffffu, o1 = offs.x >> 16, o2 = offs.y & 0xffffu, o3 = offs.y >> 16;
        const uint32_t o4 = offs.z & 0xffffu, o5 = offs.z >> 16, o6 = offs.w & 0xffffu, o7 = offs.w >> 16;
        w.x = (uint32_t)tl[o0] | ((uint32_t)tl[o1] << 16);
        w.y = (uint32_t)tl[o2] | ((uint32_t)tl[o3] << 16);
        w.z = (uint32_t)tl[o4] | ((uint32_t)tl[o5] << 16);
        w.w = (uint32_t)tl[o6] | ((uint32_t)tl[o7] << 16);
      } else {
        const uint32_t *tl = (const uint32_t *)tile + rowbase;
        const uint2 offs = *(const uint2 *)(tab + pe);   // 4 offsets
        w.x = tl[offs.x & 0xffffu]; w.y = tl[offs.x >> 16];
        w.z = tl[offs.y & 0xffffu]; w.w = tl[offs.y >> 16];
      }
      o[c] = w;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
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
