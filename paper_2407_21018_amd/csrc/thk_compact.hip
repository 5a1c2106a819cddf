// Key compaction K_pruned[s][t] = K[s][idx[t]] (Fig. 1; Sec. 3.3), full-width row
// copies and the tail append (gfx950, wave64).  Pure byte movement: no arithmetic
// on values.
#include "thk_prune_device.h"

namespace thk {

// A run of rows of K_pruned is a run of bytes (dense rows, or rows with padding behind them,
// which is written as zeros); the unit may start and end anywhere (see compact_rows).
template <int DT>
__global__ __launch_bounds__(256) void k_compact_flat(CompactArgs a) {
  using E = Elem<DT>;
  extern __shared__ u32x4 smem[];
  int16_t *tab = (int16_t *)smem;                         // [8 * T], padded to 2 KiB
  const int64_t u = blockIdx.x / a.blocks_per_unit;
  const int blk = (int)(blockIdx.x % a.blocks_per_unit);
  const int64_t s0 = (int64_t)blk * a.rows_per_block;
  const int64_t s1 = min(a.n_rows, s0 + a.rows_per_block);
  const FlatOut<DT> out((char *)a.dst + ((size_t)u * a.dst_unit_rows + a.dst_row0) * a.ld * E::EB);
  compact_build_tab<DT>(tab, a.idx + (size_t)u * a.T, a.T, a.ld, out.sh);
  __syncthreads();
  compact_rows<DT>((const u32x4 *)((const char *)a.src + ((size_t)u * a.src_unit_rows + a.src_row0) * kD * E::EB),
                   out, s0, s1, a.T, a.ld, tab, smem + 128);
}

// Full-width row copy dst[u][dst_row0 + r][:] = src[u][src_row0 + r][:], r < n_rows.
// One block per unit; rows move in ascending chunks, each chunk loaded completely
// before any of it is stored, so a downward shift inside one buffer
// (dst_row0 <= src_row0) is safe.  src and dst may alias: neither is declared restrict.
template <int DT>
__global__ __launch_bounds__(256) void k_copy_rows(const void *src, void *dst,
                                                   int64_t src_unit_rows, int64_t src_row0,
                                                   int64_t dst_unit_rows, int64_t dst_row0,
                                                   int64_t n_rows) {
  using E = Elem<DT>;
  constexpr int CPR = kD / E::VEC;     // 16-byte chunks per row
  constexpr int PER = 8;               // chunks per thread per pass
  const int64_t u = blockIdx.x;
  const u32x4 *s = (const u32x4 *)src + ((size_t)u * src_unit_rows + src_row0) * CPR;
  u32x4 *d = (u32x4 *)dst + ((size_t)u * dst_unit_rows + dst_row0) * CPR;
  const int64_t total = n_rows * CPR;
  for (int64_t c0 = 0; c0 < total; c0 += 256 * PER) {
    u32x4 r[PER];
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      const int64_t c = c0 + (int64_t)j * 256 + threadIdx.x;
      if (c < total) r[j] = s[c];
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      const int64_t c = c0 + (int64_t)j * 256 + threadIdx.x;
      if (c < total) d[c] = r[j];
    }
    __syncthreads();
  }
}

// The same copy when source and destination ranges cannot touch each other: many blocks per
// unit, each streaming its own run of rows (eight 16-byte chunks in flight per thread).
template <int DT>
__global__ __launch_bounds__(256) void k_copy_rows_wide(const void *__restrict__ src, void *__restrict__ dst,
                                                        int64_t src_unit_rows, int64_t src_row0,
                                                        int64_t dst_unit_rows, int64_t dst_row0,
                                                        int64_t n_rows, int64_t rows_per_block, int blocks_per_unit) {
  using E = Elem<DT>;
  constexpr int CPR = kD / E::VEC;
  constexpr int PER = 8;
  const int64_t u = blockIdx.x / blocks_per_unit;
  const int64_t r0 = (int64_t)(blockIdx.x % blocks_per_unit) * rows_per_block;
  const int64_t r1 = min(n_rows, r0 + rows_per_block);
  const u32x4 *s = (const u32x4 *)src + ((size_t)u * src_unit_rows + src_row0 + r0) * CPR;
  u32x4 *d = (u32x4 *)dst + ((size_t)u * dst_unit_rows + dst_row0 + r0) * CPR;
  const int64_t total = (r1 - r0) * CPR;
  for (int64_t c0 = 0; c0 < total; c0 += 256 * PER) {
    u32x4 r[PER];
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      const int64_t c = c0 + (int64_t)j * 256 + threadIdx.x;
      if (c < total) r[j] = ld_stream(s + c);
    }
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      const int64_t c = c0 + (int64_t)j * 256 + threadIdx.x;
      if (c < total) st_stream(d + c, r[j]);
    }
  }
}

// One new token per unit: K_tail[u][k_row] = k_new[u], Vdst[u][v_row] = v_new[u].
template <int DT>
__global__ __launch_bounds__(256) void k_tail_append(const void *__restrict__ k_new,
                                                     const void *__restrict__ v_new,
                                                     void *__restrict__ k_dst, void *__restrict__ v_dst,
                                                     int64_t U, int64_t k_unit_rows, int64_t k_row,
                                                     int64_t v_unit_rows, int64_t v_row) {
  using E = Elem<DT>;
  constexpr int CPR = kD / E::VEC;   // 16-byte chunks per row
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= U * CPR) return;
  const int64_t u = i / CPR;
  const int c = (int)(i % CPR);
  ((u32x4 *)k_dst)[((size_t)u * k_unit_rows + k_row) * CPR + c] = ((const u32x4 *)k_new)[i];
  ((u32x4 *)v_dst)[((size_t)u * v_unit_rows + v_row) * CPR + c] = ((const u32x4 *)v_new)[i];
}

hipError_t launch_compact(int dtype, const void *src, int64_t src_unit_rows, int64_t src_row0,
                          const int16_t *idx, void *dst, int64_t dst_unit_rows, int64_t dst_row0,
                          int64_t U, int64_t n_rows, int T, int ld_keep, hipStream_t st) {
  clear_stale_hip_error();
  if (n_rows <= 0) return hipSuccess;
  const int eb = dtype == THK_BF16 ? 2 : 4;
  CompactArgs a;
  a.src = src; a.dst = dst; a.idx = idx;
  a.src_unit_rows = src_unit_rows; a.src_row0 = src_row0;
  a.dst_unit_rows = dst_unit_rows; a.dst_row0 = dst_row0; a.n_rows = n_rows;
  a.T = T; a.ld = ld_keep;
  // 4 waves x 4 tiles of 32 rows; smaller blocks (down to one tile per wave) while the call has
  // fewer than four blocks per compute unit: a wave's tiles go load -> LDS -> gather -> store one
  // after the other, so a small call is as long as its longest block
  a.rows_per_block = 512;
  while (a.rows_per_block > 128 && U * ((n_rows + a.rows_per_block - 1) / a.rows_per_block) < 4 * kCUs) a.rows_per_block /= 2;
  a.blocks_per_unit = (int)((n_rows + a.rows_per_block - 1) / a.rows_per_block);
  const dim3 grid((unsigned)(U * a.blocks_per_unit)), block(256);
  const size_t lds = 2048 + 4 * compact_tile_bytes(eb);
  void *kargs[] = {(void *)&a};
  const void *fn = dtype == THK_BF16 ? (const void *)k_compact_flat<THK_BF16> : (const void *)k_compact_flat<THK_F32>;
  const hipError_t e = launch_main_kernel(fn, grid, block, kargs, lds, st);
  return e != hipSuccess ? e : hipGetLastError();
}

hipError_t launch_copy_rows(int dtype, const void *src, int64_t src_unit_rows, int64_t src_row0, void *dst,
                            int64_t dst_unit_rows, int64_t dst_row0, int64_t U, int64_t n_rows,
                            hipStream_t st) {
  clear_stale_hip_error();
  if (n_rows <= 0) return hipSuccess;
  // byte ranges the call touches, over all units: disjoint ranges may be copied in any order
  auto ceil_div = [](int64_t a, int64_t b) { return (a + b - 1) / b; };
  constexpr int64_t kMaxBlocks = 0x7fffffff;
  const size_t rowb = (size_t)kD * (dtype == THK_BF16 ? 2 : 4);
  const char *s_lo = (const char *)src + (size_t)src_row0 * rowb;
  const char *s_hi = (const char *)src + ((size_t)(U - 1) * src_unit_rows + src_row0 + n_rows) * rowb;
  const char *d_lo = (const char *)dst + (size_t)dst_row0 * rowb;
  const char *d_hi = (const char *)dst + ((size_t)(U - 1) * dst_unit_rows + dst_row0 + n_rows) * rowb;
  const bool disjoint = s_hi <= d_lo || d_hi <= s_lo;
  const dim3 block(256);
  if (disjoint && n_rows > 64) {
    // ~8 blocks per compute unit, at least 64 rows each
    int64_t bpu = ceil_div((int64_t)kCUs * 8, U);
    const int64_t cap = ceil_div(n_rows, 64);
    if (bpu > cap) bpu = cap;
    if (bpu < 1) bpu = 1;
    const int64_t rpb = ceil_div(n_rows, bpu);
    bpu = ceil_div(n_rows, rpb);
    if (U * bpu <= kMaxBlocks) {
      const dim3 grid((unsigned)(U * bpu));
      if (dtype == THK_BF16)
        hipLaunchKernelGGL((k_copy_rows_wide<THK_BF16>), grid, block, 0, st, src, dst, src_unit_rows, src_row0, dst_unit_rows, dst_row0, n_rows, rpb, (int)bpu);
      else
        hipLaunchKernelGGL((k_copy_rows_wide<THK_F32>), grid, block, 0, st, src, dst, src_unit_rows, src_row0, dst_unit_rows, dst_row0, n_rows, rpb, (int)bpu);
      return hipGetLastError();
    }
  }
  const dim3 grid((unsigned)U);
  if (dtype == THK_BF16)
    hipLaunchKernelGGL((k_copy_rows<THK_BF16>), grid, block, 0, st, src, dst, src_unit_rows, src_row0, dst_unit_rows, dst_row0, n_rows);
  else
    hipLaunchKernelGGL((k_copy_rows<THK_F32>), grid, block, 0, st, src, dst, src_unit_rows, src_row0, dst_unit_rows, dst_row0, n_rows);
  return hipGetLastError();
}

hipError_t launch_tail_append(int dtype, const void *k_new, const void *v_new, void *k_dst, void *v_dst,
                              int64_t U, int64_t k_unit_rows, int64_t k_row, int64_t v_unit_rows,
                              int64_t v_row, hipStream_t st) {
  clear_stale_hip_error();
  const int cpr = dtype == THK_BF16 ? 16 : 32;
  const dim3 grid((unsigned)((U * cpr + 255) / 256)), block(256);
  if (dtype == THK_BF16)
    hipLaunchKernelGGL((k_tail_append<THK_BF16>), grid, block, 0, st, k_new, v_new, k_dst, v_dst, U, k_unit_rows, k_row, v_unit_rows, v_row);
  else
    hipLaunchKernelGGL((k_tail_append<THK_F32>), grid, block, 0, st, k_new, v_new, k_dst, v_dst, U, k_unit_rows, k_row, v_unit_rows, v_row);
  return hipGetLastError();
}

}  // namespace thk
