// One-launch prune: score -> Top_T -> compaction (Sec. 3.2 selection, Fig. 1 storage) --
// gfx950, wave64.
//
// Every 256-thread block owns one (unit, row block) item and does three things:
//   A. column sums of squares of its rows -> partial[item] (fp64), then it
//      announces itself on the unit's arrival counter;
//   B. the block that arrives LAST for a unit merges the unit's partials in
//      row-block order, forms the scores with the pre-computed query norms,
//      runs the Top_T selection and publishes the index list; the other blocks
//      of the unit wait for the list (bounded spin);
//   C. every block compacts ITS OWN rows with the published index list.
// Units of more than 64 blocks do B differently: the last block of each GROUP of blocks merges
// the group's partials and publishes the group vector (words with their own validity mark);
// every block then reads the unit's group vectors and makes scores and index list for itself.
// Two forms: k_prune_onepass keeps the block's rows on chip (registers and the
// LDS tiles) from A to C, so K is read from memory once; k_prune_fused streams
// the rows in A and reads them again in C (any block size; the second read comes
// from the memory-side cache or HBM).
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
// another (partial sums, the counter, the index list) moves through relaxed
// device-scope atomic loads and stores, which go to the coherence point
// themselves.  Before it bumps the counter a producer waits until its partial
// sums have been acknowledged (s_waitcnt vmcnt(0) in every wave, then the block
// barrier): a workgroup-scope release fence compiles to nothing here (a block's
// waves share one L1), and without the wait the counter can overtake the data on
// its way to memory.  The index list needs no such ordering: each of its 32-bit
// words carries its own validity mark, the waiting blocks poll the words
// themselves, and k_prune_prep clears them before every call.
#include <stdlib.h>

#include <algorithm>

#include "thk_prune_proto.h"

namespace thk {

// Per unit: query norms, and the counters, index-list words and done marks back to zero.  With
// one query head per unit a wavefront takes a unit (four units per block, nothing shared between
// them); with several, a block takes a unit and its waves share the heads.
template <int DT>
__global__ __launch_bounds__(256) void k_prune_prep(PruneFusedArgs a, int64_t U) {
  __shared__ double hn[4 * kD];
  const int lane = threadIdx.x % kWave;
  int64_t u;
  bool clear;
  if (a.G > 1) {
    u = blockIdx.x;
    block_query_norm<DT, 4>(a.q_obs, u, a.G, a.S_obs, a.qn + (size_t)u * kD, hn);
    clear = threadIdx.x < kWave;
  } else {
    u = (int64_t)blockIdx.x * 4 + threadIdx.x / kWave;
    if (u >= U) return;
    wave_query_norm<DT>(a.q_obs, u, 1, a.S_obs, a.qn + (size_t)u * kD, lane);
    clear = true;
  }
  if (!clear) return;
  if (lane == 0) a.arrived[u] = 0;
  if (a.GS > 0) {
    if (lane < kMaxGroups) a.arrived_g[(size_t)u * kMaxGroups + lane] = 0;
    for (int i = lane; i < kMaxGroups * kD; i += kWave) a.gpartial[(size_t)u * kMaxGroups * kD + i] = 0.0;
  }
  a.idx_pub[(size_t)u * kWave + lane] = 0u;
  for (int i = lane; i < a.NB; i += kWave) a.done[(size_t)u * a.NB + i] = 0;
}

__device__ __forceinline__ bool unit_index_list(const PruneFusedArgs &a, int64_t u, int64_t item,
                                                double *s_part, float *s_sc, int16_t *s_idx,
                                                int *s_flag) {
  const int tid = threadIdx.x;
  // the query norms are needed last; their load travels with the stores below
  const double qn_c = tid < kD ? a.qn[(size_t)u * kD + tid] : 0.0;
  if (tid < kD) pub_store_f64(a.partial + (size_t)item * kD + tid, s_part[tid]);
  block_stores_done();

  const double *src = a.partial + (size_t)u * a.NB * kD;
  if (a.GS > 0) {
    // Units of many blocks, two levels.  The last block of a group of a.GS consecutive blocks
    // merges the group's sums into one vector and publishes it; EVERY block of the unit then
    // reads the (at most 16) group vectors, adds them in group order and makes the index list
    // for itself -- the same bits everywhere.  Nobody waits for a block that waits: the group
    // vectors come from blocks that only had to finish their own rows.
    const int blk = (int)(item - u * a.NB);
    const int g = blk / a.GS;
    const int gsize = min(a.GS, a.NB - g * a.GS);
    double *gp = a.gpartial + (size_t)u * kMaxGroups * kD;
    if (arrive(a.arrived_g + (size_t)u * kMaxGroups + g, gsize, s_flag)) {
      const double gs = merge_partials(src + (size_t)g * a.GS * kD, gsize, s_part);
      if (tid < kD) pub_store_marked(gp + (size_t)g * kD + tid, gs);
    }
    const int n_grp = (a.NB + a.GS - 1) / a.GS;
    // thread (c, half) polls channel c of groups 8 half .. 8 half + 7; all loads in flight at once
    constexpr int HG = kMaxGroups / 2;
    const int c = tid & (kD - 1), j0 = (tid >> 7) * HG;
    unsigned long long w[HG];
#pragma unroll
    for (int j = 0; j < HG; ++j) w[j] = pub_load_bits(gp + (size_t)min(j0 + j, n_grp - 1) * kD + c);
    bool ok;
    for (int n = 0;; ++n) {
      bool miss = false;
#pragma unroll
      for (int j = 0; j < HG; ++j) miss |= (w[j] & 1ull) == 0;
      if (!__any(miss) || n >= a.spin_limit) { ok = !miss; break; }
      __builtin_amdgcn_s_sleep(16);
#pragma unroll
      for (int j = 0; j < HG; ++j)
        if ((w[j] & 1ull) == 0) w[j] = pub_load_bits(gp + (size_t)min(j0 + j, n_grp - 1) * kD + c);
    }
    double kss = 0.0;
#pragma unroll
    for (int j = 0; j < HG; ++j) kss += j0 + j < n_grp ? __longlong_as_double((long long)(w[j] & ~1ull)) : 0.0;
    if (tid == 0) *s_flag = 1;
    __syncthreads();
    if (!ok) *s_flag = 0;      // any thread that ran out of polls
    if (tid >= kD) s_part[c] = kss;
    __syncthreads();
    if (*s_flag == 0) return false;
    if (tid < kD) kss += s_part[c];
    score_and_select(a, u, qn_c, kss, s_sc, s_idx, blk == 0);
    return true;
  }

  if (arrive(a.arrived + u, a.NB, s_flag)) {
    const double kss = merge_partials(src, a.NB, s_part);   // s_part: its sums are published already
    score_and_select(a, u, qn_c, kss, s_sc, s_idx, true);
    if (tid < kWave) {
      const uint32_t lo = 2 * tid < a.T ? (uint16_t)s_idx[2 * tid] : 0u;
      const uint32_t hi = 2 * tid + 1 < a.T ? (uint16_t)s_idx[2 * tid + 1] : 0u;
      __hip_atomic_store(a.idx_pub + (size_t)u * kWave + tid, lo | (hi << 16) | kPubValid, __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
    }
    return true;
  }
  // ---- wait (bounded) for the unit's index list: every word carries its own validity mark, so
  // the list needs no separate flag and no ordering between its words
  if (tid < kWave) {
    const uint32_t *p = a.idx_pub + (size_t)u * kWave + tid;
    uint32_t w = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (int n = 0; __any((w & kPubValid) == 0) && n < a.spin_limit; ++n) {
      __builtin_amdgcn_s_sleep(16);
      if ((w & kPubValid) == 0) w = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    const bool ok = __all((w & kPubValid) != 0);
    if (ok) {
      s_idx[2 * tid] = (int16_t)(w & 0x7fffu);
      s_idx[2 * tid + 1] = (int16_t)((w >> 16) & 0x7fffu);
    }
    if (tid == 0) *s_flag = ok;
  }
  __syncthreads();
  return *s_flag != 0;
}

// Form 1: stream the rows for the column sums, re-read them for the compaction.
template <int DT>
__global__ __launch_bounds__(256) void k_prune_fused(PruneFusedArgs a) {
  using E = Elem<DT>;
  extern __shared__ u32x4 smem[];
  int16_t *tab = (int16_t *)smem;            // 2 KiB
  u32x4 *tiles = smem + 128;                 // 4 x [32][128] elements
  __shared__ double red[4][kD];
  __shared__ double s_part[kD];
  __shared__ float s_sc[kD];
  __shared__ int16_t s_idx[kD];
  __shared__ int s_flag;
  const int tid = threadIdx.x;
  const int64_t item = blockIdx.x;
  const int64_t u = item / a.NB;
  const int blk = (int)(item % a.NB);
  const int64_t s0 = (int64_t)blk * a.RB;
  const int64_t s1 = min(a.S, s0 + a.RB);
  const u32x4 *src = (const u32x4 *)((const char *)a.k + (size_t)u * a.S * kD * E::EB);

  colsum_block<DT, 2, false>(src, s0, s1, s_part, red);
  __syncthreads();
  if (!unit_index_list(a, u, item, s_part, s_sc, s_idx, &s_flag)) return;

  const FlatOut<DT> out((char *)a.kp + (size_t)u * a.kp_unit_rows * a.ld * E::EB);
  compact_build_tab<DT>(tab, s_idx, a.T, a.ld, out.sh);
  __syncthreads();
  const int64_t s1c = min(s1, a.S_keep);   // rows past S_keep stay at full width with the caller
  if (s0 < s1c) compact_rows<DT>(src, out, s0, s1c, a.T, a.ld, tab, tiles);
  if (tid == 0) a.done[item] = 1;
}

// Form 2: K is read from memory ONCE.  The block's rows (NTW tiles of 32 rows per wave, RB =
// 128 * NTW rows) are held from the column sums until the index list arrives: the first
// NTW - NLT tiles of a wave in registers, the last NLT in the wave's LDS tiles, which are idle
// until the compaction anyway.  The compaction then empties the LDS tiles first and stages the
// register tiles through the freed slot.  What hides the wait for the list is the other blocks
// resident on the compute unit; the bytes they hold together cover the bandwidth-delay
// product of the stream.
// registers that hold rows: (NTW - NLT) tiles x 32 (bf16) or 64 (fp32) per lane
template <int DT, int NTW, int NLT>
__global__ __launch_bounds__(256, (NTW - NLT) * 16 * Elem<DT>::EB <= 32 ? 4 : (NTW - NLT) * 16 * Elem<DT>::EB <= 96 ? 3 : 2)
void k_prune_onepass(PruneFusedArgs a) {
  using E = Elem<DT>;
  constexpr int VEC = E::VEC, CPR = kD / VEC, TR = kCompactTileRows, NLD = TR * CPR / kWave;
  constexpr int NRT = NTW - NLT;             // tiles per wave held in registers
  extern __shared__ u32x4 smem[];
  int16_t *tab = (int16_t *)smem;            // 2 KiB
  u32x4 *tiles = smem + 128;                 // [4 waves][NLT] x [32][128] elements
  __shared__ double red[4][kD];
  __shared__ double s_part[kD];
  __shared__ float s_sc[kD];
  __shared__ int16_t s_idx[kD];
  __shared__ int s_flag;
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int64_t item = blockIdx.x;
  const int64_t u = item / a.NB;
  const int blk = (int)(item % a.NB);
  const int64_t s0 = (int64_t)blk * a.RB;   // a.RB == 128 * NTW
  const int64_t s1 = min(a.S, s0 + a.RB);
  const u32x4 *src = (const u32x4 *)((const char *)a.k + (size_t)u * a.S * kD * E::EB);
  u32x4 *wtile = tiles + (size_t)wave * NLT * Tile<DT>::CHUNKS;   // this wave's NLT tiles
  if (a.ld != a.T)
#pragma unroll
    for (int n = 0; n < NLT; ++n) tile_clear_padding<DT>(wtile + (size_t)n * Tile<DT>::CHUNKS, lane);

  // tile n of this wave = rows s0 + (4 n + wave) * 32 .. + 32, nr of them inside [s0, hi)
  auto tile_row0 = [&](int n) { return s0 + (int64_t)(4 * n + wave) * TR; };
  auto tile_rows = [&](int n, int64_t hi) { return (int)max((int64_t)0, min((int64_t)TR, hi - tile_row0(n))); };

  // A launch of two or more rounds of resident blocks would run in lock-step (everybody loads,
  // everybody waits for the index lists, everybody stores).  The first round's units therefore
  // start one after the other, a unit's transfer time apart; the later rounds inherit the
  // spacing because a unit's blocks leave, and their successors start, together.
  if (item < a.stagger_blocks) {
    int ticks = (int)(u % a.stagger_units) * a.stagger_ticks;
    for (; ticks >= 127; ticks -= 127) __builtin_amdgcn_s_sleep(127);
    for (; ticks >= 16; ticks -= 16) __builtin_amdgcn_s_sleep(16);
  }

  // ---- load: every chunk of the block's rows is in flight at once ----------------------------
  u32x4 r[NTW][NLD];
#pragma unroll
  for (int n = 0; n < NTW; ++n) {
    const int nr = tile_rows(n, s1);
    const u32x4 *tsrc = src + (size_t)tile_row0(n) * CPR;
    const int cmax = nr * CPR - 1;
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
      const u32x4 zero = {0u, 0u, 0u, 0u};
      // chunks past a ragged tile's end repeat its last chunk (in bounds; excluded below)
      r[n][j] = nr > 0 ? ld_stream(tsrc + min(j * kWave + lane, cmax)) : zero;
    }
  }

  // ---- column sums of squares; the last NLT tiles then move to LDS -----------------------------
  double dacc[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) dacc[v] = 0.0;
#pragma unroll
  for (int nn = 0; nn < NTW; ++nn) {
    const int n = (nn + NRT) % NTW;          // LDS-bound tiles first: their registers free up early
    const int nr = tile_rows(n, s1);
    float facc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) facc[v] = 0.f;
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
      float f[VEC];
      E::unpack(r[n][j], f);
      const bool valid = (j * kWave + lane) / CPR < nr;
#pragma unroll
      for (int v = 0; v < VEC; ++v) facc[v] = valid ? fmaf(f[v], f[v], facc[v]) : facc[v];
      if (n >= NRT) wtile[(size_t)(n - NRT) * Tile<DT>::CHUNKS + Tile<DT>::slot(j * kWave + lane)] = r[n][j];
    }
#pragma unroll
    for (int v = 0; v < VEC; ++v) dacc[v] += (double)facc[v];
  }
#pragma unroll
  for (int v = 0; v < VEC; ++v) dacc[v] = add_lane_groups<CPR>(dacc[v]);
  if (lane < CPR)
#pragma unroll
    for (int v = 0; v < VEC; ++v) red[wave][lane * VEC + v] = dacc[v];
  __syncthreads();
  if (tid < kD) s_part[tid] = ((red[0][tid] + red[1][tid]) + red[2][tid]) + red[3][tid];
  __syncthreads();

  if (!unit_index_list(a, u, item, s_part, s_sc, s_idx, &s_flag)) return;

  // ---- compaction: the LDS tiles first, then the register tiles through slot 0 ---------------
  const FlatOut<DT> dst((char *)a.kp + (size_t)u * a.kp_unit_rows * a.ld * E::EB);
  compact_build_tab<DT>(tab, s_idx, a.T, a.ld, dst.sh);
  __syncthreads();
  const int64_t s1c = min(s1, a.S_keep);
#pragma unroll
  for (int n = NRT; n < NTW; ++n) {
    const int nr = tile_rows(n, s1c);
    if (nr > 0) compact_emit_tile<DT>(wtile + (size_t)(n - NRT) * Tile<DT>::CHUNKS, dst, tile_row0(n), nr, a.ld, tab, lane);
  }
#pragma unroll
  for (int n = 0; n < NRT; ++n) {
    const int nr = tile_rows(n, s1c);
    if (nr > 0) {   // wave-uniform
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();       // the slot's previous tile has been read
#pragma unroll
      for (int j = 0; j < NLD; ++j) wtile[Tile<DT>::slot(j * kWave + lane)] = r[n][j];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      compact_emit_tile<DT>(wtile, dst, tile_row0(n), nr, a.ld, tab, lane);
    }
  }
  if (tid == 0) a.done[item] = 1;
}

// One block per unit: compact the row blocks that k_prune_fused left undone.
template <int DT>
__global__ __launch_bounds__(256) void k_prune_repair(PruneFusedArgs a) {
  using E = Elem<DT>;
  extern __shared__ u32x4 smem[];
  int16_t *tab = (int16_t *)smem;
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
  const FlatOut<DT> dst((char *)a.kp + (size_t)u * a.kp_unit_rows * a.ld * E::EB);
  if (a.GS > 0) {
    // The blocks of a two-level unit make the list for themselves and block 0 stores the
    // caller's copy, so the copy may be missing.  All group vectors are there by now: the same
    // sums in the same order give the same list.
    __shared__ float s_sc[kD];
    __shared__ int16_t s_idx[kD];
    const int tid = threadIdx.x;
    const int n_grp = (a.NB + a.GS - 1) / a.GS;
    const double *gp = a.gpartial + (size_t)u * kMaxGroups * kD;
    double kss = 0.0;
    if (tid < kD) {
      double half[2] = {0.0, 0.0};
      for (int j = 0; j < n_grp; ++j)
        half[j / (kMaxGroups / 2)] += __longlong_as_double((long long)(pub_load_bits(gp + (size_t)j * kD + tid) & ~1ull));
      kss = half[0] + half[1];
    }
    score_and_select(a, u, tid < kD ? a.qn[(size_t)u * kD + tid] : 0.0, kss, s_sc, s_idx, true);
    compact_build_tab<DT>(tab, s_idx, a.T, a.ld, dst.sh);
  } else {
    compact_build_tab<DT>(tab, a.idx + (size_t)u * a.T, a.T, a.ld, dst.sh);
  }
  __syncthreads();
  const u32x4 *src = (const u32x4 *)((const char *)a.k + (size_t)u * a.S * kD * E::EB);
  for (int blk = 0; blk < a.NB; ++blk) {
    if (done[blk]) continue;   // block-uniform: every thread reads the same byte
    const int64_t s0 = (int64_t)blk * a.RB;
    const int64_t s1c = min(a.S_keep, s0 + a.RB);
    if (s0 < s1c) compact_rows<DT>(src, dst, s0, s1c, a.T, a.ld, tab, tiles);
  }
}

// blocks per group for a unit of NB blocks (0 = one-level arrival)
static int group_size(int NB) { return NB > 64 ? (NB + kMaxGroups - 1) / kMaxGroups : 0; }

size_t prune_fused_ws_bytes(int64_t U, int NB) {
  size_t b = (size_t)U * NB * kD * sizeof(double);   // partial
  if (group_size(NB) > 0) {
    b += (size_t)U * kMaxGroups * kD * sizeof(double);   // gpartial
    b += (size_t)U * kMaxGroups * sizeof(int);           // arrived_g
  }
  b += (size_t)U * kD * sizeof(double);              // qn
  b += (size_t)U * sizeof(int);                      // arrived
  b = (b + 15) & ~(size_t)15;
  b += (size_t)U * kWave * sizeof(uint32_t);         // idx_pub
  b += ((size_t)U * NB + 15) & ~(size_t)15;          // done
  return b;
}

hipError_t launch_prune_fused(int dtype, const void *q_obs, const void *k, float *score, int16_t *idx,
                              void *kp, void *ws, int64_t U, int64_t S, int64_t S_keep,
                              int64_t kp_unit_rows, int G, int S_obs, int T, int ld, int NB, int64_t RB,
                              int hold, int spin_limit, int given, hipStream_t st) {
  clear_stale_hip_error();
  PruneFusedArgs a;
  a.given = given;
  const int eb = dtype == THK_BF16 ? 2 : 4;
  a.k = k; a.q_obs = q_obs; a.kp = kp; a.score = score; a.idx = idx;
  char *w = (char *)ws;
  a.partial = (double *)w; w += (size_t)U * NB * kD * sizeof(double);
  a.GS = group_size(NB);
  a.stagger_blocks = 0; a.stagger_units = 1; a.stagger_ticks = 0;
  if (hold != 0) {
    // resident blocks per compute unit (LDS decides): 3 with bf16 tiles, 2 with fp32 tiles
    const int64_t resident = (int64_t)kCUs * (dtype == THK_BF16 ? 3 : 2);
    const int64_t total = U * NB;
    const int64_t res_units = resident / NB;
    double ns = -1.0;
    if (env_switches().stagger_set) ns = env_switches().stagger_ns;
    else if (res_units >= 2 && total >= 2 * resident)
      // 0.6 of the time a unit's rows in and compacted rows out take at 5.7 TB/s: the full time
      // would be the spacing of the steady state, but the first round loads against no stores
      // and a wider spread only delays it (swept 0..1.5: 0.5-0.7 is best from 2 to 50 rounds)
      ns = 0.6 * (double)S * kD * eb * 1.5 / 5.7e3;
    if (ns > 0.0 && res_units >= 2) {
      a.stagger_blocks = (int32_t)(res_units * NB);
      a.stagger_units = (int32_t)res_units;
      a.stagger_ticks = std::max((int32_t)(ns * 2.4 / 64.0), 1);   // 2.4 GHz, s_sleep counts 64-cycle ticks
    }
  }
  a.gpartial = nullptr; a.arrived_g = nullptr;
  if (a.GS > 0) {
    a.gpartial = (double *)w; w += (size_t)U * kMaxGroups * kD * sizeof(double);
    a.arrived_g = (int *)w;   w += (size_t)U * kMaxGroups * sizeof(int);
  }
  a.qn = (double *)w;      w += (size_t)U * kD * sizeof(double);
  a.arrived = (int *)w;    w += (size_t)U * sizeof(int);
  w = (char *)(((uintptr_t)w + 15) & ~(uintptr_t)15);
  a.idx_pub = (uint32_t *)w; w += (size_t)U * kWave * sizeof(uint32_t);
  a.done = (unsigned char *)w;
  a.S = S; a.S_keep = S_keep; a.kp_unit_rows = kp_unit_rows; a.RB = RB; a.T = T; a.ld = ld; a.G = G; a.S_obs = S_obs; a.NB = NB; a.spin_limit = spin_limit;
  const size_t lds = 2048 + 4 * compact_tile_bytes(eb);
  const dim3 gu((unsigned)U), gi((unsigned)(U * NB));
  // hold == 0: the re-reading form; otherwise RB == 128 * hold and the rows are held on chip
  const void *main_fn = nullptr;
  int nlt = 1;   // LDS tiles per wave
  if (dtype == THK_BF16) {
    switch (hold) {
      case 0: main_fn = (const void *)k_prune_fused<THK_BF16>; break;
      case 1: main_fn = (const void *)k_prune_onepass<THK_BF16, 1, 1>; break;
      case 2: main_fn = (const void *)k_prune_onepass<THK_BF16, 2, 1>; break;
      case 4: main_fn = (const void *)k_prune_onepass<THK_BF16, 4, 1>; break;
    }
  } else {
    switch (hold) {
      case 0: main_fn = (const void *)k_prune_fused<THK_F32>; break;
      case 1: main_fn = (const void *)k_prune_onepass<THK_F32, 1, 1>; break;
      case 2: main_fn = (const void *)k_prune_onepass<THK_F32, 2, 1>; break;
    }
  }
  if (main_fn == nullptr || (hold != 0 && RB != 128 * hold)) return hipErrorInvalidValue;
  const size_t lds_main = 2048 + 4 * (size_t)nlt * compact_tile_bytes(eb);
  {
    // one record per main kernel: [dtype][hold]
    static DynLds main_set[2][5], repair_set;
    hipError_t e = ensure_dyn_lds(main_fn, lds_main, main_set[dtype == THK_BF16 ? 1 : 0][hold]);
    if (e != hipSuccess) return e;
    if (dtype == THK_F32) e = ensure_dyn_lds((const void *)k_prune_repair<THK_F32>, lds, repair_set);
    if (e != hipSuccess) return e;
  }
  void *kargs[] = {(void *)&a};
  const unsigned prep_blocks = (unsigned)(a.G > 1 ? U : (U + 3) / 4);
  if (dtype == THK_BF16)
    hipLaunchKernelGGL((k_prune_prep<THK_BF16>), dim3(prep_blocks), dim3(256), 0, st, a, U);
  else
    hipLaunchKernelGGL((k_prune_prep<THK_F32>), dim3(prep_blocks), dim3(256), 0, st, a, U);
  hipError_t le = launch_main_kernel(main_fn, gi, dim3(256), kargs, lds_main, st);
  if (le != hipSuccess) return le;
  if (dtype == THK_BF16)
    hipLaunchKernelGGL((k_prune_repair<THK_BF16>), gu, dim3(256), lds, st, a);
  else
    hipLaunchKernelGGL((k_prune_repair<THK_F32>), gu, dim3(256), lds, st, a);
  return hipGetLastError();
}

}  // namespace thk
