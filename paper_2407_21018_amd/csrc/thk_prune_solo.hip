// Single-launch prune: score -> Top_T -> compaction (Sec. 3.2 selection, Fig. 1 storage) with
// NOTHING before or after the one kernel -- gfx950, wave64.
//
// The three-launch form (thk_prune_fused.hip) needs a kernel in front that clears the hand-off
// state and computes the query norms, and one behind that compacts what a block left undone
// when its bounded wait ran out.  For calls of a few hundred microseconds and less those two
// launches and the gaps around them are 10-15 % of the call.  Here both jobs move inside:
//
//   * Blocks 0 .. U-1 of the grid are PROLOGUE blocks, one per unit, the U * NB row blocks of
//     k_prune_onepass follow.  A prologue block has no rows; it clears its unit's hand-off state
//     (index-list words, group vectors, give-up flags and tickets), computes the query norms,
//     waits until all of that has been acknowledged, and only then initialises the unit's
//     arrival counters.  (A unit's prologue block directly in front of its row blocks, the
//     first layout, put NB + 1 blocks per unit into a chip that holds a whole number of NB-block
//     units: units straddled the rounds of resident blocks and long launches ran 6-12 % slower.)
//   * The arrival counters are the first shared thing a row block touches, and they are TAGGED:
//     the upper 48 bits hold the call's nonce.  A block whose atomic add returns a word with
//     another tag has arrived before the prologue's initialisation (which will overwrite what
//     it added): it waits for the tag and adds again.  A block that has arrived under the right
//     tag is thereby ordered after everything the prologue published.  Nothing has to be clean
//     when the kernel starts.  The block that completes a counter stores 0 into it, so that a
//     replay of the same launch from a graph, which carries the same nonce, does not mistake
//     the previous replay's count for its own.
//   * One block of every unit never waits: the FINISHER, whose arrival completes the unit's
//     sums.  A block that gives up waiting raises a flag for its rows and draws a ticket from
//     the unit's give-up counter; the finisher draws the closing ticket, learns from it how
//     many blocks gave up before, and compacts their rows after its own (re-reading them).
//     A block that gives up later than that finds the closing ticket in the counter: the list is
//     there by then, so it fetches it and carries on by itself.  Every block exits whatever the
//     others do.  All sums run in a fixed order: the result does not depend on who arrives last.
//
// Waiting is safe for the same reason as in the three-launch form: a block only waits for blocks
// of its own unit, which have lower or neighbouring block numbers and were dispatched with it
// (the prologue blocks have the lowest numbers of all).
#include <algorithm>
#include <atomic>
#include <chrono>

#include "thk_prune_proto.h"

namespace thk {

// What a block knows when solo_index_list returns.
enum ListState { kGaveUp = 0, kHaveList = 1, kFinisher = 2 };
constexpr int kFinisherDone = 1 << 24;   // the finisher's closing ticket on the give-up counter
constexpr int kSurePolls = 1 << 20;      // polls for something that is known to be in place
constexpr int kInitPolls = 1 << 22;      // polls for the prologue's initialisation (a block that was dispatched earlier)

// ---- the prologue block --------------------------------------------------------------------
// lds: at least 5 * 128 doubles.
template <int DT>
__device__ __forceinline__ void solo_prologue(const PruneFusedArgs &a, int64_t u, double *lds) {
  const int tid = threadIdx.x;
  double *hn = lds, *qn_l = lds + 4 * kD;
  // test hook (THK_PRUNE_PROLOGUE_DELAY_US): a late prologue makes the row blocks arrive on
  // counters that are not initialised yet, the path that otherwise needs an unlucky schedule
  for (int t = a.prologue_delay; t > 0; t -= 127) __builtin_amdgcn_s_sleep(127);
  if (tid < kWave) __hip_atomic_store(a.idx_pub + (size_t)u * kWave + tid, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  for (int i = tid; i < a.NB; i += 256)
    __hip_atomic_store(a.undone + (size_t)u * a.NB + i, (unsigned char)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (tid == 0) {
    __hip_atomic_store(a.gaveup + u, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(a.arrived + u, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (a.GS > 0)
    for (int i = tid; i < kMaxGroups * kD; i += 256) pub_store_f64(a.gpartial + (size_t)u * kMaxGroups * kD + i, 0.0);
  block_query_norm<DT, 4>(a.q_obs, u, a.G, a.S_obs, qn_l, hn);
  __syncthreads();
  if (tid < kD) pub_store_f64(a.qn + (size_t)u * kD + tid, qn_l[tid]);
  block_stores_done();
  // everything above has landed: the counters may now be found initialised
  if (a.GS > 0) {
    const int n_grp = (a.NB + a.GS - 1) / a.GS;
    if (tid < n_grp)
      __hip_atomic_store(a.tctr_g + (size_t)u * kMaxGroups + tid, a.nonce << 16, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  } else if (tid == 0) {
    __hip_atomic_store(a.tctr + u, a.nonce << 16, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// One arrival on a tagged counter: true in every thread of the block that makes the count `full`.
__device__ __forceinline__ bool arrive_tagged(unsigned long long *ctr, unsigned long long nonce, int full,
                                              int *s_flag) {
  if (threadIdx.x == 0) {
    unsigned long long old = atomicAdd(ctr, 1ull);
    if ((old >> 16) != nonce) {
      // earlier than the prologue's initialisation, whose store wipes what was just added
      for (int n = 0; n < kInitPolls; ++n) {
        if ((__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >> 16) == nonce) break;
        __builtin_amdgcn_s_sleep(8);
      }
      old = atomicAdd(ctr, 1ull);
    }
    const bool last = (int)(old & 0xffffu) == full - 1;
    // nobody comes after the last arrival: leave a word without the tag behind
    if (last) __hip_atomic_store(ctr, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *s_flag = last;
  }
  __syncthreads();
  const bool last = *s_flag != 0;
  __syncthreads();   // everyone has read the flag before it is reused
  return last;
}

// One-level form: the published index list -> s_idx, polling at most `limit` times.  True in
// every thread if the whole list was there.
__device__ __forceinline__ bool read_list_words(const PruneFusedArgs &a, int64_t u, int16_t *s_idx, int *s_flag,
                                                int limit) {
  const int tid = threadIdx.x;
  if (tid < kWave) {
    const uint32_t *p = a.idx_pub + (size_t)u * kWave + tid;
    uint32_t w = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (int n = 0; __any((w & kPubValid) == 0) && n < limit; ++n) {
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
  const bool ok = *s_flag != 0;
  __syncthreads();   // everyone has read the flag before it is reused
  return ok;
}

// Two-level form: the unit's column sums from its (at most 16) group vectors, added in group
// order, polling at most `limit` times.  Thread (c, half) polls channel c of groups 8 half ..
// 8 half + 7, all loads in flight at once.  True in every thread if all vectors were there; the
// sum is then valid in threads < 128.  s_part: 128 doubles of LDS.
__device__ __forceinline__ bool read_group_sums(const PruneFusedArgs &a, int64_t u, double *s_part, int *s_flag,
                                                int limit, double &kss) {
  const int tid = threadIdx.x;
  const double *gp = a.gpartial + (size_t)u * kMaxGroups * kD;
  const int n_grp = (a.NB + a.GS - 1) / a.GS;
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
    if (!__any(miss) || n >= limit) { ok = !miss; break; }
    __builtin_amdgcn_s_sleep(16);
#pragma unroll
    for (int j = 0; j < HG; ++j)
      if ((w[j] & 1ull) == 0) w[j] = pub_load_bits(gp + (size_t)min(j0 + j, n_grp - 1) * kD + c);
  }
  kss = 0.0;
#pragma unroll
  for (int j = 0; j < HG; ++j) kss += j0 + j < n_grp ? __longlong_as_double((long long)(w[j] & ~1ull)) : 0.0;
  if (tid == 0) *s_flag = 1;
  __syncthreads();
  if (!ok) *s_flag = 0;      // any thread that ran out of polls
  if (tid >= kD) s_part[c] = kss;
  __syncthreads();
  const bool all_ok = *s_flag != 0;
  if (tid < kD) kss += s_part[c];
  __syncthreads();           // flag and s_part may be reused
  return all_ok;
}

// A row block's way from its column sums (s_part) to the unit's index list (s_idx).
// item: u * NB + the block's number among the unit's row blocks.
__device__ __forceinline__ int solo_index_list(const PruneFusedArgs &a, int64_t u, int64_t item, double *s_part,
                                               float *s_sc, int16_t *s_idx, int *s_flag) {
  const int tid = threadIdx.x;
  if (tid < kD) pub_store_f64(a.partial + (size_t)item * kD + tid, s_part[tid]);
  block_stores_done();

  const double *src = a.partial + (size_t)u * a.NB * kD;
  if (a.GS > 0) {
    // Two levels: the last block of a group of a.GS consecutive blocks merges the group's sums
    // into one vector and publishes it; EVERY block of the unit then reads the (at most 16)
    // group vectors, adds them in group order and makes the index list for itself -- the same
    // bits everywhere.  The block that publishes the unit's LAST vector is the finisher: every
    // publisher counts its group only after the vector has landed, so the finisher finds all of
    // them at its first look.  It also stores the caller's copy of scores and list.
    const int blk = (int)(item - u * a.NB);
    const int g = blk / a.GS;
    const int gsize = min(a.GS, a.NB - g * a.GS);
    const int n_grp = (a.NB + a.GS - 1) / a.GS;
    double *gp = a.gpartial + (size_t)u * kMaxGroups * kD;
    bool finisher = false;
    const bool group_last = arrive_tagged(a.tctr_g + (size_t)u * kMaxGroups + g, a.nonce, gsize, s_flag);
    // from here on the prologue's work is visible: the query norms travel with whatever comes next
    const double qn_c = tid < kD ? pub_load_f64(a.qn + (size_t)u * kD + tid) : 0.0;
    if (group_last) {
      const double gs = merge_partials(src + (size_t)g * a.GS * kD, gsize, s_part);
      if (tid < kD) pub_store_marked(gp + (size_t)g * kD + tid, gs);
      block_stores_done();
      finisher = arrive(a.arrived + u, n_grp, s_flag);
    }
    double kss;
    if (!read_group_sums(a, u, s_part, s_flag, finisher ? kSurePolls : a.spin_limit, kss)) return kGaveUp;
    score_and_select(a, u, qn_c, kss, s_sc, s_idx, finisher);
    return finisher ? kFinisher : kHaveList;
  }

  if (arrive_tagged(a.tctr + u, a.nonce, a.NB, s_flag)) {
    const double qn_c = tid < kD ? pub_load_f64(a.qn + (size_t)u * kD + tid) : 0.0;
    const double kss = merge_partials(src, a.NB, s_part);   // s_part: its sums are published already
    score_and_select(a, u, qn_c, kss, s_sc, s_idx, true);
    if (tid < kWave) {
      const uint32_t lo = 2 * tid < a.T ? (uint16_t)s_idx[2 * tid] : 0u;
      const uint32_t hi = 2 * tid + 1 < a.T ? (uint16_t)s_idx[2 * tid + 1] : 0u;
      __hip_atomic_store(a.idx_pub + (size_t)u * kWave + tid, lo | (hi << 16) | kPubValid, __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
    }
    return kFinisher;
  }
  // ---- wait (bounded) for the unit's index list
  return read_list_words(a, u, s_idx, s_flag, a.spin_limit) ? kHaveList : kGaveUp;
}

// A block whose wait ran out leaves its rows to the unit's finisher: it raises its flag, makes
// sure the flag has landed, and draws a ticket.  A ticket drawn after the finisher's closing one
// means that the finisher will not look again -- and that the list is in place: the block then
// fetches it after all (true) and goes on as usual.
__device__ __forceinline__ bool hand_over_rows(const PruneFusedArgs &a, int64_t u, int64_t item, double *s_part,
                                               float *s_sc, int16_t *s_idx, int *s_flag) {
  const int tid = threadIdx.x;
  if (tid == 0)
    __hip_atomic_store(a.undone + item, (unsigned char)1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  block_stores_done();
  if (tid == 0) *s_flag = atomicAdd(a.gaveup + u, 1) >= kFinisherDone;
  __syncthreads();
  const bool late = *s_flag != 0;
  __syncthreads();
  if (!late) return false;
  if (a.GS > 0) {
    const double qn_c = tid < kD ? pub_load_f64(a.qn + (size_t)u * kD + tid) : 0.0;
    double kss;
    read_group_sums(a, u, s_part, s_flag, kSurePolls, kss);
    score_and_select(a, u, qn_c, kss, s_sc, s_idx, false);
  } else {
    read_list_words(a, u, s_idx, s_flag, kSurePolls);
  }
  return true;
}

// The finisher closes the unit BEFORE it compacts its own rows: it draws the closing ticket from
// the give-up counter, whose value is the number of blocks that gave up so far (their flags are
// in place: a block raises its flag, waits for the acknowledgement, and only then draws its
// ticket).  A block that gives up later finds the closing ticket, fetches the list -- published
// before the ticket was drawn; the late block polls for it all the same -- and carries on by
// itself.  (Drawing the ticket after the finisher's own rows instead, behind a wait for the
// acknowledgement of everything it had published, measured the same on every shape.)
__device__ __forceinline__ int close_unit(const PruneFusedArgs &a, int64_t u, int *s_flag) {
  if (threadIdx.x == 0) *s_flag = atomicAdd(a.gaveup + u, kFinisherDone);
  __syncthreads();
  const int n = *s_flag;
  __syncthreads();
  return n;
}

// ... and after its own rows it compacts the row blocks whose flags are raised (re-reading them
// from memory).  tab: the gather table of the unit.
template <int DT>
__device__ __forceinline__ void serve_gaveup(const PruneFusedArgs &a, int64_t u, const u32x4 *src,
                                             const FlatOut<DT> &dst, const int16_t *tab, u32x4 *tiles) {
  const unsigned char *flags = a.undone + (size_t)u * a.NB;
  for (int blk = 0; blk < a.NB; ++blk) {
    // block-uniform: every thread reads the same byte
    if (__hip_atomic_load(flags + blk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) continue;
    const int64_t s0 = (int64_t)blk * a.RB;
    const int64_t s1c = min(a.S_keep, s0 + a.RB);
    if (s0 < s1c) compact_rows<DT>(src, dst, s0, s1c, a.T, a.ld, tab, tiles);
  }
}

// The row blocks keep their rows (NTW tiles of 32 rows per wave, RB = 128 * NTW rows) on chip
// from the column sums until the index list arrives: the first NTW - NLT tiles of a wave in
// registers, the last NLT in the wave's LDS tiles -- exactly as k_prune_onepass does.
template <int DT, int NTW, int NLT>
__global__ __launch_bounds__(256, (NTW - NLT) * 16 * Elem<DT>::EB <= 32 ? 4 : (NTW - NLT) * 16 * Elem<DT>::EB <= 96 ? 3 : 2)
void k_prune_solo(PruneFusedArgs a) {
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
  const int tid = threadIdx.x, lane = tid % kWave;
  const int wave = tid / kWave;
  if ((int64_t)blockIdx.x < a.U) {
    solo_prologue<DT>(a, blockIdx.x, (double *)tiles);   // the tiles are free in a block without rows
    return;
  }
  const int64_t item = (int64_t)blockIdx.x - a.U;
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

  // the graded start of the launch's first round (see k_prune_onepass)
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

  int st = solo_index_list(a, u, item, s_part, s_sc, s_idx, &s_flag);
  if (st == kGaveUp) {
    if (!hand_over_rows(a, u, item, s_part, s_sc, s_idx, &s_flag)) return;
    st = kHaveList;
  }
  const int n_gaveup = st == kFinisher ? close_unit(a, u, &s_flag) : 0;

  // ---- compaction: the LDS tiles first, then the register tiles through slot 0 ---------------
  // (row numbers are formed again from an opaque copy of the wave index: kept alive from the
  // load phase they would cost registers that this kernel does not have)
  int wave_c = wave;
  asm volatile("" : "+v"(wave_c));
  auto tile_row0_c = [&](int n) { return s0 + (int64_t)(4 * n + wave_c) * TR; };
  auto tile_rows_c = [&](int n, int64_t hi) { return (int)max((int64_t)0, min((int64_t)TR, hi - tile_row0_c(n))); };
  const FlatOut<DT> dst((char *)a.kp + (size_t)u * a.kp_unit_rows * a.ld * E::EB);
  compact_build_tab<DT>(tab, s_idx, a.T, a.ld, dst.sh);
  __syncthreads();
  const int64_t s1c = min(s1, a.S_keep);
#pragma unroll
  for (int n = NRT; n < NTW; ++n) {
    const int nr = tile_rows_c(n, s1c);
    if (nr > 0) compact_emit_tile<DT>(wtile + (size_t)(n - NRT) * Tile<DT>::CHUNKS, dst, tile_row0_c(n), nr, a.ld, tab, lane);
  }
#pragma unroll
  for (int n = 0; n < NRT; ++n) {
    const int nr = tile_rows_c(n, s1c);
    if (nr > 0) {   // wave-uniform
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();       // the slot's previous tile has been read
#pragma unroll
      for (int j = 0; j < NLD; ++j) wtile[Tile<DT>::slot(j * kWave + lane)] = r[n][j];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      compact_emit_tile<DT>(wtile, dst, tile_row0_c(n), nr, a.ld, tab, lane);
    }
  }
  if (n_gaveup > 0) {   // block-uniform
    __syncthreads();   // every wave is done with the tiles, which the re-read uses
    serve_gaveup<DT>(a, u, src, dst, tab, tiles);
  }
}

// ---- host side --------------------------------------------------------------------------------
namespace {
// A 48-bit number, never 0, different for every call of the process and spread over the whole
// range, so that what an earlier call or other data left in a workspace does not look like it.
unsigned long long next_nonce48() {
  static std::atomic<unsigned long long> counter{
      (unsigned long long)std::chrono::steady_clock::now().time_since_epoch().count() * 0x9e3779b97f4a7c15ull};
  unsigned long long z = counter.fetch_add(0x9e3779b97f4a7c15ull, std::memory_order_relaxed);
  z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
  z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
  z = (z ^ (z >> 31)) >> 16;
  return z != 0 ? z : 1;
}
int solo_group_size(int NB) { return NB > 64 ? (NB + kMaxGroups - 1) / kMaxGroups : 0; }
}  // namespace

size_t prune_solo_ws_bytes(int64_t U, int NB) {
  size_t b = (size_t)U * NB * kD * sizeof(double);                                   // partial
  if (solo_group_size(NB) > 0) {
    b += (size_t)U * kMaxGroups * kD * sizeof(double);                               // gpartial
    b += (size_t)U * kMaxGroups * sizeof(unsigned long long);                        // tctr_g
  }
  b += (size_t)U * kD * sizeof(double);                                              // qn
  b += (size_t)U * sizeof(unsigned long long);                                       // tctr
  b += 2 * (size_t)U * sizeof(int);                                                  // arrived, gaveup
  b = (b + 15) & ~(size_t)15;
  b += (size_t)U * kWave * sizeof(uint32_t);                                         // idx_pub
  b += ((size_t)U * NB + 15) & ~(size_t)15;                                          // undone
  return b;
}

hipError_t launch_prune_solo(int dtype, const void *q_obs, const void *k, float *score, int16_t *idx, void *kp,
                             void *ws, int64_t U, int64_t S, int64_t S_keep, int64_t kp_unit_rows, int G,
                             int S_obs, int T, int ld, int NB, int64_t RB, int hold, int spin_limit,
                             hipStream_t st) {
  clear_stale_hip_error();
  PruneFusedArgs a = {};
  const int eb = dtype == THK_BF16 ? 2 : 4;
  a.k = k; a.q_obs = q_obs; a.kp = kp; a.score = score; a.idx = idx;
  a.GS = solo_group_size(NB);
  char *w = (char *)ws;
  a.partial = (double *)w; w += (size_t)U * NB * kD * sizeof(double);
  if (a.GS > 0) {
    a.gpartial = (double *)w;            w += (size_t)U * kMaxGroups * kD * sizeof(double);
    a.tctr_g = (unsigned long long *)w;  w += (size_t)U * kMaxGroups * sizeof(unsigned long long);
  }
  a.qn = (double *)w;                w += (size_t)U * kD * sizeof(double);
  a.tctr = (unsigned long long *)w;  w += (size_t)U * sizeof(unsigned long long);
  a.arrived = (int *)w;              w += (size_t)U * sizeof(int);
  a.gaveup = (int *)w;               w += (size_t)U * sizeof(int);
  w = (char *)(((uintptr_t)w + 15) & ~(uintptr_t)15);
  a.idx_pub = (uint32_t *)w;         w += (size_t)U * kWave * sizeof(uint32_t);
  a.undone = (unsigned char *)w;
  a.nonce = next_nonce48();
  // at most 500 us, in 64-cycle ticks at about 2.4 GHz
  a.prologue_delay = (int32_t)(std::min(std::max(env_switches().prologue_delay_us, 0L), 500L) * 2400 / 64);
  a.S = S; a.S_keep = S_keep; a.kp_unit_rows = kp_unit_rows; a.RB = RB; a.T = T; a.ld = ld; a.G = G;
  a.S_obs = S_obs; a.NB = NB; a.spin_limit = spin_limit;
  a.stagger_blocks = 0; a.stagger_units = 1; a.stagger_ticks = 0;
  a.U = U;
  {
    // the graded start of the first round, as in the three-launch form
    const int64_t resident = (int64_t)kCUs * (dtype == THK_BF16 ? 3 : 2);
    const int64_t total = U * NB;
    const int64_t res_units = resident / NB;
    double ns = -1.0;
    if (env_switches().stagger_set) ns = env_switches().stagger_ns;
    else if (res_units >= 2 && total >= 2 * resident) ns = 0.6 * (double)S * kD * eb * 1.5 / 5.7e3;
    if (ns > 0.0 && res_units >= 2) {
      a.stagger_blocks = (int32_t)(res_units * NB);
      a.stagger_units = (int32_t)res_units;
      a.stagger_ticks = std::max((int32_t)(ns * 2.4 / 64.0), 1);   // 2.4 GHz, s_sleep counts 64-cycle ticks
    }
  }
  const void *fn = nullptr;
  if (dtype == THK_BF16) {
    switch (hold) {
      case 1: fn = (const void *)k_prune_solo<THK_BF16, 1, 1>; break;
      case 2: fn = (const void *)k_prune_solo<THK_BF16, 2, 1>; break;
      case 4: fn = (const void *)k_prune_solo<THK_BF16, 4, 1>; break;
    }
  } else {
    switch (hold) {
      case 1: fn = (const void *)k_prune_solo<THK_F32, 1, 1>; break;
      case 2: fn = (const void *)k_prune_solo<THK_F32, 2, 1>; break;
    }
  }
  if (fn == nullptr || RB != 128 * hold || U * ((int64_t)NB + 1) > 2147483647LL) return hipErrorInvalidValue;
  const size_t lds = 2048 + 4 * compact_tile_bytes(eb);
  static DynLds set[2][5];
  hipError_t e = ensure_dyn_lds(fn, lds, set[dtype == THK_BF16 ? 1 : 0][hold]);
  if (e != hipSuccess) return e;
  void *kargs[] = {(void *)&a};
  e = launch_main_kernel(fn, dim3((unsigned)(U * (NB + 1))), dim3(256), kargs, lds, st);
  return e != hipSuccess ? e : hipGetLastError();
}

}  // namespace thk
