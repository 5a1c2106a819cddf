// Device-side building blocks of the prune path, shared by the stand-alone
// kernels (k_colsum, k_finalize, k_select, k_compact_flat) and the fused one.
#pragma once
#include "thk_internal.h"

namespace thk {

// ---------------------------------------------------------------------------
// Column reduction of rows [s0, s1) of one [S, 128] unit by a 256-thread block:
// sums of squares (P == 2) or of absolute values (P == 1) per channel, written
// as 128 doubles to `out`.  A 16-byte load covers VEC channels, so LPR = 128 /
// VEC lanes cover a row and the block covers RPB rows per step; each thread
// keeps the same VEC channels for all its rows.  Squares of bf16 values are
// exact in fp32; fp32 chains are UNR terms long and are then folded into fp64
// accumulators, which carry every later merge.  red: LDS, 4 x 128 doubles.
// ---------------------------------------------------------------------------
// STREAM: the rows are not read again soon (non-temporal loads); the one-launch prune that
// re-reads its rows for the compaction wants them cached instead.
template <int DT, int P, bool STREAM = true>
__device__ __forceinline__ void colsum_block(const u32x4 *__restrict__ base, int64_t s0, int64_t s1,
                                             double *__restrict__ out, double (*red)[kD]) {
  using E = Elem<DT>;
  constexpr int VEC = E::VEC, LPR = kD / VEC, RPB = 256 / LPR, UNR = 8;
  const int tid = threadIdx.x;
  const int cl = tid % LPR, rg = tid / LPR;
  double dacc[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) dacc[v] = 0.0;

  for (int64_t s = s0 + rg; s < s1; s += (int64_t)RPB * UNR) {
    u32x4 r[UNR];
#pragma unroll
    for (int j = 0; j < UNR; ++j) {
      const int64_t row = s + (int64_t)j * RPB;
      const u32x4 zero = {0u, 0u, 0u, 0u};
      r[j] = row >= s1 ? zero : STREAM ? ld_stream(base + row * LPR + cl) : base[row * LPR + cl];
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
  for (int v = 0; v < VEC; ++v) dacc[v] = add_lane_groups<LPR>(dacc[v]);

  const int wave = tid / kWave, lane = tid % kWave;
  if (lane < LPR)
#pragma unroll
    for (int v = 0; v < VEC; ++v) red[wave][lane * VEC + v] = dacc[v];
  __syncthreads();
  if (tid < kD) out[tid] = ((red[0][tid] + red[1][tid]) + red[2][tid]) + red[3][tid];
}

// ---------------------------------------------------------------------------
// sum over the G query heads of unit u of ||Q_obs,g[:, c]||_2 (Sec. 3.2, with the
// observation window), for c = threadIdx.x < 128 (other threads return 0).
// The unit's heads hold G * S_obs contiguous rows of Q_obs; heads are taken
// kQnHeads at a time, each thread squares (in fp64) the VEC channels it owns
// over the rows of its row group, row groups are folded by shuffles inside a
// wave and through LDS across the waves.  NT threads per block, all of which
// must call; red: LDS [kQnHeads][NT / 64][128] doubles.
// ---------------------------------------------------------------------------
constexpr int kQnHeads = 4;

template <int DT, int NT>
__device__ __forceinline__ double unit_query_norm(const void *__restrict__ q_obs, int64_t u, int G,
                                                  int S_obs, double (*red)[NT / kWave][kD]) {
  using E = Elem<DT>;
  constexpr int VEC = E::VEC, LPR = kD / VEC, RG = NT / LPR, NW = NT / kWave, GC = kQnHeads;
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int cl = tid % LPR, rg = tid / LPR;
  // unit u = (layer*batch, KV head) reads query heads u * G .. u * G + G - 1
  const u32x4 *qbase = (const u32x4 *)((const char *)q_obs + (size_t)u * G * S_obs * kD * E::EB);
  double tot = 0.0;
  for (int g0 = 0; g0 < G; g0 += GC) {
    const int ng = min(GC, G - g0);
    double qa[GC][VEC];
#pragma unroll
    for (int g = 0; g < GC; ++g)
#pragma unroll
      for (int v = 0; v < VEC; ++v) qa[g][v] = 0.0;
    for (int i0 = 0; i0 < S_obs; i0 += RG) {
      u32x4 r[GC];
      const int i = i0 + rg;
      const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int g = 0; g < GC; ++g)
        r[g] = (g < ng && i < S_obs) ? qbase[((size_t)(g0 + g) * S_obs + i) * LPR + cl] : zero;
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
  return tot;
}

// ---------------------------------------------------------------------------
// The same quantity, sum_g ||Q_obs,g[:, c]||_2, computed by ONE wavefront without LDS or
// barriers: the wave loads 64 / LPR window rows per step (eight steps in flight), every lane
// squares its VEC channels in fp64, the row groups are folded by shuffles, and lanes
// 0 .. LPR-1 write the unit's 128 values to qn_u.
// ---------------------------------------------------------------------------
// Sum over the window rows of one head of the squared entries, per channel, in every lane that
// owns the channel (lane % LPR picks VEC consecutive channels).
template <int DT>
__device__ __forceinline__ void wave_head_sumsq(const u32x4 *__restrict__ qhead, int S_obs, int lane,
                                                double (&qa)[Elem<DT>::VEC]) {
  using E = Elem<DT>;
  constexpr int VEC = E::VEC, LPR = kD / VEC, RG = kWave / LPR, UNR = 8;
  const int cl = lane % LPR, rg = lane / LPR;
#pragma unroll
  for (int v = 0; v < VEC; ++v) qa[v] = 0.0;
  for (int i0 = 0; i0 < S_obs; i0 += RG * UNR) {
    u32x4 r[UNR];
#pragma unroll
    for (int j = 0; j < UNR; ++j) {
      const int i = i0 + j * RG + rg;
      const u32x4 zero = {0u, 0u, 0u, 0u};
      r[j] = i < S_obs ? qhead[(size_t)i * LPR + cl] : zero;
    }
#pragma unroll
    for (int j = 0; j < UNR; ++j) {
      float f[VEC];
      E::unpack(r[j], f);
#pragma unroll
      for (int v = 0; v < VEC; ++v) qa[v] += (double)f[v] * (double)f[v];
    }
  }
#pragma unroll
  for (int v = 0; v < VEC; ++v) qa[v] = add_lane_groups<LPR>(qa[v]);
}

template <int DT>
__device__ __forceinline__ void wave_query_norm(const void *__restrict__ q_obs, int64_t u, int G, int S_obs,
                                                double *__restrict__ qn_u, int lane) {
  using E = Elem<DT>;
  constexpr int VEC = E::VEC, LPR = kD / VEC;
  const int cl = lane % LPR, rg = lane / LPR;
  const u32x4 *qbase = (const u32x4 *)((const char *)q_obs + (size_t)u * G * S_obs * kD * E::EB);
  double tot[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) tot[v] = 0.0;
  for (int g = 0; g < G; ++g) {
    double qa[VEC];
    wave_head_sumsq<DT>(qbase + (size_t)g * S_obs * LPR, S_obs, lane, qa);
#pragma unroll
    for (int v = 0; v < VEC; ++v) tot[v] += sqrt(qa[v]);
  }
  if (rg == 0)
#pragma unroll
    for (int v = 0; v < VEC; ++v) qn_u[cl * VEC + v] = tot[v];
}

// The same for a unit with several query heads, by a block of NW wavefronts: NW heads at a time,
// one per wave, their norms handed to wave 0 through LDS and added there in head order (the
// result equals wave_query_norm's bit for bit).  hn: NW * 128 doubles of LDS.
template <int DT, int NW>
__device__ __forceinline__ void block_query_norm(const void *__restrict__ q_obs, int64_t u, int G, int S_obs,
                                                 double *__restrict__ qn_u, double *hn) {
  using E = Elem<DT>;
  constexpr int VEC = E::VEC, LPR = kD / VEC;
  const int lane = threadIdx.x % kWave, w = threadIdx.x / kWave;
  const int cl = lane % LPR, rg = lane / LPR;
  const u32x4 *qbase = (const u32x4 *)((const char *)q_obs + (size_t)u * G * S_obs * kD * E::EB);
  double tot[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) tot[v] = 0.0;
  for (int g0 = 0; g0 < G; g0 += NW) {
    if (g0 + w < G) {
      double qa[VEC];
      wave_head_sumsq<DT>(qbase + (size_t)(g0 + w) * S_obs * LPR, S_obs, lane, qa);
      if (rg == 0)
#pragma unroll
        for (int v = 0; v < VEC; ++v) hn[w * kD + cl * VEC + v] = sqrt(qa[v]);
    }
    __syncthreads();
    if (w == 0 && rg == 0)
      for (int j = 0; j < NW && g0 + j < G; ++j)
#pragma unroll
        for (int v = 0; v < VEC; ++v) tot[v] += hn[j * kD + cl * VEC + v];
    __syncthreads();
  }
  if (w == 0 && rg == 0)
#pragma unroll
    for (int v = 0; v < VEC; ++v) qn_u[cl * VEC + v] = tot[v];
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

__device__ inline void select_wave(float s_lo, float s_hi, int T, int16_t *out, int lane) {
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

// ---------------------------------------------------------------------------
// The same selection inside a 256-thread block whose other blocks wait for the list: one
// wavefront, no LDS traffic and no barrier inside the search.  The T-th largest key is found by
// bisection on its 32 bits (count of keys >= candidate = two ballots and two population counts,
// all in scalar registers); channels with a larger key are kept, and of those that tie with it
// the lowest-numbered ones, as many as are still missing -- channel c is kept iff fewer than T
// channels rank before it (larger score, or equal score and lower index).  The kept channels are
// emitted in ascending order through ballot + prefix popcount.  1.5 us inside the prune kernels
// when all 32 rounds run (the wave gets about every third issue slot of its SIMD there).
// (Its predecessor counted, per channel, the channels ranking before it, 64 LDS broadcast reads
// per thread and three barriers: a few hundred cycles alone, but 2.0-2.9 us (median 2.4) inside
// the prune kernels, where the neighbouring blocks' compaction keeps the LDS pipeline busy.)
// sc: 128 scores in LDS (complete and visible); out: LDS, T entries, visible to the block on
// return.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void select_block(const float *sc, int T, int16_t *out) {
  using u64 = unsigned long long;
  if (threadIdx.x < kWave) {
    const int lane = threadIdx.x;
    auto key_of = [](float s) {
      const uint32_t b = __float_as_uint(s);
      return (b & 0x80000000u) ? ~b : (b | 0x80000000u);   // unsigned order == float order
    };
    const uint32_t k0 = key_of(sc[lane]), k1 = key_of(sc[lane + kWave]);
    // thr ends as the largest v with count(key >= v) >= T: the T-th largest key.  The search stops
    // as soon as a candidate has EXACTLY T keys at or above it: those are the list (every one of
    // them is larger than every other key, so no tie crosses the boundary).  With 128 scores
    // spread over a few binades that happens after some ten rounds; only a tie across the T-th
    // place runs all 32 and is then resolved by channel number.
    uint32_t thr = 0;
    bool exact = false;
    for (int bit = 31; bit >= 0; --bit) {
      const uint32_t cand = thr | (1u << bit);
      const int n = __popcll(__ballot(k0 >= cand)) + __popcll(__ballot(k1 >= cand));
      if (n >= T) thr = cand;   // wave-uniform
      if (n == T) { exact = true; break; }
    }
    const u64 below = (1ull << lane) - 1ull;
    bool keep0 = k0 >= thr, keep1 = k1 >= thr;
    if (!exact) {
      const u64 e0 = __ballot(k0 == thr), e1 = __ballot(k1 == thr);
      const int need = T - __popcll(__ballot(k0 > thr)) - __popcll(__ballot(k1 > thr));   // ties to keep, >= 1
      keep0 = k0 > thr || (k0 == thr && __popcll(e0 & below) < need);
      keep1 = k1 > thr || (k1 == thr && __popcll(e0) + __popcll(e1 & below) < need);
    }
    const u64 m0 = __ballot(keep0), m1 = __ballot(keep1);
    if (keep0) out[__popcll(m0 & below)] = (int16_t)lane;
    if (keep1) out[__popcll(m0) + __popcll(m1 & below)] = (int16_t)(lane + kWave);
  }
  __syncthreads();
}

// ---------------------------------------------------------------------------
// Compaction of rows [s0, s1) of one unit whose K_pruned rows are dense (row pitch T), by a
// 256-thread block.  Each wavefront works alone on tiles of 32 rows:
//   1. 16-byte coalesced loads of the full-width rows into its LDS tile;
//   2. for every 16-byte chunk of the OUTPUT, a table lookup gives the LDS element offsets of
//      its VEC source elements (the pattern of row * pitch + idx[t] repeats every 8 output rows
//      because 8 * T elements is a whole number of chunks), the elements are gathered from LDS,
//      packed and stored with one 16-byte store.
// The unit's first output element may sit anywhere: chunks are aligned in MEMORY.  With
// sh = elements between the 16-byte boundary below the unit's start and that start, position
// q = e + sh counts from the boundary, chunk k holds positions [VEC k, VEC k + VEC), and the
// table is built with the shift inside (entry i belongs to element i - sh of an 8-row block;
// the first sh entries point into the block before, with negative offsets).  A tile's rows end
// where they end: the chunks it does not own completely (at most one at each end, shared with
// the neighbouring tile or lying partly outside the unit) are written element by element.
// Rows with padding behind them (pitch ld > T elements) are rows of ld elements whose last
// ld - T come from nowhere: the table points them at the padding chunk of the LDS row, which is
// cleared once, so they are written as zeros along with the rest (leaving them out would make
// the end of every row a partial write, which costs more than the bytes).
// s0 must be a multiple of 32.  tab: LDS, 8 * ld int16 (<= 2 KiB); tiles: LDS, 4 tiles.
// ---------------------------------------------------------------------------
constexpr int kCompactTileRows = 32;

// A tile in LDS: 32 full-width rows, one 16-byte chunk of padding after each, so that
// consecutive rows start four banks apart (rows 256 or 512 bytes apart would all start in the
// same bank, and the gather below reads the same channels of up to eight rows in one step).
template <int DT>
struct Tile {
  static constexpr int CPR = kD / Elem<DT>::VEC;          // 16-byte chunks per row
  static constexpr int PITCH = CPR + 1;                   // chunks from row to row in LDS
  static constexpr int CHUNKS = kCompactTileRows * PITCH; // chunks per tile
  static constexpr int ROW_ELEMS = PITCH * Elem<DT>::VEC; // elements from row to row in LDS
  // LDS chunk of the tile's id-th 16-byte chunk in memory order
  __device__ static inline int slot(int id) { return (id / CPR) * PITCH + id % CPR; }
};
constexpr size_t compact_tile_bytes(int eb) { return (size_t)kCompactTileRows * (kD * eb + 16); }

// Where a unit's dense output starts: the 16-byte boundary at or below it and the distance in
// elements.
template <int DT>
struct FlatOut {
  u32x4 *o;
  int sh;
  __device__ explicit FlatOut(void *unit_start) {
    const int back = (int)((uintptr_t)unit_start & 15);
    sh = back / Elem<DT>::EB;
    o = (u32x4 *)((char *)unit_start - back);   // pointer arithmetic, so that it stays a global pointer
  }
};

template <int DT>
__device__ __forceinline__ void compact_build_tab(int16_t *tab, const int16_t *uidx, int T, int ld, int sh) {
  const int period = 8 * ld;
  for (int i = threadIdx.x; i < period; i += 256) {
    int e = i - sh, back = 0;
    if (e < 0) { e += period; back = 8 * Tile<DT>::ROW_ELEMS; }   // an element of the 8-row block before
    const int row = e / ld, t = e - row * ld;
    // BYTE offsets (at most 8 rows of 272 or 528 bytes: they fit 16 bits), so that a gather address
    // is base + entry with no shift in between; kD: the zero chunk
    tab[i] = (int16_t)((row * Tile<DT>::ROW_ELEMS + (t < T ? (int)uidx[t] : kD) - back) * (int)sizeof(typename Elem<DT>::Bits));
  }
}

// VEC elements of the LDS row (or block of rows) at tl through the VEC table entries (signed byte
// offsets) at te.
template <int DT>
__device__ __forceinline__ u32x4 gather_chunk(const typename Elem<DT>::Bits *tl, const int16_t *te) {
  using ET = typename Elem<DT>::Bits;
  const char *b = (const char *)tl;
  auto at = [&](int off) { return *(const ET *)(b + off); };
  u32x4 w;
  if constexpr (DT == THK_BF16) {
    const u32x4 offs = *(const u32x4 *)te;   // 8 entries
    const int o0 = (int16_t)(offs.x & 0xffffu), o1 = (int)offs.x >> 16, o2 = (int16_t)(offs.y & 0xffffu);
    const int o3 = (int)offs.y >> 16, o4 = (int16_t)(offs.z & 0xffffu), o5 = (int)offs.z >> 16;
    const int o6 = (int16_t)(offs.w & 0xffffu), o7 = (int)offs.w >> 16;
    w.x = (uint32_t)at(o0) | ((uint32_t)at(o1) << 16);
    w.y = (uint32_t)at(o2) | ((uint32_t)at(o3) << 16);
    w.z = (uint32_t)at(o4) | ((uint32_t)at(o5) << 16);
    w.w = (uint32_t)at(o6) | ((uint32_t)at(o7) << 16);
  } else {
    const uint2 offs = *(const uint2 *)te;   // 4 entries
    w.x = at((int16_t)(offs.x & 0xffffu)); w.y = at((int)offs.x >> 16);
    w.z = at((int16_t)(offs.y & 0xffffu)); w.w = at((int)offs.y >> 16);
  }
  return w;
}

// Step 2 for one tile that is already in LDS: rows r0 .. r0 + nr of the unit (r0 a multiple of
// 32), ld elements each in the output.
template <int DT>
__device__ __forceinline__ void compact_emit_tile(const u32x4 *tile, const FlatOut<DT> &out, int64_t r0, int nr,
                                                  int ld, const int16_t *tab, int lane) {
  using E = Elem<DT>;
  using ET = typename E::Bits;
  constexpr int VEC = E::VEC;
  const ET *tl0 = (const ET *)tile;
  const int period = 8 * ld;
  const int64_t base = r0 * ld;                      // first element of the tile; a multiple of VEC
  const int nq = nr * ld;                            // positions base + sh .. base + sh + nq of the unit
  // tile-relative positions p = q - base in [sh, sh + nq); chunks [VEC c, VEC c + VEC)
  const int c_lo = (out.sh + VEC - 1) / VEC, c_hi = (out.sh + nq) / VEC;   // whole chunks: c_lo <= c < c_hi
  u32x4 *o = out.o + base / VEC;
  {
    // chunk c lies in 8-row block pb = c / cpp of the tile, at chunk rc = c % cpp of the table's
    // period.  A tile spans four periods (and the shift), so the first quotient is four
    // comparisons, and from one step to the next (c += 64) quotient and remainder move by
    // constants: no division in the loop, which runs in every block between the arrival of
    // the index list and the block's last store.
    const int cpp = period / VEC;
    const int dq = kWave / cpp, dr = kWave - dq * cpp;   // uniform
    int c = c_lo + lane;
    int pb = (c >= cpp) + (c >= 2 * cpp) + (c >= 3 * cpp) + (c >= 4 * cpp);
    int rc = c - pb * cpp;
    for (; c < c_hi; c += kWave) {
      st_stream(o + c, gather_chunk<DT>(tl0 + pb * 8 * Tile<DT>::ROW_ELEMS, tab + rc * VEC));
      rc += dr;
      pb += dq;
      if (rc >= cpp) { rc -= cpp; ++pb; }
    }
  }
  // positions outside the whole chunks: [sh, min(VEC c_lo, sh + nq)) and [max(VEC c_hi, VEC c_lo), sh + nq)
  const int head_end = min(c_lo * VEC, out.sh + nq);
  const int n_head = head_end - out.sh;
  const int tail_beg = max(c_hi * VEC, head_end);
  const int n_tail = out.sh + nq - tail_beg;
  if (lane < n_head + n_tail) {                       // at most 2 (VEC - 1) lanes
    const int p = lane < n_head ? out.sh + lane : tail_beg + (lane - n_head);
    const int pb = p / period;
    const int pe = p - pb * period;
    ((ET *)o)[p] = *(const ET *)((const char *)(tl0 + pb * 8 * Tile<DT>::ROW_ELEMS) + tab[pe]);
  }
}

// The padding chunk of every LDS row of a wave's tile, cleared (the source of the zeros above).
template <int DT>
__device__ __forceinline__ void tile_clear_padding(u32x4 *tile, int lane) {
  if (lane < kCompactTileRows) tile[lane * Tile<DT>::PITCH + Tile<DT>::CPR] = u32x4{0u, 0u, 0u, 0u};
}

template <int DT>
__device__ __forceinline__ void compact_rows(const u32x4 *__restrict__ src, const FlatOut<DT> &out,
                                             int64_t s0, int64_t s1, int T, int ld, const int16_t *tab,
                                             u32x4 *tiles) {
  using E = Elem<DT>;
  constexpr int VEC = E::VEC, CPR = kD / VEC, TR = kCompactTileRows;
  constexpr int NLD = TR * CPR / kWave;   // 16-byte loads per lane per tile
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  u32x4 *tile = tiles + wave * Tile<DT>::CHUNKS;
  if (ld != T) tile_clear_padding<DT>(tile, lane);
  for (int64_t r0 = s0 + (int64_t)wave * TR; r0 < s1; r0 += 4 * TR) {
    const int nr = (int)min((int64_t)TR, s1 - r0);
    // rows past the end of a ragged last tile re-read its last row (kept in bounds, never gathered)
    u32x4 r[NLD];
    const u32x4 *tsrc = src + (size_t)r0 * CPR;
    const int cmax = nr * CPR - 1;
#pragma unroll
    for (int j = 0; j < NLD; ++j) r[j] = ld_stream(tsrc + min(j * kWave + lane, cmax));
#pragma unroll
    for (int j = 0; j < NLD; ++j) tile[Tile<DT>::slot(j * kWave + lane)] = r[j];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    compact_emit_tile<DT>(tile, out, r0, nr, ld, tab, lane);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
}

}  // namespace thk
