// Decode attention over the pruned key cache plus the unpruned tail
// (Sec. 3.3, Fig. 2; attention formula of Sec. 3.2) -- gfx950, wave64.
//
// Work split.  A 256-thread block serves one (unit, query-head group, S-split):
// GT query heads that read the same KV head share every K and V byte the block
// streams.  Its four wavefronts work independently on 64-row tiles, each with
// its own running softmax state (max, sum, acc[128]); the states are merged
// once at the end through LDS.  With n_split > 1 the block writes its state to
// the workspace and k_decode_merge combines the splits in index order.
//
// One tile, one wavefront.
//   K_pruned rows are T elements long and in general not 16-byte multiples, but
//   a run of whole rows is a flat byte range.  The range, widened to 16-byte
//   boundaries, is fetched with coalesced 16-byte loads and mirrored into LDS;
//   lane r then walks row r out of LDS (row-per-lane, so no cross-lane
//   reduction is needed for the q.K dot products).  V rows are 128 elements:
//   they are fetched straight into registers, 16 bytes per lane, LPR lanes per
//   row, each lane accumulating its VEC output channels over the rows it sees.
//   The tile's probabilities travel from the row-per-lane layout to the
//   lane-group layout through a 64-float LDS line per query head.
#include <math.h>

#include "thk_internal.h"

namespace thk {

constexpr int kTailRows = 16;   // rows per tile in the full-width tail segment
constexpr int kMaxSplitDev = 4096;   // largest n_split the API accepts

__device__ inline void wave_sync_lds() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Cross-lane reductions over the 64 lanes with DPP row shifts and row
// broadcasts: after the four row_shr steps lane 15 of every 16-lane row holds
// the row's result, row_bcast:15 folds rows 0->1 and 2->3, row_bcast:31 folds
// the lower half into rows 2 and 3, and lane 63 holds the total.
template <int CTRL, int ROW_MASK>
__device__ inline float dpp_move(float identity, float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(identity), __float_as_int(x), CTRL,
                                                    ROW_MASK, 0xf, false));
}
__device__ inline float wave_max(float x) {
  const float id = -INFINITY;
  x = fmaxf(x, dpp_move<0x111, 0xf>(id, x));   // row_shr:1
  x = fmaxf(x, dpp_move<0x112, 0xf>(id, x));   // row_shr:2
  x = fmaxf(x, dpp_move<0x114, 0xf>(id, x));   // row_shr:4
  x = fmaxf(x, dpp_move<0x118, 0xf>(id, x));   // row_shr:8
  x = fmaxf(x, dpp_move<0x142, 0xa>(id, x));   // row_bcast:15 into rows 1, 3
  x = fmaxf(x, dpp_move<0x143, 0xc>(id, x));   // row_bcast:31 into rows 2, 3
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}
__device__ inline float wave_sum(float x) {
  x += dpp_move<0x111, 0xf>(0.f, x);
  x += dpp_move<0x112, 0xf>(0.f, x);
  x += dpp_move<0x114, 0xf>(0.f, x);
  x += dpp_move<0x118, 0xf>(0.f, x);
  x += dpp_move<0x142, 0xa>(0.f, x);
  x += dpp_move<0x143, 0xc>(0.f, x);
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

// 16 bytes at byte offset `off` of a tensor of `total` bytes; bytes past the end read as 0.
__device__ inline uint4 load_chunk_guarded(const char *base, size_t off, size_t total) {
  if (off + 16 <= total) return *(const uint4 *)(base + off);
  uint32_t w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    uint32_t x = 0;
    if (off + 4 * i + 2 <= total) x |= (uint32_t) * (const uint16_t *)(base + off + 4 * i);
    if (off + 4 * i + 4 <= total) x |= (uint32_t) * (const uint16_t *)(base + off + 4 * i + 2) << 16;
    w[i] = x;
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// RA bytes of an LDS row at element offset t, widened to floats.
template <int DT, int RA>
__device__ inline void lds_row_read(const char *rowp, int t, float *f) {
  using E = Elem<DT>;
  const char *p = rowp + (size_t)t * E::EB;
  if constexpr (DT == THK_BF16) {
    if constexpr (RA == 16) {
      float g[8]; E::unpack(*(const uint4 *)p, g);
#pragma unroll
      for (int i = 0; i < 8; ++i) f[i] = g[i];
    } else if constexpr (RA == 8) {
      const uint2 r = *(const uint2 *)p;
      f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
      f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
    } else if constexpr (RA == 4) {
      const uint32_t r = *(const uint32_t *)p;
      f[0] = __uint_as_float(r << 16); f[1] = __uint_as_float(r & 0xffff0000u);
    } else {
      f[0] = __uint_as_float((uint32_t) * (const uint16_t *)p << 16);
    }
  } else {
    if constexpr (RA == 16) {
      const float4 r = *(const float4 *)p; f[0] = r.x; f[1] = r.y; f[2] = r.z; f[3] = r.w;
    } else if constexpr (RA == 8) {
      const float2 r = *(const float2 *)p; f[0] = r.x; f[1] = r.y;
    } else {
      f[0] = *(const float *)p;
    }
  }
}

template <int DT, int GT>
struct TileState {
  float m[GT];                       // running max (log2 domain)
  float l[GT];                       // per-lane partial sum of probabilities
  float acc[GT][Elem<DT>::VEC];      // per-lane partial output channels
};

// The K bytes of one tile staged in registers: the flat byte range of its rows,
// widened to 16-byte boundaries, KB chunks per lane at most.
template <int KB>
struct KStage {
  uint4 r[KB];
  int nch;     // 16-byte chunks in the widened range
  int shift;   // bytes between the widened start and the first row
};

// Issue the global loads of a tile of `nrows` rows, W elements wide with row
// stride ld (elements), starting at byte kbeg of tensor kg (ktot bytes).
template <int DT, int KB>
__device__ __forceinline__ void k_issue(KStage<KB> &ks, const char *__restrict__ kg, size_t kbeg,
                                        size_t ktot, int nrows, int W, int ld, int lane) {
  constexpr int EB = Elem<DT>::EB;
  const size_t kend = kbeg + ((size_t)(nrows - 1) * ld + W) * EB;
  const size_t a0 = kbeg & ~(size_t)15;
  ks.shift = (int)(kbeg - a0);
  ks.nch = (int)((kend - a0 + 15) >> 4);
  if (a0 + (size_t)ks.nch * 16 <= ktot) {   // whole range inside the tensor (wave-uniform)
    // chunk indices past the range are clamped to its last chunk: every load stays in bounds and
    // no lane is predicated off; the duplicates land in LDS slots that no row read touches
    const char *p = kg + a0;
    const int last = ks.nch - 1;
#pragma unroll
    for (int j = 0; j < KB; ++j) ks.r[j] = *(const uint4 *)(p + (size_t)min(j * kWave + lane, last) * 16);
  } else {                                   // the last bytes of the tensor: guarded loads
#pragma unroll
    for (int j = 0; j < KB; ++j)
      ks.r[j] = (j * kWave + lane < ks.nch) ? load_chunk_guarded(kg, a0 + ((size_t)j * kWave + lane) * 16, ktot)
                                            : make_uint4(0, 0, 0, 0);
  }
}

template <int KB>
__device__ __forceinline__ void k_commit(const KStage<KB> &ks, char *kbuf, int lane) {
#pragma unroll
  for (int j = 0; j < KB; ++j) ((uint4 *)kbuf)[j * kWave + lane] = ks.r[j];   // kbuf holds KB * 64 chunks
}

template <int DT>
__device__ __forceinline__ void v_issue(uint4 (&vr)[16], const uint4 *__restrict__ vg, int nrows, int b, int lane);

// One tile whose K bytes are already in LDS (kbuf): logits, running softmax,
// acc += p.V.  vg: the tile's value rows (16-byte chunks, 128 elements per row).
template <int DT, int GT, int RA>
__device__ __forceinline__ void tile_compute(int shift, int nrows, int W, int ld,
                                             const float *__restrict__ qs,
                                             const uint4 *__restrict__ vg, uint4 (&vr)[16],
                                             const char *kbuf, float *ps,
                                             TileState<DT, GT> &st, float scale, int lane) {
  using E = Elem<DT>;
  constexpr int VEC = E::VEC, EB = E::EB;
  constexpr int LPR = kD / VEC;              // lanes (= 16-byte chunks) per V row
  constexpr int RPL = kWave / LPR;           // V rows per wave-wide load
  constexpr int VB = 16;                     // V loads per lane per batch
  constexpr int NB = LPR / VB;               // batches per 64-row tile (1 bf16, 2 fp32)
  constexpr int EPR = RA / EB;               // elements per LDS row read
  const int vrow = lane / LPR;

  // ---- logits: lane r owns row r -------------------------------------------
  const int rr = min(lane, nrows - 1);
  const char *rowp = kbuf + shift + (size_t)rr * ld * EB;
  float z[GT];
#pragma unroll
  for (int g = 0; g < GT; ++g) z[g] = 0.f;
  int t = 0;
#pragma unroll 2
  for (; t + EPR <= W; t += EPR) {
    float f[EPR];
    lds_row_read<DT, RA>(rowp, t, f);
#pragma unroll
    for (int g = 0; g < GT; ++g)
#pragma unroll
      for (int e = 0; e < EPR; ++e) z[g] = fmaf(f[e], qs[g * kD + t + e], z[g]);
  }
  for (; t < W; ++t) {
    const float f = E::load1(rowp, t);
#pragma unroll
    for (int g = 0; g < GT; ++g) z[g] = fmaf(f, qs[g * kD + t], z[g]);
  }

  // ---- running softmax (base-2 exponent, scale folded in) ----------------
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    const float zz = lane < nrows ? z[g] * scale : -INFINITY;
    const float m_new = fmaxf(st.m[g], wave_max(zz));   // finite: the tile has >= 1 row
    const float corr = exp2f(st.m[g] - m_new);
    const float p = exp2f(zz - m_new);
    st.l[g] = st.l[g] * corr + p;
    st.m[g] = m_new;
#pragma unroll
    for (int v = 0; v < VEC; ++v) st.acc[g][v] *= corr;
    ps[g * kWave + lane] = p;
  }
  wave_sync_lds();

  // ---- acc += p . V --------------------------------------------------------
#pragma unroll
  for (int b = 0; b < NB; ++b) {
#pragma unroll
    for (int i = 0; i < VB; ++i) {
      const int row = (b * VB + i) * RPL + vrow;
      float f[VEC];
      E::unpack(vr[i], f);
#pragma unroll
      for (int g = 0; g < GT; ++g) {
        const float p = ps[g * kWave + row];
#pragma unroll
        for (int v = 0; v < VEC; ++v) st.acc[g][v] = fmaf(p, f[v], st.acc[g][v]);
      }
    }
    if (b + 1 < NB) v_issue<DT>(vr, vg, nrows, b + 1, lane);
  }
  wave_sync_lds();   // ps and kbuf are rewritten by the next tile
}

// A batch of 16 wave-wide loads of a tile's value rows (batch b) into registers.
// Rows past a ragged tile's end re-read its last row: their probability is 0.
template <int DT>
__device__ __forceinline__ void v_issue(uint4 (&vr)[16], const uint4 *__restrict__ vg, int nrows, int b, int lane) {
  constexpr int LPR = kD / Elem<DT>::VEC, RPL = kWave / LPR;
  if (nrows == kWave) {
#pragma unroll
    for (int i = 0; i < 16; ++i) vr[i] = vg[(size_t)(b * 16 + i) * kWave + lane];
  } else {
    const int vrow = lane / LPR, vcol = lane % LPR;
#pragma unroll
    for (int i = 0; i < 16; ++i) vr[i] = vg[(size_t)min((b * 16 + i) * RPL + vrow, nrows - 1) * LPR + vcol];
  }
}

// KB: 16-byte K chunks a lane may have to stage for one 64-row pruned tile.
// Register budget: 2 waves per SIMD (8 per CU); each wave keeps a V tile and the next
// K tile in flight, so bytes in flight do not depend on more resident waves.
template <int DT, int GT, int RA, int KB>
__global__ __launch_bounds__(256, 2) void k_decode(DecodeArgs a, int groups, int kbuf_bytes) {
  using E = Elem<DT>;
  constexpr int VEC = E::VEC, EB = E::EB, LPR = kD / VEC;
  constexpr int KBT = kTailRows * kD * EB / 16 / kWave;   // chunks per lane of a tail tile
  extern __shared__ uint4 smem[];
  float *qk = (float *)smem;                 // [GT][128] gathered query channels, 0 beyond T
  float *qf = qk + GT * kD;                  // [GT][128] full query
  float *mrg = qf + GT * kD;                 // [4][GT][130] per-wave states for the final merge
  char *wbase = (char *)(mrg + 4 * GT * (kD + 2));
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int wstride = kbuf_bytes + GT * kWave * 4;
  char *kbuf = wbase + (size_t)wave * wstride;
  float *ps = (float *)(kbuf + kbuf_bytes);

  const int sp = (int)(blockIdx.x % a.n_split);
  const int64_t ug = blockIdx.x / a.n_split;
  const int gi = (int)(ug % groups);
  const int64_t u = ug / groups;             // (layer, batch, KV head)
  const int G = a.N_q / a.N_kv;
  const int64_t bn0 = u * G + (int64_t)gi * GT;   // first query head served (heads of unit u: u*G ..)

  const int64_t s0 = min(a.S, (int64_t)sp * a.rows_per_split);
  const int64_t s1 = min(a.S, s0 + a.rows_per_split);
  const int nt_p = (int)((s1 - s0 + 63) >> 6);
  const int nt_t = (sp == a.n_split - 1) ? (a.s_tail + kTailRows - 1) / kTailRows : 0;
  const char *kpg = (const char *)a.kp;

  // the first tile's key and value bytes start moving before anything else happens
  auto tile_k = [&](KStage<KB> &k_, int ti) {
    const int64_t r0 = s0 + (int64_t)ti * 64;
    k_issue<DT, KB>(k_, kpg, ((size_t)u * a.S + r0) * a.ldk * EB, a.kp_bytes,
                    (int)min((int64_t)64, s1 - r0), a.T, a.ldk, lane);
  };
  auto tile_v = [&](uint4 (&v_)[16], int ti) {
    const int64_t r0 = s0 + (int64_t)ti * 64;
    v_issue<DT>(v_, (const uint4 *)a.v + ((size_t)u * a.S + r0) * LPR, (int)min((int64_t)64, s1 - r0), 0, lane);
  };
  KStage<KB> ks;
  uint4 va[16], vb[16];
  if (wave < nt_p) { tile_k(ks, wave); tile_v(va, wave); }

  // query: gather the kept channels (Sec. 3.3: the query is pruned with the stored mask)
  const int16_t *uidx = a.idx + (size_t)u * a.T;
  for (int o = tid; o < GT * kD; o += 256) {
    const int g = o / kD, c = o % kD;
    const size_t qb = (size_t)(bn0 + g) * kD;
    qf[o] = E::load1(a.q, qb + c);
    qk[o] = c < a.T ? E::load1(a.q, qb + uidx[c]) : 0.f;
  }
  __syncthreads();

  TileState<DT, GT> st;
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    st.m[g] = -INFINITY; st.l[g] = 0.f;
#pragma unroll
    for (int v = 0; v < VEC; ++v) st.acc[g][v] = 0.f;
  }

  // ---- pruned segment: the K and V bytes of this wave's next tile are in flight
  // while the current one is computed (two value-register sets, used alternately)
  auto tile_run = [&](uint4 (&v_)[16], int ti, int shift) {
    const int64_t r0 = s0 + (int64_t)ti * 64;
    tile_compute<DT, GT, RA>(shift, (int)min((int64_t)64, s1 - r0), a.T, a.ldk, qk,
                             (const uint4 *)a.v + ((size_t)u * a.S + r0) * LPR, v_, kbuf, ps, st,
                             a.scale_log2, lane);
  };
  for (int ti = wave; ti < nt_p; ti += 8) {
    int shift = ks.shift;
    k_commit<KB>(ks, kbuf, lane);
    if (ti + 4 < nt_p) { tile_k(ks, ti + 4); tile_v(vb, ti + 4); }
    wave_sync_lds();
    tile_run(va, ti, shift);
    if (ti + 4 >= nt_p) break;
    shift = ks.shift;
    k_commit<KB>(ks, kbuf, lane);
    if (ti + 8 < nt_p) { tile_k(ks, ti + 8); tile_v(va, ti + 8); }
    wave_sync_lds();
    tile_run(vb, ti + 4, shift);
  }

  // ---- unpruned tail segment (full-width keys, full query) ------------------
  for (int ti = wave; ti < nt_t; ti += 4) {
    const int j0 = ti * kTailRows;
    const int nrows = min(kTailRows, a.s_tail - j0);
    const size_t row0 = (size_t)u * a.s_tail_cap + j0;
    KStage<KBT> kt;
    k_issue<DT, KBT>(kt, (const char *)a.kt, row0 * kD * EB, (size_t)a.units * a.s_tail_cap * kD * EB,
                     nrows, kD, kD, lane);
    const uint4 *vg = (const uint4 *)a.vt + row0 * LPR;
    v_issue<DT>(va, vg, nrows, 0, lane);
    k_commit<KBT>(kt, kbuf, lane);
    wave_sync_lds();
    tile_compute<DT, GT, 16>(0, nrows, kD, kD, qf, vg, va, kbuf, ps, st, a.scale_log2, lane);
  }

  // ---- wave state -> LDS ---------------------------------------------------
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    const float lt = wave_sum(st.l[g]);
#pragma unroll
    for (int off = LPR; off < kWave; off <<= 1)
#pragma unroll
      for (int v = 0; v < VEC; ++v) st.acc[g][v] += __shfl_xor(st.acc[g][v], off);
    float *rec = mrg + (size_t)(wave * GT + g) * (kD + 2);
    if (lane == 0) { rec[0] = st.m[g]; rec[1] = lt; }
    if (lane < LPR)
#pragma unroll
      for (int v = 0; v < VEC; ++v) rec[2 + lane * VEC + v] = st.acc[g][v];
  }
  __syncthreads();

  // ---- merge the four waves; write the output or this split's state --------
  for (int o = tid; o < GT * kD; o += 256) {
    const int g = o / kD, c = o % kD;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) M = fmaxf(M, mrg[(size_t)(w * GT + g) * (kD + 2)]);
    float Lsum = 0.f, A = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float *rec = mrg + (size_t)(w * GT + g) * (kD + 2);
      const float wgt = rec[0] == -INFINITY ? 0.f : exp2f(rec[0] - M);
      Lsum = fmaf(rec[1], wgt, Lsum);
      A = fmaf(rec[2 + c], wgt, A);
    }
    const size_t bn = (size_t)(bn0 + g);
    if (a.n_split == 1) {
      E::store1(a.out, bn * kD + c, A / Lsum);
    } else {
      float *rec = a.ws + (bn * a.n_split + sp) * (kD + 2);
      rec[2 + c] = A;
      if (c == 0) { rec[0] = M; rec[1] = Lsum; }
    }
  }
}

// Merge of the per-split states: m = max m_i, l = sum l_i 2^(m_i - m),
// acc = sum acc_i 2^(m_i - m), out = acc / l.  One 128-thread block per query
// head, thread c owns channel c.  The (m_i, l_i) pairs are read once per wave
// (lane i takes splits i, i+64, ..), turned into weights kept in LDS, and the
// acc_i[c] loads of eight splits are in flight together.  Splits are combined
// in index order, so the result does not depend on timing.
template <int DT>
__global__ __launch_bounds__(128) void k_decode_merge(const float *__restrict__ ws,
                                                      void *__restrict__ out, int n_split) {
  using E = Elem<DT>;
  __shared__ float wgt[kMaxSplitDev];
  __shared__ float red[2][2];
  const int c = threadIdx.x, lane = c % kWave, wave = c / kWave;
  const size_t bn = blockIdx.x;
  const float *rec0 = ws + bn * n_split * (kD + 2);
  // pass 1: running max over this thread's splits
  float mloc = -INFINITY;
  for (int i = c; i < n_split; i += 128) mloc = fmaxf(mloc, rec0[(size_t)i * (kD + 2)]);
  mloc = wave_max(mloc);
  if (lane == 0) red[0][wave] = mloc;
  __syncthreads();
  const float M = fmaxf(red[0][0], red[0][1]);
  // pass 2: weights into LDS
  for (int i = c; i < n_split; i += 128) {
    const float mi = rec0[(size_t)i * (kD + 2)];
    wgt[i] = mi == -INFINITY ? 0.f : exp2f(mi - M);
  }
  __syncthreads();
  float Lsum = 0.f, A = 0.f;
  int i = 0;
  for (; i + 8 <= n_split; i += 8) {
    float lv[8], av[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float *rec = rec0 + (size_t)(i + j) * (kD + 2);
      lv[j] = rec[1];
      av[j] = rec[2 + c];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      Lsum = fmaf(lv[j], wgt[i + j], Lsum);
      A = fmaf(av[j], wgt[i + j], A);
    }
  }
  for (; i < n_split; ++i) {
    const float *rec = rec0 + (size_t)i * (kD + 2);
    Lsum = fmaf(rec[1], wgt[i], Lsum);
    A = fmaf(rec[2 + c], wgt[i], A);
  }
  E::store1(out, bn * kD + c, A / Lsum);
}

template <int DT, int GT, int KB>
static hipError_t launch_decode_ra(const DecodeArgs &a, int ra, int groups, int kbuf, hipStream_t st) {
  const size_t lds = (size_t)(2 * GT * kD + 4 * GT * (kD + 2)) * 4 + 4 * ((size_t)kbuf + GT * kWave * 4);
  const dim3 grid((unsigned)(a.units * groups * a.n_split)), block(256);
#define THK_LAUNCH(RA)                                                                        \
  do {                                                                                        \
    hipError_t e = hipSuccess;                                                                \
    if (lds > 48 * 1024)                                                                      \
      e = hipFuncSetAttribute((const void *)k_decode<DT, GT, RA, KB>,                         \
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);          \
    if (e != hipSuccess) return e;                                                            \
    hipLaunchKernelGGL((k_decode<DT, GT, RA, KB>), grid, block, lds, st, a, groups, kbuf);    \
  } while (0)
  if (ra == 16) THK_LAUNCH(16);
  else if (ra == 8) THK_LAUNCH(8);
  else if (ra == 4) THK_LAUNCH(4);
  else {
    if constexpr (DT == THK_BF16) THK_LAUNCH(2);
    else return hipErrorInvalidValue;
  }
#undef THK_LAUNCH
  return hipGetLastError();
}

template <int DT, int GT>
static hipError_t launch_decode_gt(const DecodeArgs &a, int groups, hipStream_t st) {
  constexpr int eb = Elem<DT>::EB;
  // row alignment of K_pruned relative to its 16-byte aligned base: every row
  // starts at a multiple of ld * eb bytes
  const size_t rowb = (size_t)a.ldk * eb;
  int ra = 16;
  while (rowb % ra) ra >>= 1;
  // LDS bytes for one 64-row tile widened to 16-byte boundaries, and the
  // chunks per lane that staging it takes
  int kbuf = (int)(64 * rowb + 32);
  const int tailbuf = kTailRows * kD * eb;
  if (kbuf < tailbuf) kbuf = tailbuf;
  kbuf = (kbuf + 15) & ~15;
  const int max_nch = (int)((64 * rowb + (ra == 16 ? 0 : 14) + 15) / 16);
  const int kb = (max_nch + kWave - 1) / kWave;
  constexpr int KB_NARROW = (DT == THK_BF16) ? 10 : 17;   // T <= 79 (bf16) / T <= 67 (fp32)
  constexpr int KB_WIDE = (DT == THK_BF16) ? 17 : 33;     // up to T = ld = 128
  const int kbsel = kb <= KB_NARROW ? KB_NARROW : KB_WIDE;
  if (kbuf < kbsel * kWave * 16) kbuf = kbsel * kWave * 16;   // every staged chunk has an LDS slot
  if (kb <= KB_NARROW) return launch_decode_ra<DT, GT, KB_NARROW>(a, ra, groups, kbuf, st);
  if (kb <= KB_WIDE) return launch_decode_ra<DT, GT, KB_WIDE>(a, ra, groups, kbuf, st);
  return hipErrorInvalidValue;
}

template <int DT>
static hipError_t launch_decode_dt(const DecodeArgs &a, hipStream_t st) {
  const int G = a.N_q / a.N_kv;
  const int gt = (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1;
  const int groups = G / gt;
  hipError_t e;
  if (gt == 4) e = launch_decode_gt<DT, 4>(a, groups, st);
  else if (gt == 2) e = launch_decode_gt<DT, 2>(a, groups, st);
  else e = launch_decode_gt<DT, 1>(a, groups, st);
  if (e != hipSuccess) return e;
  if (a.n_split > 1) {
    const int64_t heads = a.units / a.N_kv * a.N_q;
    hipLaunchKernelGGL((k_decode_merge<DT>), dim3((unsigned)heads), dim3(128), 0, st, a.ws, a.out, a.n_split);
    e = hipGetLastError();
  }
  return e;
}

hipError_t launch_decode(const DecodeArgs &a, hipStream_t st) {
  return a.dtype == THK_BF16 ? launch_decode_dt<THK_BF16>(a, st) : launch_decode_dt<THK_F32>(a, st);
}

}  // namespace thk
