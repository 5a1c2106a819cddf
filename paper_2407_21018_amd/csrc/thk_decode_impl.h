// Decode attention over the pruned key cache plus the unpruned tail
// (Sec. 3.3, Fig. 2; attention formula of Sec. 3.2) -- gfx950, wave64.
// Template body shared by the per-(dtype, group width) translation units.
//
// Work split.  A 256-thread block serves one (unit, query-head group, S-split):
// GT query heads that read the same KV head share every K and V byte the block
// streams.  Its four wavefronts work independently on tiles of TR rows, each
// with its own running softmax state (max, sum, acc[128]); the states are merged
// once at the end through LDS.  With n_split > 1 the block writes its state to
// the workspace and k_decode_merge combines the splits in index order.
//
// One tile, one wavefront.
//   K_pruned rows are T elements long and in general not 16-byte multiples, but
//   a run of whole rows is a flat byte range.  The range, widened to 16-byte
//   boundaries, is fetched with coalesced 16-byte loads into registers (the
//   next tile's range is in flight while the current tile is computed) and
//   mirrored into the wave's LDS slab.  LPK = 64 / TR lanes then walk one row
//   out of LDS, each taking a contiguous share of its channels, so the q.K dot
//   product needs at most one neighbour exchange.  V rows are 128 elements:
//   they go straight into registers, 16 bytes per lane, each lane accumulating
//   its VEC output channels over the rows it sees.  The tile's probabilities
//   travel from the row layout to the V layout through a TR-float LDS line per
//   query head.
#pragma once
#include <math.h>

#include "thk_internal.h"

namespace thk {

constexpr int kTailRows = 16;   // rows per tile in the full-width tail segment
constexpr int kQS = kD + 8;     // floats per query vector in LDS: 128 channels + 8 zeros

__device__ inline void wave_sync_lds() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Cross-lane reductions over the 64 lanes with DPP row shifts and row
// broadcasts: after the four row_shr steps lane 15 of every 16-lane row holds
// the row's result, row_bcast:15 folds rows 0->1 and 2->3, row_bcast:31 folds
// the lower half into rows 2 and 3, and lane 63 holds the total.  A lane whose
// DPP source does not exist receives `old`; passing the lane's own value as
// `old` makes the step a no-op there (max(x, x); x + 0 needs the identity 0)
// and lets the compiler fold the move into the arithmetic instruction.
template <int CTRL, int ROW_MASK>
__device__ inline float dpp_move(float old, float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(x), CTRL,
                                                    ROW_MASK, 0xf, false));
}
// Wave-wide maximum with the DPP step folded into v_max_f32 (one instruction per
// step, written out because the compiler keeps a separate v_mov_dpp).  In-place
// form: a lane whose DPP source does not exist, or whose row is masked off, is
// not written and keeps its value.  The s_nop covers the two wait states a DPP
// read needs after the VALU write of the same register.
#define THK_DPP_MAX(x, ctrl) \
  asm volatile("s_nop 1\n\tv_max_f32_dpp %0, %0, %0 " ctrl : "+v"(x))
__device__ inline float wave_max(float x) {
  THK_DPP_MAX(x, "row_shr:1 row_mask:0xf bank_mask:0xf");
  THK_DPP_MAX(x, "row_shr:2 row_mask:0xf bank_mask:0xf");
  THK_DPP_MAX(x, "row_shr:4 row_mask:0xf bank_mask:0xf");
  THK_DPP_MAX(x, "row_shr:8 row_mask:0xf bank_mask:0xf");
  THK_DPP_MAX(x, "row_bcast:15 row_mask:0xa bank_mask:0xf");
  THK_DPP_MAX(x, "row_bcast:31 row_mask:0xc bank_mask:0xf");
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}
__device__ inline float max_nn(float a, float b) { return a > b ? a : b; }   // inputs are never NaN
__device__ inline float wave_sum(float x) {
  x += dpp_move<0x111, 0xf>(0.f, x);
  x += dpp_move<0x112, 0xf>(0.f, x);
  x += dpp_move<0x114, 0xf>(0.f, x);
  x += dpp_move<0x118, 0xf>(0.f, x);
  x += dpp_move<0x142, 0xa>(0.f, x);
  x += dpp_move<0x143, 0xc>(0.f, x);
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}
// value of the neighbouring lane (lane ^ 1): quad_perm [1,0,3,2]
__device__ inline float lane_swap1(float x) { return dpp_move<0xB1, 0xf>(0.f, x); }
__device__ inline double lane_swap1(double x) {
  const long long b = __double_as_longlong(x);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xffffffffll), 0xB1, 0xf, 0xf, false);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), 0xB1, 0xf, 0xf, false);
  return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
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

// DW consecutive 32-bit words from LDS (address aligned to DW * 4 bytes).
template <int DW>
__device__ inline void lds_words(const char *p, uint32_t (&w)[DW]) {
  if constexpr (DW == 4) {
    const u32x4 r = *(const u32x4 *)p; w[0] = r.x; w[1] = r.y; w[2] = r.z; w[3] = r.w;
  } else if constexpr (DW == 2) {
    const uint2 r = *(const uint2 *)p; w[0] = r.x; w[1] = r.y;
  } else {
    w[0] = *(const uint32_t *)p;
  }
}

// a.lo * b.lo + a.hi * b.hi + c with a, b pairs of bf16 (v_dot2c_f32_bf16)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ inline float dot2_bf16(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}

template <int DT> struct LogitType { using type = float; };
template <> struct LogitType<THK_F32> { using type = double; };
__device__ inline float fma_z(float a, float b, float c) { return fmaf(a, b, c); }
__device__ inline double fma_z(double a, double b, double c) { return fma(a, b, c); }

template <int DT, int GT>
struct TileState {
  float m[GT];                       // running max (log2 domain)
  float l[GT];                       // per-lane partial sum of probabilities
  float acc[GT][Elem<DT>::VEC];      // per-lane partial output channels
  float accp[GT][4];                 // channel-pruned values only: partial sums of 4 kept channels
};

// A lane's view of a tile of channel-pruned value rows staged in its wave's LDS slab: rows are
// ld elements apart, groups of 4 kept channels go to lanes (col), and rpw rows are handled per
// step (rsub = this lane's row within a step).
constexpr int kPsPad = 32;   // zero rows behind a wave's probabilities (channel-pruned values only)

struct VPruned {
  char *vbuf;
  int shift;        // bytes from the slab start to the tile's first row
  int ld;
  int rpw, rsub, col;
  bool active;
};

// Issue the global loads of a tile of `nrows` rows, W elements wide with row
// stride ld (elements), starting at byte kbeg of tensor kg.  The range is
// widened to 16-byte boundaries, so up to 15 bytes before the first row and
// after the last row are read as well: before is always inside the tensor (its
// base is 16-byte aligned); after can pass the tensor's last element by less
// than 16 bytes, inside the 16-byte granule that holds it (the API requires
// that granule to be readable).  Chunk indices past the range are clamped to
// its last chunk: no lane is predicated off, and the duplicates land in LDS
// slots that no row read touches.
// kr receives KB chunks per lane (the tile's K bytes staged in registers);
// returns the byte distance between the widened start and the first row.
template <int DT, int KB>
__device__ __forceinline__ int k_issue(u32x4 (&kr)[KB], const char *__restrict__ kg, size_t kbeg,
                                       int nrows, int W, int ld, int lane) {
  constexpr int EB = Elem<DT>::EB;
  const size_t kend = kbeg + ((size_t)(nrows - 1) * ld + W) * EB;
  const size_t a0 = kbeg & ~(size_t)15;
  const int last = (int)((kend - a0 + 15) >> 4) - 1;
  const char *p = kg + a0;
#pragma unroll
  for (int j = 0; j < KB; ++j) kr[j] = ld_stream((const u32x4 *)(p + (size_t)min(j * kWave + lane, last) * 16));
  return (int)(kbeg - a0);
}

template <int KB>
__device__ __forceinline__ void k_commit(const u32x4 (&kr)[KB], char *kbuf, int lane) {
#pragma unroll
  for (int j = 0; j < KB; ++j) ((u32x4 *)kbuf)[j * kWave + lane] = kr[j];   // kbuf holds KB * 64 chunks
}

// Shape of the value loads of one TR-row tile: NV wave-wide loads per batch.
template <int DT, int TR>
struct VShape {
  static constexpr int LPR = kD / Elem<DT>::VEC;     // lanes (16-byte chunks) per V row
  static constexpr int RPL = kWave / LPR;            // V rows per wave-wide load
  static constexpr int NL = TR / RPL;                // loads per lane per tile
  static constexpr int NV = NL < 16 ? NL : 16;       // loads per lane per batch
  static constexpr int NB = NL / NV;                 // batches per tile
};

// Batch b of a tile's value rows into registers.  Rows past a ragged tile's end
// re-read its last row: their probability is 0.
template <int DT, int TR, int NV>
__device__ __forceinline__ void v_issue(u32x4 (&vr)[NV], const u32x4 *__restrict__ vg,
                                        int nrows, int b, int lane) {
  using VS = VShape<DT, TR>;
  if (nrows == TR) {
#pragma unroll
    for (int i = 0; i < VS::NV; ++i) vr[i] = ld_stream(vg + (size_t)(b * VS::NV + i) * kWave + lane);
  } else {
    const int vrow = lane / VS::LPR, vcol = lane % VS::LPR;
#pragma unroll
    for (int i = 0; i < VS::NV; ++i)
      vr[i] = ld_stream(vg + (size_t)min((b * VS::NV + i) * VS::RPL + vrow, nrows - 1) * VS::LPR + vcol);
  }
}

// One tile whose K bytes are already in LDS (kbuf): logits, running softmax,
// acc += p.V.  vg: the tile's value rows (16-byte chunks, 128 elements per row).
// qs: [GT][kQS] floats, entries 128..135 of every vector are zero; qp: the same
// vectors as packed bf16 pairs, [GT][kQS / 2] words (bf16 inputs only).
// PV = 0: value rows are full width (vg, vr).  PV = 1: value rows are channel-pruned; their
// bytes are in vrp (KBV staged chunks per lane) and are walked out of LDS as described by vp.
// PV = 2: a full-width tile (the tail) of a kernel that also carries pruned-value sums, which
// follow every change of the running maximum.
// Precision of a logit.  bf16 inputs: products are exact in fp32 and the sum runs in fp32.  fp32
// inputs: the dot product and the scaling run in fp64 and the running maximum is subtracted
// before the result is rounded to fp32, so the error of exp2(z - m) does not grow with |z| (an
// fp32 logit of a few thousand -- channel scales of sigma = 2 on query and keys -- is only
// accurate to 1e-4 in absolute terms, which is the whole error budget of fp32 outputs).
template <int DT, int GT, int RA, int TR, int NV, int PV = 0, int KBV = 1>
__device__ __forceinline__ void tile_compute(int shift, int nrows, int W, int ld,
                                             const float *__restrict__ qs,
                                             const uint32_t *__restrict__ qp,
                                             const u32x4 *__restrict__ vg,
                                             u32x4 (&vr)[NV], const char *kbuf,
                                             float *ps, TileState<DT, GT> &st, double scale_d, int lane,
                                             const u32x4 (*vrp)[KBV] = nullptr, const VPruned *vp = nullptr) {
  using E = Elem<DT>;
  using ZT = typename LogitType<DT>::type;   // accumulator of a logit: float (bf16 inputs), double (fp32 inputs)
  const ZT scale = (ZT)scale_d;
  using VS = VShape<DT, TR>;
  constexpr int VEC = E::VEC, EB = E::EB;
  constexpr int LPK = kWave / TR;            // lanes that share one K row (1 or 2)
  constexpr int EPR = RA / EB;               // elements per LDS row read (one granule)
  const int vrow = lane / VS::LPR;
  const int r = lane / LPK, h = lane % LPK;

  // ---- logits: LPK lanes per row, contiguous granule ranges ----------------
  const int rr = min(r, nrows - 1);
  const char *rowp = kbuf + shift + (size_t)rr * ld * EB;
  const int n_gran = W / EPR;
  const int gran0 = (n_gran + LPK - 1) / LPK;              // granules of lane share 0 = trip count
  const int my_first = h * gran0;
  const int my_cnt = (LPK == 1 || h == 0) ? gran0 : n_gran - gran0;
  ZT z[GT];
#pragma unroll
  for (int g = 0; g < GT; ++g) z[g] = (ZT)0;
  if constexpr (DT == THK_BF16 && RA >= 4) {
    // bf16 pairs straight from LDS into v_dot2c_f32_bf16: products are exact, sums in fp32.
    // Keys and packed query share their byte offsets (two bytes per channel), so one offset
    // walks both; the steps that every lane has run without a test, and where share 0 has one
    // granule more, the lanes of share 1 take granule 0 against the zero slot of q in that step.
    constexpr int DW = RA / 4;   // words per granule
    const int common = LPK == 1 ? gran0 : n_gran - gran0;
    const char *kw_p = rowp + my_first * RA;
    const char *qw_p = (const char *)qp + my_first * RA;
    constexpr int UNR = (GT == 4 && DW == 2) ? 1 : 2;   // the one shape that ran out of registers at 2
#pragma unroll UNR
    for (int i = 0; i < common; ++i) {
      uint32_t kw[DW];
      lds_words<DW>(kw_p + i * RA, kw);
#pragma unroll
      for (int g = 0; g < GT; ++g) {
        uint32_t qw[DW];
        lds_words<DW>(qw_p + g * (kQS * 2) + i * RA, qw);
#pragma unroll
        for (int d = 0; d < DW; ++d) z[g] = dot2_bf16(kw[d], qw[d], z[g]);
      }
    }
    if (LPK == 2 && common < gran0) {
      uint32_t kw[DW];
      lds_words<DW>(rowp + (h == 0 ? common * RA : 0), kw);
      const char *qz = (const char *)qp + (h == 0 ? common * RA : kD * 2);
#pragma unroll
      for (int g = 0; g < GT; ++g) {
        uint32_t qw[DW];
        lds_words<DW>(qz + g * (kQS * 2), qw);
#pragma unroll
        for (int d = 0; d < DW; ++d) z[g] = dot2_bf16(kw[d], qw[d], z[g]);
      }
    }
  } else {
#pragma unroll 2
    for (int i = 0; i < gran0; ++i) {
      // a lane whose share is exhausted re-reads granule 0 against the zero slot of q
      const bool valid = (LPK == 1) || i < my_cnt;
      const int tk = valid ? (my_first + i) * EPR : 0;
      const int tq = valid ? tk : kD;
      float f[EPR];
      lds_row_read<DT, RA>(rowp, tk, f);
#pragma unroll
      for (int g = 0; g < GT; ++g)
#pragma unroll
        for (int e = 0; e < EPR; ++e) z[g] = fma_z((ZT)f[e], (ZT)qs[g * kQS + tq + e], z[g]);
    }
  }
  for (int t = n_gran * EPR; t < W; ++t) {   // elements past the last whole granule: share 0
    const float f = E::load1(rowp, t);
    const int tq = (LPK == 1 || h == 0) ? t : kD;
#pragma unroll
    for (int g = 0; g < GT; ++g) z[g] = fma_z((ZT)f, (ZT)qs[g * kQS + tq], z[g]);
  }
  if constexpr (LPK == 2) {
#pragma unroll
    for (int g = 0; g < GT; ++g) z[g] += lane_swap1(z[g]);
  }

  // ---- running softmax (base-2 exponent, scale folded in) ----------------
  // every row is held by LPK lanes, so l counts each probability LPK times
  float pr[GT];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    const ZT zs = z[g] * scale;
    const float zz = r < nrows ? (float)zs : -INFINITY;
    const float m_new = max_nn(st.m[g], wave_max(zz));   // finite: the tile has >= 1 row
    if (m_new != st.m[g]) {                             // wave-uniform; rare after the first tiles
      const float corr = __builtin_amdgcn_exp2f(st.m[g] - m_new);
      st.l[g] *= corr;
#pragma unroll
      for (int v = 0; v < VEC; ++v) st.acc[g][v] *= corr;
      if constexpr (PV != 0) {
#pragma unroll
        for (int e = 0; e < 4; ++e) st.accp[g][e] *= corr;
      }
      st.m[g] = m_new;
    }
    // fp32 inputs: z - m in fp64, then one rounding (m_new is the maximum of the ROUNDED logits, so
    // the difference may exceed 0 by half an fp32 ulp of a logit: a factor 1 + 1e-4 at most)
    if constexpr (DT == THK_F32)
      pr[g] = r < nrows ? __builtin_amdgcn_exp2f((float)(zs - (ZT)m_new)) : 0.f;
    else
      pr[g] = __builtin_amdgcn_exp2f(zz - m_new);
    st.l[g] += pr[g];
  }
  // probabilities to LDS as [row][GT]
  if constexpr (GT == 4) {
    *(float4 *)(ps + r * 4) = make_float4(pr[0], pr[1], pr[2], pr[3]);
  } else if constexpr (GT == 2) {
    *(float2 *)(ps + r * 2) = make_float2(pr[0], pr[1]);
  } else {
#pragma unroll
    for (int g = 0; g < GT; ++g) ps[r * GT + g] = pr[g];
  }
  if constexpr (PV == 1) {
    // ---- accp += p . V_pruned: value bytes to LDS, then 4 kept channels per lane ----------
    k_commit<KBV>(*vrp, vp->vbuf, lane);
    wave_sync_lds();
    // Rows r0 + rsub, r0 = 0, rpw, 2 rpw, ...; NS steps are read before they are used.  Nothing
    // branches: a row past the tile's end takes the bytes of the tile's last row and a weight of 0
    // -- rows nrows .. TR - 1 of ps were written as 0 above, and rows TR .. TR + kPsPad - 1 are
    // zero for the whole kernel (four steps of at most 8 rows may start at row nrows - 1).
    constexpr int NS = GT == 1 ? 4 : 2;   // steps read before they are used (registers)
    const int rowb = vp->ld * EB;
    const int vstep = vp->rpw * rowb, pstep = vp->rpw * GT;
    int voff = vp->shift + vp->col * 4 * EB + vp->rsub * rowb;
    const int vlast = vp->shift + vp->col * 4 * EB + (nrows - 1) * rowb;
    const float *pp = ps + vp->rsub * GT;
    for (int r0 = 0; r0 < nrows; r0 += NS * vp->rpw) {
      float f[NS][4], pg[NS][GT];
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        const char *vrow = vp->vbuf + min(voff, vlast);
        if constexpr (DT == THK_BF16) {
          const uint2 w = *(const uint2 *)vrow;
          f[i][0] = __uint_as_float(w.x << 16); f[i][1] = __uint_as_float(w.x & 0xffff0000u);
          f[i][2] = __uint_as_float(w.y << 16); f[i][3] = __uint_as_float(w.y & 0xffff0000u);
        } else {
          const float4 w = *(const float4 *)vrow;
          f[i][0] = w.x; f[i][1] = w.y; f[i][2] = w.z; f[i][3] = w.w;
        }
        if constexpr (GT == 4) {
          const float4 t4 = *(const float4 *)pp;
          pg[i][0] = t4.x; pg[i][1] = t4.y; pg[i][2] = t4.z; pg[i][3] = t4.w;
        } else if constexpr (GT == 2) {
          const float2 t2 = *(const float2 *)pp;
          pg[i][0] = t2.x; pg[i][1] = t2.y;
        } else {
#pragma unroll
          for (int g = 0; g < GT; ++g) pg[i][g] = pp[g];
        }
        voff += vstep;
        pp += pstep;
      }
#pragma unroll
      for (int i = 0; i < NS; ++i)
#pragma unroll
        for (int g = 0; g < GT; ++g)
#pragma unroll
          for (int e = 0; e < 4; ++e) st.accp[g][e] = fmaf(pg[i][g], f[i][e], st.accp[g][e]);
    }
  } else {
  wave_sync_lds();

  // ---- acc += p . V --------------------------------------------------------
#pragma unroll
  for (int b = 0; b < VS::NB; ++b) {
#pragma unroll
    for (int i = 0; i < VS::NV; ++i) {
      const int row = (b * VS::NV + i) * VS::RPL + vrow;
      float f[VEC];
      E::unpack(vr[i], f);
      float pv[GT];
      if constexpr (GT == 4) {
        const float4 t4 = *(const float4 *)(ps + row * 4);
        pv[0] = t4.x; pv[1] = t4.y; pv[2] = t4.z; pv[3] = t4.w;
      } else if constexpr (GT == 2) {
        const float2 t2 = *(const float2 *)(ps + row * 2);
        pv[0] = t2.x; pv[1] = t2.y;
      } else {
#pragma unroll
        for (int g = 0; g < GT; ++g) pv[g] = ps[row * GT + g];
      }
#pragma unroll
      for (int g = 0; g < GT; ++g)
#pragma unroll
        for (int v = 0; v < VEC; ++v) st.acc[g][v] = fmaf(pv[g], f[v], st.acc[g][v]);
    }
    if (b + 1 < VS::NB) v_issue<DT, TR, NV>(vr, vg, nrows, b + 1, lane);
  }
  }
  wave_sync_lds();   // ps and kbuf are rewritten by the next tile
}

// ---- cross-block hand-off of the split records (n_split > 1, at most kFuseMaxSplit pieces) ----
// The block that finishes LAST for a (unit, head group) merges the group's split records itself,
// so the call needs no second launch.  No read-modify-write is involved (the blocks of a group
// finish together, and a contended compare-and-swap loop costs a memory round trip per
// contender): every block has a FLAG word per (group, split).  A block
//   1. stores its record with device-scope relaxed atomic stores (they reach the coherence
//      point themselves: the L2 caches of the XCDs are not coherent with each other, and a
//      device-scope fence would write back a whole L2) and waits until they are acknowledged,
//   2. stores the call's nonce into its own flag and waits for that acknowledgement,
//   3. loads the group's flags: if all of them hold the nonce it merges.
// The block whose flag store is performed last finds all flags set, and by 1. every record is
// then visible to it.  Blocks that finish within a round trip of each other may both find all
// flags set: both merge, in split order, and store the same bits.  A merging block clears the
// flags afterwards, so that a replay of the same launch from a graph, which carries the same
// nonce, starts clean; whatever else the flag words held before the call (another call's nonce,
// other data of the workspace) is not the nonce: 64 bits drawn per call.
constexpr int kFuseMaxSplit = 16;

__device__ inline void pub_store_f32(float *p, float v) {
  __hip_atomic_store((unsigned int *)p, __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline float pub_load_f32(const float *p) {
  return __uint_as_float(__hip_atomic_load((const unsigned int *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}

// Merge of the four waves' softmax states (mrg: [GT][130] floats per wave, wstride floats from
// wave to wave, in LDS, complete and visible to the block): the output row of every query head
// the block serves, or this split's state record -- and, where the call merges inside the
// launch, the output rows again, from all records, by the block that arrives last.
// grp: index of the block's (unit, head group) among all of the call's; s_last: one int of LDS.
template <int DT, int GT>
__device__ __forceinline__ void block_merge_store(const float *mrg, int wstride, const DecodeArgs &a,
                                                  int64_t bn0, int sp, int heads, int64_t grp, int *s_last) {
  using E = Elem<DT>;
  const bool fused = a.arrive != nullptr;
  for (int o = threadIdx.x; o < heads * kD; o += 256) {   // heads <= GT of the block's slots are in use
    const int g = o / kD, c = o % kD;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) M = fmaxf(M, mrg[(size_t)w * wstride + g * (kD + 2)]);
    float Lsum = 0.f, A = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float *rec = mrg + (size_t)w * wstride + g * (kD + 2);
      const float wgt = rec[0] == -INFINITY ? 0.f : exp2f(rec[0] - M);
      Lsum = fmaf(rec[1], wgt, Lsum);
      A = fmaf(rec[2 + c], wgt, A);
    }
    const size_t bn = (size_t)(bn0 + g);
    if (a.n_split == 1) {
      E::store1(a.out, bn * kD + c, A / Lsum);
    } else {
      float *rec = a.ws + (bn * a.n_split + sp) * (kD + 2);
      if (fused) {
        pub_store_f32(rec + 2 + c, A);
        if (c == 0) { pub_store_f32(rec, M); pub_store_f32(rec + 1, Lsum); }
      } else {
        rec[2 + c] = A;
        if (c == 0) { rec[0] = M; rec[1] = Lsum; }
      }
    }
  }
  if (a.n_split == 1 || !fused) return;

  // ---- the group's last block merges: m = max m_i, l = sum l_i 2^(m_i - m), acc likewise, in
  // split order (the result does not depend on who arrives last) ---------------------------
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's record stores are acknowledged
  __syncthreads();                                   // ... and every wave's
  unsigned long long *flags = a.arrive + (size_t)grp * a.n_split;
  if (threadIdx.x < kWave) {
    if (threadIdx.x == 0)
      __hip_atomic_store(flags + sp, a.nonce, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the flag is out before the flags are read
    const unsigned long long f =
        (int)threadIdx.x < a.n_split
            ? __hip_atomic_load(flags + threadIdx.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
            : a.nonce;
    const bool all = __all(f == a.nonce);
    if (threadIdx.x == 0) *s_last = all ? 1 : 0;
  }
  __syncthreads();
  if (*s_last == 0) return;
  for (int o = threadIdx.x; o < heads * kD; o += 256) {
    const int g = o / kD, c = o % kD;
    const size_t bn = (size_t)(bn0 + g);
    const float *rec0 = a.ws + bn * a.n_split * (kD + 2);
    float mv[kFuseMaxSplit], lv[kFuseMaxSplit], av[kFuseMaxSplit];
#pragma unroll
    for (int i = 0; i < kFuseMaxSplit; ++i) {   // all loads in flight at once; entries past n_split repeat the last
      const float *rec = rec0 + (size_t)min(i, a.n_split - 1) * (kD + 2);
      mv[i] = pub_load_f32(rec);
      lv[i] = pub_load_f32(rec + 1);
      av[i] = pub_load_f32(rec + 2 + c);
    }
    float M = -INFINITY;
#pragma unroll
    for (int i = 0; i < kFuseMaxSplit; ++i) M = fmaxf(M, mv[i]);
    float Lsum = 0.f, A = 0.f;
#pragma unroll
    for (int i = 0; i < kFuseMaxSplit; ++i) {
      const float wgt = (i >= a.n_split || mv[i] == -INFINITY) ? 0.f : exp2f(mv[i] - M);
      Lsum = fmaf(lv[i], wgt, Lsum);
      A = fmaf(av[i], wgt, A);
    }
    E::store1(a.out, bn * kD + c, A / Lsum);
  }
  if ((int)threadIdx.x < a.n_split)
    __hip_atomic_store(flags + threadIdx.x, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// KB: 16-byte K chunks a lane may have to stage for one TR-row pruned tile.
// WPE: resident waves per SIMD the register budget is set for.
// VP = 1: the value rows of the pruned segment hold only the T_v kept channels (a.v is
// V_pruned with rows a.ld_v elements apart, a.idx_v lists the channels).  Their bytes are staged
// like the key bytes (KB chunks per lane, the class is chosen for the wider of the two), into the
// same wave-private LDS slab once the tile's key bytes have been consumed, and each lane
// accumulates 4 kept channels; at the end the sums are scattered to their channels.  The tail
// keeps full-width value rows.
template <int DT, int GT, int RA, int KB, int TR, int WPE, int VP = 0>
__global__ __launch_bounds__(256, WPE) void k_decode(DecodeArgs a, int groups, int kbuf_bytes) {
  using E = Elem<DT>;
  using VS = VShape<DT, TR>;
  constexpr int VEC = E::VEC, EB = E::EB, LPR = VS::LPR, LPK = kWave / TR;
  constexpr int KBT = kTailRows * kD * EB / 16 / kWave;   // chunks per lane of a tail tile
  extern __shared__ uint4 smem[];
  float *qk = (float *)smem;                 // [GT][kQS] gathered query channels, 0 beyond T
  float *qf = qk + GT * kQS;                 // [GT][kQS] full query
  uint32_t *qkp = (uint32_t *)(qf + GT * kQS);   // [GT][kQS/2] qk as packed bf16 pairs (bf16 inputs)
  uint32_t *qfp = qkp + GT * (kQS / 2);          // [GT][kQS/2] qf as packed bf16 pairs
  float *mrg = (float *)(qfp + GT * (kQS / 2));  // [4][GT][130] per-wave states for the final merge
  char *wbase = (char *)(mrg + 4 * GT * (kD + 2));
  __shared__ int s_last;
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int wstride = kbuf_bytes + GT * (TR + (VP ? kPsPad : 0)) * 4;
  char *kbuf = wbase + (size_t)wave * wstride;
  float *ps = (float *)(kbuf + kbuf_bytes);
  VPruned vpd;
  vpd.vbuf = kbuf;   // the key bytes of a tile are consumed before its value bytes are staged
  vpd.shift = 0;
  vpd.ld = a.ld_v;
  {
    const int lprv = VP ? (a.T_v + 3) / 4 : 1;          // lanes per value row, <= 32
    vpd.rpw = min(kWave / lprv, 8);
    vpd.col = lane % lprv;
    vpd.active = lane / lprv < vpd.rpw;
    vpd.rsub = vpd.active ? lane / lprv : 0;   // idle lanes repeat row group 0; their sums are dropped
  }

  const int sp = (int)(blockIdx.x % a.n_split);
  const int64_t ug = blockIdx.x / a.n_split;
  const int gi = (int)(ug % groups);
  const int64_t u = ug / groups;             // (layer, batch, KV head)
  const int G = a.N_q / a.N_kv;
  const int64_t bn0 = u * G + (int64_t)gi * GT;   // first query head served (heads of unit u: u*G ..)
  // the unit's last block may have fewer than GT heads left: the other slots carry a zero query
  // (their logits are 0, their output is never stored)
  const int hb = min(GT, G - gi * GT);

  const int64_t s0 = min(a.S, (int64_t)sp * a.rows_per_split);
  const int64_t s1 = min(a.S, s0 + a.rows_per_split);
  const int nt_p = (int)((s1 - s0 + TR - 1) / TR);
  const int nt_t = (a.s_tail + kTailRows - 1) / kTailRows;   // tail tiles of the unit: tile j goes to split j % n_split
  const char *kpg = (const char *)a.kp;

  constexpr int NV = VS::NV;
  const size_t krow0 = (size_t)u * a.unit_rows + s0;     // first K_pruned / V row of this block
  const u32x4 *vbase = (const u32x4 *)a.v + krow0 * LPR;

  // the first tile's key and value bytes start moving before anything else happens
  u32x4 kr[KB];
  u32x4 vr[NV];
  u32x4 vrp[VP ? KB : 1];
  int shift_next = 0;
  if (wave < nt_p) {
    const int nr = (int)min((int64_t)TR, s1 - s0 - (int64_t)wave * TR);
    shift_next = k_issue<DT, KB>(kr, kpg, (krow0 + (size_t)wave * TR) * a.ldk * EB, nr, a.T, a.ldk, lane);
    if constexpr (VP)
      vpd.shift = k_issue<DT, KB>(vrp, (const char *)a.v, (krow0 + (size_t)wave * TR) * a.ld_v * EB, nr, a.T_v,
                                  a.ld_v, lane);
    else
      v_issue<DT, TR, NV>(vr, vbase + (size_t)wave * TR * LPR, nr, 0, lane);
  }

  // query: gather the kept channels (Sec. 3.3: the query is pruned with the stored mask)
  const int16_t *uidx = a.idx + (size_t)u * a.T;
  for (int o = tid; o < GT * kQS; o += 256) {
    const int g = o / kQS, c = o % kQS;
    const size_t qb = (size_t)(bn0 + g) * kD;
    qf[o] = (g < hb && c < kD) ? E::load1(a.q, qb + c) : 0.f;
    qk[o] = (g < hb && c < a.T) ? E::load1(a.q, qb + uidx[c]) : 0.f;
  }
  if constexpr (DT == THK_BF16) {
    const uint16_t *q16 = (const uint16_t *)a.q;
    for (int o = tid; o < GT * (kQS / 2); o += 256) {
      const int g = o / (kQS / 2), c = 2 * (o % (kQS / 2));
      const size_t qb = (size_t)(bn0 + g) * kD;
      const bool used = g < hb;
      const uint32_t f0 = used && c < kD ? q16[qb + c] : 0u, f1 = used && c + 1 < kD ? q16[qb + c + 1] : 0u;
      const uint32_t k0 = used && c < a.T ? q16[qb + uidx[c]] : 0u;
      const uint32_t k1 = used && c + 1 < a.T ? q16[qb + uidx[c + 1]] : 0u;
      qfp[o] = f0 | (f1 << 16);
      qkp[o] = k0 | (k1 << 16);
    }
  }
  if constexpr (VP) {
    for (int o = lane; o < GT * kPsPad; o += kWave) ps[GT * TR + o] = 0.f;
  }
  __syncthreads();

  TileState<DT, GT> st;
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    st.m[g] = -INFINITY; st.l[g] = 0.f;
#pragma unroll
    for (int v = 0; v < VEC; ++v) st.acc[g][v] = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) st.accp[g][e] = 0.f;
  }

  // ---- pruned segment: the K bytes of this wave's next tile are in flight while
  // the current one is computed
  for (int ti = wave; ti < nt_p; ti += 4) {
    const int nrows = (int)min((int64_t)TR, s1 - s0 - (int64_t)ti * TR);
    const u32x4 *vg = vbase + (size_t)ti * TR * LPR;
    const int shift = shift_next;
    k_commit<KB>(kr, kbuf, lane);
    if (ti != wave) {
      if constexpr (VP)
        vpd.shift = k_issue<DT, KB>(vrp, (const char *)a.v, (krow0 + (size_t)ti * TR) * a.ld_v * EB, nrows,
                                    a.T_v, a.ld_v, lane);
      else
        v_issue<DT, TR, NV>(vr, vg, nrows, 0, lane);
    }
    if (ti + 4 < nt_p) {
      const int nr = (int)min((int64_t)TR, s1 - s0 - (int64_t)(ti + 4) * TR);
      shift_next = k_issue<DT, KB>(kr, kpg, (krow0 + (size_t)(ti + 4) * TR) * a.ldk * EB, nr, a.T, a.ldk, lane);
    }
    wave_sync_lds();
    if constexpr (VP)
      tile_compute<DT, GT, RA, TR, NV, 1, KB>(shift, nrows, a.T, a.ldk, qk, qkp, vg, vr, kbuf, ps, st,
                                              a.scale_log2_d, lane, &vrp, &vpd);
    else
      tile_compute<DT, GT, RA, TR, NV>(shift, nrows, a.T, a.ldk, qk, qkp, vg, vr, kbuf, ps, st, a.scale_log2_d, lane);
  }

  // ---- unpruned tail segment (full-width keys, full query) ------------------
  for (int ti = sp + wave * a.n_split; ti < nt_t; ti += 4 * a.n_split) {
    const int j0 = ti * kTailRows;
    const int nrows = min(kTailRows, a.s_tail - j0);
    const size_t row0 = (size_t)u * a.s_tail_cap + j0;
    u32x4 kt[KBT];
    k_issue<DT, KBT>(kt, (const char *)a.kt, row0 * kD * EB, nrows, kD, kD, lane);
    // the tail's value rows: a buffer of their own, or the rows that follow row S in v
    const u32x4 *vg = a.unified_v ? (const u32x4 *)a.v + ((size_t)u * a.unit_rows + a.S + j0) * LPR
                                  : (const u32x4 *)a.vt + row0 * LPR;
    v_issue<DT, TR, NV>(vr, vg, nrows, 0, lane);
    k_commit<KBT>(kt, kbuf, lane);
    wave_sync_lds();
    tile_compute<DT, GT, 16, TR, NV, (VP ? 2 : 0)>(0, nrows, kD, kD, qf, qfp, vg, vr, kbuf, ps, st, a.scale_log2_d,
                                                    lane);
  }

  // ---- wave state -> LDS ---------------------------------------------------
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    const float lt = wave_sum(st.l[g]) * (1.0f / LPK);
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
  if constexpr (VP) {
    // the sums over the pruned rows go to their channels, one row-within-step group at a time
    const int16_t *uidv = a.idx_v + (size_t)u * a.T_v;
    int cv[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int t = vpd.col * 4 + e;
      cv[e] = t < a.T_v ? uidv[t] : -1;
    }
    for (int rs = 0; rs < vpd.rpw; ++rs) {
      wave_sync_lds();
      if (vpd.active && vpd.rsub == rs) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (cv[e] >= 0) {
#pragma unroll
            for (int g = 0; g < GT; ++g) mrg[(size_t)(wave * GT + g) * (kD + 2) + 2 + cv[e]] += st.accp[g][e];
          }
        }
      }
    }
  }
  __syncthreads();

  block_merge_store<DT, GT>(mrg, GT * (kD + 2), a, bn0, sp, hb, ug, &s_last);
}

// ---- host side: pick the instantiation for a shape --------------------------
struct DecodeLaunch {
  int ra;      // byte alignment of K_pruned rows (16, 8, 4, 2)
  int kb;      // staged chunks per lane needed for one tile
};

template <int DT>
inline DecodeLaunch decode_launch_params(const DecodeArgs &a, int tr) {
  constexpr int eb = Elem<DT>::EB;
  DecodeLaunch p;
  // every row starts at a multiple of ld * eb bytes from the 16-byte aligned base
  const size_t rowb = (size_t)a.ldk * eb;
  p.ra = 16;
  while (rowb % p.ra) p.ra >>= 1;
  const int max_nch = (int)((tr * rowb + (p.ra == 16 ? 0 : 14) + 15) / 16);
  p.kb = (max_nch + kWave - 1) / kWave;
  return p;
}

template <int DT, int GT, int RA, int KB, int TR, int WPE, int VP>
inline hipError_t decode_launch_one(const DecodeArgs &a, int groups, hipStream_t st) {
  constexpr int eb = Elem<DT>::EB;
  int kbuf = KB * kWave * 16;                      // every staged chunk has an LDS slot
  const int tailbuf = kTailRows * kD * eb;
  if (kbuf < tailbuf) kbuf = tailbuf;
  const size_t lds = (size_t)(3 * GT * kQS + 4 * GT * (kD + 2)) * 4 + 4 * ((size_t)kbuf + GT * (TR + (VP ? kPsPad : 0)) * 4);
  const dim3 grid((unsigned)(a.units * groups * a.n_split)), block(256);
  {
    static DynLds set;   // one per instantiation
    const hipError_t e = ensure_dyn_lds((const void *)k_decode<DT, GT, RA, KB, TR, WPE, VP>, lds, set);
    if (e != hipSuccess) return e;
  }
  void *kargs[] = {(void *)&a, (void *)&groups, (void *)&kbuf};
  const hipError_t e = launch_main_kernel((const void *)k_decode<DT, GT, RA, KB, TR, WPE, VP>, grid, block, kargs, lds, st);
  return e != hipSuccess ? e : hipGetLastError();
}

template <int DT, int GT, int KB, int TR, int WPE, int VP>
inline hipError_t decode_launch_ra(const DecodeArgs &a, int ra, int groups, hipStream_t st) {
  if (ra == 16) return decode_launch_one<DT, GT, 16, KB, TR, WPE, VP>(a, groups, st);
  if (ra == 8) return decode_launch_one<DT, GT, 8, KB, TR, WPE, VP>(a, groups, st);
  if (ra == 4) return decode_launch_one<DT, GT, 4, KB, TR, WPE, VP>(a, groups, st);
  if constexpr (DT == THK_BF16) {
    if (ra == 2) return decode_launch_one<DT, GT, 2, KB, TR, WPE, VP>(a, groups, st);
  }
  return hipErrorInvalidValue;
}

// Tiles of 32 rows: two lanes share a key row, waves stay light (4 per SIMD when
// K staging is narrow and at most two query heads share the block, else 3).
template <int DT, int GT, int VP = 0>
hipError_t decode_launch_gt(const DecodeArgs &a, int groups, hipStream_t st) {
  constexpr int TR = 32;
  DecodeLaunch p = decode_launch_params<DT>(a, TR);
  if constexpr (VP) {
    // the value tile is staged with the same chunk count: size the class for the wider of the two
    const int kbv = (int)((TR * (size_t)a.ld_v * Elem<DT>::EB + 15 + 15) / 16 + kWave - 1) / kWave;
    if (kbv > p.kb) p.kb = kbv;
  }
  constexpr int KBN = (DT == THK_BF16) ? 5 : 10;   // T <= 79
  constexpr int KBW = (DT == THK_BF16) ? 9 : 17;   // up to ld_keep = 128
  // fp32 stages twice as many registers per tile: one wave per SIMD fewer than bf16 (at four
  // the fp32 kernels spilled 27-63 registers and ran at 3.7 TB/s instead of 5.3)
  constexpr int WN = DT == THK_F32 ? ((VP || GT == 4) ? 2 : 3) : (GT <= 2 ? 4 : 3);
  constexpr int WW = DT == THK_F32 ? 2 : (VP ? 2 : 3);
  if (p.kb <= KBN) return decode_launch_ra<DT, GT, KBN, TR, WN, VP>(a, p.ra, groups, st);
  if (p.kb <= KBW) return decode_launch_ra<DT, GT, KBW, TR, WW, VP>(a, p.ra, groups, st);
  return hipErrorInvalidValue;
}

}  // namespace thk
