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

__device__ inline void wave_sync_lds() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ inline float wave_max(float x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
  return x;
}
__device__ inline float wave_sum(float x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
  return x;
}

// 16 bytes at byte offset `off` of a tensor of `total` bytes; bytes past the end read as 0.
__device__ inline uint4 load_chunk(const char *base, size_t off, size_t total) {
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

// Process one tile of `nrows` (<= 64) rows whose keys are W elements wide with
// row stride ld (elements) starting at byte kbeg of tensor kg (ktot bytes), and
// whose value rows start at vg (16-byte chunks, 128 elements per row).
template <int DT, int GT, int RA>
__device__ __forceinline__ void attn_tile(const char *__restrict__ kg, size_t kbeg, size_t ktot,
                                          int nrows, int W, int ld,
                                          const float *__restrict__ qs,
                                          const uint4 *__restrict__ vg, char *kbuf, float *ps,
                                          TileState<DT, GT> &st, float scale, int lane) {
  using E = Elem<DT>;
  constexpr int VEC = E::VEC, EB = E::EB;
  constexpr int LPR = kD / VEC;              // lanes (= 16-byte chunks) per V row
  constexpr int RPL = kWave / LPR;           // V rows per wave-wide load
  constexpr int VB = 16;                     // V loads per lane per batch
  constexpr int NB = LPR / VB;               // batches per 64-row tile (1 bf16, 2 fp32)
  constexpr int KBATCH = (DT == THK_BF16) ? 10 : 16;
  constexpr int EPR = RA / EB;               // elements per LDS row read

  // ---- 1. fetch: first K batch, then the first V batch, then K -> LDS -------
  const size_t kend = kbeg + ((size_t)(nrows - 1) * ld + W) * EB;
  const size_t a0 = kbeg & ~(size_t)15;
  const int shift = (int)(kbeg - a0);
  const int nch = (int)((kend - a0 + 15) >> 4);

  uint4 kr[KBATCH];
#pragma unroll
  for (int j = 0; j < KBATCH; ++j) {
    const int c = j * kWave + lane;
    if (c < nch) kr[j] = load_chunk(kg, a0 + (size_t)c * 16, ktot);
  }
  uint4 vr[VB];
  const int vrow = lane / LPR;
#pragma unroll
  for (int i = 0; i < VB; ++i) {
    const int row = i * RPL + vrow;
    vr[i] = row < nrows ? vg[(size_t)i * kWave + lane] : make_uint4(0, 0, 0, 0);
  }
#pragma unroll
  for (int j = 0; j < KBATCH; ++j) {
    const int c = j * kWave + lane;
    if (c < nch) ((uint4 *)kbuf)[c] = kr[j];
  }
  for (int cb = KBATCH * kWave; cb < nch; cb += KBATCH * kWave) {   // wide rows only
#pragma unroll
    for (int j = 0; j < KBATCH; ++j) {
      const int c = cb + j * kWave + lane;
      if (c < nch) kr[j] = load_chunk(kg, a0 + (size_t)c * 16, ktot);
    }
#pragma unroll
    for (int j = 0; j < KBATCH; ++j) {
      const int c = cb + j * kWave + lane;
      if (c < nch) ((uint4 *)kbuf)[c] = kr[j];
    }
  }
  wave_sync_lds();

  // ---- 2. logits: lane r owns row r --------------------------------------
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

  // ---- 3. running softmax (base-2 exponent, scale folded in) -------------
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

  // ---- 4. acc += p . V ----------------------------------------------------
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
    if (b + 1 < NB) {
#pragma unroll
      for (int i = 0; i < VB; ++i) {
        const int row = ((b + 1) * VB + i) * RPL + vrow;
        vr[i] = row < nrows ? vg[(size_t)((b + 1) * VB + i) * kWave + lane] : make_uint4(0, 0, 0, 0);
      }
    }
  }
  wave_sync_lds();   // ps and kbuf are rewritten by the next tile
}

template <int DT, int GT, int RA>
__global__ __launch_bounds__(256) void k_decode(DecodeArgs a, int groups, int kbuf_bytes) {
  using E = Elem<DT>;
  constexpr int VEC = E::VEC, EB = E::EB, LPR = kD / VEC;
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

  const int64_t s0 = min(a.S, (int64_t)sp * a.rows_per_split);
  const int64_t s1 = min(a.S, s0 + a.rows_per_split);
  const int nt_p = (int)((s1 - s0 + 63) >> 6);
  const int nt_t = (sp == a.n_split - 1) ? (a.s_tail + kTailRows - 1) / kTailRows : 0;
  for (int ti = wave; ti < nt_p + nt_t; ti += 4) {
    if (ti < nt_p) {
      const int64_t r0 = s0 + (int64_t)ti * 64;
      const int nrows = (int)min((int64_t)64, s1 - r0);
      attn_tile<DT, GT, RA>((const char *)a.kp, ((size_t)u * a.S + r0) * a.ldk * EB, a.kp_bytes,
                            nrows, a.T, a.ldk, qk,
                            (const uint4 *)a.v + ((size_t)u * a.S + r0) * LPR, kbuf, ps, st,
                            a.scale_log2, lane);
    } else {
      const int j0 = (ti - nt_p) * kTailRows;
      const int nrows = min(kTailRows, a.s_tail - j0);
      const size_t row0 = (size_t)u * a.s_tail_cap + j0;
      attn_tile<DT, GT, 16>((const char *)a.kt, row0 * kD * EB,
                            (size_t)a.units * a.s_tail_cap * kD * EB, nrows, kD, kD, qf,
                            (const uint4 *)a.vt + row0 * LPR, kbuf, ps, st, a.scale_log2, lane);
    }
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
// acc = sum acc_i 2^(m_i - m), out = acc / l.  One block per query head,
// thread c owns channel c; splits are visited in index order.
template <int DT>
__global__ __launch_bounds__(128) void k_decode_merge(const float *__restrict__ ws,
                                                      void *__restrict__ out, int n_split) {
  using E = Elem<DT>;
  const int c = threadIdx.x;
  const size_t bn = blockIdx.x;
  const float *rec0 = ws + bn * n_split * (kD + 2);
  float M = -INFINITY;
  for (int i = 0; i < n_split; ++i) M = fmaxf(M, rec0[(size_t)i * (kD + 2)]);
  float Lsum = 0.f, A = 0.f;
  for (int i = 0; i < n_split; ++i) {
    const float *rec = rec0 + (size_t)i * (kD + 2);
    const float wgt = rec[0] == -INFINITY ? 0.f : exp2f(rec[0] - M);
    Lsum = fmaf(rec[1], wgt, Lsum);
    A = fmaf(rec[2 + c], wgt, A);
  }
  E::store1(out, bn * kD + c, A / Lsum);
}

template <int DT, int GT>
static hipError_t launch_decode_ra(const DecodeArgs &a, int ra, int groups, hipStream_t st) {
  const int eb = Elem<DT>::EB;
  int kbuf = (int)(64 * (size_t)a.ldk * eb + 32);
  const int tailbuf = kTailRows * kD * eb;
  if (kbuf < tailbuf) kbuf = tailbuf;
  kbuf = (kbuf + 15) & ~15;
  const size_t lds = (size_t)(2 * GT * kD + 4 * GT * (kD + 2)) * 4 + 4 * ((size_t)kbuf + GT * kWave * 4);
  const dim3 grid((unsigned)(a.units * groups * a.n_split)), block(256);
#define THK_LAUNCH(RA)                                                                        \
  do {                                                                                        \
    hipError_t e = hipSuccess;                                                                \
    if (lds > 48 * 1024)                                                                      \
      e = hipFuncSetAttribute((const void *)k_decode<DT, GT, RA>,                             \
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);          \
    if (e != hipSuccess) return e;                                                            \
    hipLaunchKernelGGL((k_decode<DT, GT, RA>), grid, block, lds, st, a, groups, kbuf);        \
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

template <int DT>
static hipError_t launch_decode_dt(const DecodeArgs &a, hipStream_t st) {
  const int eb = Elem<DT>::EB;
  const int G = a.N_q / a.N_kv;
  // row alignment of K_pruned relative to its 16-byte aligned base: every row
  // starts at a multiple of ld * eb bytes
  const size_t rowb = (size_t)a.ldk * eb;
  int ra = 16;
  while (rowb % ra) ra >>= 1;
  const int gt = (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1;
  const int groups = G / gt;
  hipError_t e;
  if (gt == 4) e = launch_decode_ra<DT, 4>(a, ra, groups, st);
  else if (gt == 2) e = launch_decode_ra<DT, 2>(a, ra, groups, st);
  else e = launch_decode_ra<DT, 1>(a, ra, groups, st);
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
