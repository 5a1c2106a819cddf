// Value-channel score (Appendix "Value Cache Pruning"):
//   Score_v[j] = sum over the G query heads of a KV head of
//                || softmax(Q_obs K^T / sqrt(D)) V[:, j] ||_2 .
// The S_obs x S attention matrix times V is the one dense contraction of the method, so this
// file uses the matrix cores: a streaming attention over K and V (each read once) with the
// running-maximum softmax, followed by a small kernel that merges the pieces and takes the
// column norms.
//
// k_value_attn (bf16): 4 waves per block.  The G * S_obs query rows of one KV head are cut into
// tiles of 32 rows; a block carries QT of them (1, 2 or 4) and streams the keys in chunks of
// 128 rows; wave w works on query tile w % QT and on the QT consecutive 32-key sub-tiles
// number w / QT of every chunk.  Per 32-key sub-tile a wave computes
//   S^T = K_sub Q^T        8 x v_mfma_f32_32x32x16_bf16 (A = keys from LDS, B = queries in VGPRs)
//   P^T = exp2(S^T - m)    in the accumulator layout, which already is the B-operand layout
//   O^T += V_sub^T P^T     16 x MFMA (P^T as two bf16 terms, hi + lo); the A operand (values
//                          transposed) comes from row-major LDS through ds_read_b64_tr_b16
// so neither the softmax maximum (a query is a lane column: 16 registers and one cross-half
// exchange) nor the probabilities ever move between lanes.
#include "thk_internal.h"

namespace thk {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int kRec = 32 * kD + 64;   // floats per partial record: O^T [128][32], m [32], l [32]
constexpr float kNegBig = -1.0e30f;  // finite stand-in for "no key seen yet"

// One 32-key sub-tile of the running-maximum softmax in the MFMA accumulator layout: lane
// (n, h) holds, for query column n, the 16 keys kb + (r / 4) * 8 + h * 4 + r % 4.  Hides keys
// past `lim`, updates the running maximum (rescaling the row sum and the output accumulators
// when some query's maximum moved) and leaves the probabilities exp2(s * scale_log2 - m) in s.
__device__ __forceinline__ void softmax_step(f32x16 &s, int64_t kb, int h, int64_t lim, int64_t lim_min,
                                             float scale_log2, float &m_run, float &l_run, f32x16 (&o)[4]) {
  if (kb + 31 > lim_min) {   // wave-uniform: only the sub-tiles that reach the window or the end
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int64_t key = kb + (r >> 2) * 8 + h * 4 + (r & 3);
      if (key > lim) s[r] = -INFINITY;
    }
  }
  float mt = s[0];
#pragma unroll
  for (int r = 1; r < 16; ++r) mt = fmaxf(mt, s[r]);
  mt = fmaxf(mt, __shfl_xor(mt, 32));
  // the running maximum lives in the log2 domain (scale_log2 > 0 keeps the order)
  const float m_new = fmaxf(m_run, mt * scale_log2);
  if (__any(m_new > m_run)) {
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    l_run *= alpha;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
    m_run = m_new;
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) s[r] = __builtin_amdgcn_exp2f(fmaf(s[r], scale_log2, -m_run));
}

constexpr int kXcds = 8;   // workgroup i of a launch runs on XCD i % 8, each XCD behind an L2 of its own

// Which (query block, S piece, unit) a workgroup takes.  With one query block per unit the
// order is plain.  With several (more than 128 query rows per KV head) the blocks that stream
// the SAME keys and values are placed 8 workgroup numbers apart: same XCD, dispatched one after
// the other, so the second finds the rows in that XCD's L2 instead of fetching them again.
// False: a surplus workgroup of the rounded-up grid.
__device__ __forceinline__ bool value_block_work(const ValueAttnArgs &a, int &qb, int &sp, int64_t &u) {
  const int64_t bid = blockIdx.x;
  int64_t piece;   // (unit, S piece)
  if (a.n_qblk == 1) {
    qb = 0;
    piece = bid;
  } else {
    const int x = (int)(bid % kXcds);
    const int64_t slot = bid / kXcds;
    qb = (int)(slot % a.n_qblk);
    piece = (slot / a.n_qblk) * kXcds + x;
  }
  sp = (int)(piece % a.n_split);
  u = piece / a.n_split;
  return u < a.U;
}

// Partial record of one (unit, split, query tile): O^T [128][32], then m [32] and l [32].
__device__ __forceinline__ void write_record(float *rec, const f32x16 (&o)[4], float m_run, float l_tot, int n,
                                             int h) {
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int d = dt * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
      rec[d * 32 + n] = o[dt][r];
    }
  if (h == 0) {
    rec[32 * kD + n] = m_run;
    rec[32 * kD + 32 + n] = l_tot;
  }
}

// ---------------------------------------------------------------- bf16 ----
constexpr int kKst = 272;  // LDS bytes per key row: 16-lane b128 reads of 16 rows hit 64 distinct banks
constexpr int kVst = 320;  // LDS bytes per value row: the 4-row x 32-byte transposing reads of a
                           // half-wave cover all 64 banks once

template <int QT>
__global__ __launch_bounds__(256, 2) void k_value_attn_bf16(ValueAttnArgs a) {
  constexpr int KW = 4 / QT;     // waves that share a query tile, each on its own key sub-tiles
  constexpr int KT = QT;         // 32-key sub-tiles per wave and chunk
  constexpr int CR = 128;        // rows per chunk = KW * KT * 32
  constexpr int NP = 8;          // 16-row staging passes per chunk
  __shared__ __attribute__((aligned(16))) unsigned char smem[CR * (kKst + kVst)];
  unsigned char *Ks = smem, *Vs = smem + CR * kKst;

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int qt = w % QT, ksub = w / QT;
  const int n = lane & 31, h = lane >> 5;

  int qb, sp;
  int64_t u;
  if (!value_block_work(a, qb, sp, u)) return;

  const int rows_q = a.G * a.S_obs;
  const int qtile = qb * QT + qt;
  const int row = qtile * 32 + n;      // this lane's query row in the unit's (head, window row) list
  const int64_t S = a.S;

  // Query operand: 8 k-steps of 8 channels for this lane's (row, half).
  bf16x8 qreg[8];
  {
    const uint16_t *qp = (const uint16_t *)a.q_obs + ((size_t)u * rows_q + (row < rows_q ? row : 0)) * kD + h * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      u32x4 r = *(const u32x4 *)(qp + ks * 16);
      if (row >= rows_q) r = u32x4{0u, 0u, 0u, 0u};
      qreg[ks] = __builtin_bit_cast(bf16x8, r);
    }
  }
  // Last key this lane's query may see, and the smallest such limit in the call.
  const int64_t lim = a.causal ? S - a.S_obs + (row % a.S_obs) : S - 1;
  const int64_t lim_min = a.causal ? S - a.S_obs : S - 1;

  const int64_t k0 = (int64_t)sp * a.rows_per_split;
  const int64_t k1 = (k0 + a.rows_per_split < S) ? k0 + a.rows_per_split : S;
  const int nchunks = (int)((k1 - k0 + CR - 1) / CR);

  const unsigned char *kg = (const unsigned char *)a.k + (size_t)u * S * (kD * 2);
  const unsigned char *vg = (const unsigned char *)a.v + (size_t)u * S * (kD * 2);
  const int srow = tid >> 4, scol = (tid & 15) * 16;

  u32x4 pk[NP], pv[NP];
  // quarter q of the next chunk's loads: q = 0, 1 the two halves of the key rows, q = 2, 3 of
  // the value rows
  auto fetch_part = [&](int c, int q) {
    const unsigned char *g = q < 2 ? kg : vg;
#pragma unroll
    for (int pp = 0; pp < NP / 2; ++pp) {
      const int p = (q & 1) * (NP / 2) + pp;
      int64_t gr = k0 + (int64_t)c * CR + p * 16 + srow;
      gr = gr < S ? gr : S - 1;   // rows past the end repeat the last one; their weights are zero
      const u32x4 x = ld_stream((const u32x4 *)(g + gr * (kD * 2) + scol));
      if (q < 2) pk[p] = x; else pv[p] = x;
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      *(u32x4 *)(Ks + (p * 16 + srow) * kKst + scol) = pk[p];
      *(u32x4 *)(Vs + (p * 16 + srow) * kVst + scol) = pv[p];
    }
  };

  f32x16 o[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  float m_run = kNegBig, l_run = 0.f;

  // LDS addresses of this lane's operands inside a sub-tile
  const unsigned char *ka_p = Ks + (ksub * KT * 32 + n) * kKst + h * 16;
  const int j = lane & 15, gsub = (lane >> 4) & 1;
  const unsigned char *va_p = Vs + (ksub * KT * 32 + h * 4 + (j >> 2)) * kVst + (gsub * 16 + 4 * (j & 3)) * 2;

  if (nchunks > 0) {
#pragma unroll
    for (int q = 0; q < 4; ++q) fetch_part(0, q);
    stash();
  }
  __syncthreads();
  for (int c = 0; c < nchunks; ++c) {
    // the next chunk's loads are issued in four parts spread over this chunk's work, so that the
    // memory system has requests in flight throughout the compute phase
    const bool more = c + 1 < nchunks;
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      if (more) {
#pragma unroll
        for (int q = t * (4 / KT); q < (t + 1) * (4 / KT); ++q) fetch_part(c + 1, q);
      }
      const int64_t kb = k0 + (int64_t)c * CR + (ksub * KT + t) * 32;   // first key of the sub-tile
      if (kb >= k1) continue;
      const unsigned char *ka_t = ka_p + t * 32 * kKst, *va_t = va_p + t * 32 * kVst;
      f32x16 s;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 ka = *(const bf16x8 *)(ka_t + ks * 32);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[ks], s, 0, 0, 0);
      }
      softmax_step(s, kb, h, lim, lim_min, a.scale_log2, m_run, l_run, o);
      // The probabilities enter the second product as TWO bf16 terms, p = hi + lo with hi the
      // nearest bf16 to p and lo the nearest bf16 to p - hi (that difference is exact in fp32):
      // |p - hi - lo| <= 2^-18 p, so the matrix product loses nothing that fp32 arithmetic keeps.
      // The row sum takes the fp32 values.
      bf16x8 ph[2], pl[2];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const __bf16 hi = (__bf16)s[r];
        ph[r >> 3][r & 7] = hi;
        pl[r >> 3][r & 7] = (__bf16)(s[r] - (float)hi);
        l_run += s[r];
      }
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) {
          const unsigned char *vp = va_t + (k2 * 16) * kVst + dt * 64;
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4 *)(vp));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4 *)(vp + 8 * kVst));
          const bf16x8 va = __builtin_bit_cast(
              bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, ph[k2], o[dt], 0, 0, 0);
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pl[k2], o[dt], 0, 0, 0);
        }
      }
    }
    __syncthreads();
    if (c + 1 < nchunks) stash();
    __syncthreads();
  }

  // The waves that carried the same query tile over different key sub-tiles meet in LDS (the
  // staging buffers are free after the loop's last barrier): common maximum, rescale, and the
  // wave of sub-tile 0 adds the others up.
  float l_tot = l_run + __shfl_xor(l_run, 32);
  if constexpr (KW > 1) {
    float *mx = (float *)smem;                 // [KW][QT][32] maxima, then [KW][QT][32] sums
    float *ox = mx + 2 * KW * QT * 32;         // [KW - 1][QT][64 registers][64 lanes]
    if (h == 0) mx[(ksub * QT + qt) * 32 + n] = m_run;
    __syncthreads();
    float M = m_run;
#pragma unroll
    for (int k = 0; k < KW; ++k) M = fmaxf(M, mx[(k * QT + qt) * 32 + n]);
    const float alpha = __builtin_amdgcn_exp2f(m_run - M);
    l_tot *= alpha;
    m_run = M;
    if (ksub > 0) {
      float *dst = ox + (size_t)((ksub - 1) * QT + qt) * 64 * 64 + lane;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) dst[(dt * 16 + r) * 64] = o[dt][r] * alpha;
      if (h == 0) mx[(KW + ksub) * QT * 32 + qt * 32 + n] = l_tot;
    }
    __syncthreads();
    if (ksub > 0) return;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
#pragma unroll
    for (int k = 1; k < KW; ++k) {
      const float *src = ox + (size_t)((k - 1) * QT + qt) * 64 * 64 + lane;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] += src[(dt * 16 + r) * 64];
      l_tot += mx[(KW + k) * QT * 32 + qt * 32 + n];
    }
  }
  // partial record of (unit, split, query tile)
  const int nqt = a.n_qblk * QT;
  write_record(a.part + (((size_t)u * a.n_split + sp) * nqt + qtile) * kRec, o, m_run, l_tot, n, h);
}

// ---------------------------------------------------------------- fp32 ----
// The same streaming attention in full fp32 on v_mfma_f32_32x32x2_f32 (one 32-key tile per
// step, one wave per query tile, QT waves per block).  The contraction index of an MFMA step is
// the lane half h: step j of the logits multiplies channel 8 * (j / 4) + 4 * h + j % 4, so a
// lane reads its four channels of four consecutive steps as one 16-byte LDS word; step j of
// O^T += V^T P^T multiplies key (j / 4) * 8 + 4 * h + j % 4, which is accumulator register j of
// P^T.  Probabilities stay fp32.
constexpr int kKstF = 528;  // LDS bytes per key row (b128 reads of 16 rows: 64 distinct banks)
constexpr int kVstF = 544;  // LDS bytes per value row (the two halves read rows 4 apart: 32 banks apart)

template <int QT>
__global__ __launch_bounds__(64 * QT) void k_value_attn_f32(ValueAttnArgs a) {
  __shared__ __attribute__((aligned(16))) unsigned char Ks[32 * kKstF];
  __shared__ __attribute__((aligned(16))) unsigned char Vs[32 * kVstF];
  constexpr int NT = 64 * QT;
  const int tid = threadIdx.x, lane = tid & 63, qt = tid >> 6;
  const int n = lane & 31, h = lane >> 5;

  int qb, sp;
  int64_t u;
  if (!value_block_work(a, qb, sp, u)) return;

  const int rows_q = a.G * a.S_obs;
  const int qtile = qb * QT + qt;
  const int row = qtile * 32 + n;
  const int64_t S = a.S;

  float4 qreg[16];   // channels 8 * jj + 4 * h .. + 3 of this lane's query row
  {
    const float *qp = (const float *)a.q_obs + ((size_t)u * rows_q + (row < rows_q ? row : 0)) * kD + h * 4;
#pragma unroll
    for (int jj = 0; jj < 16; ++jj) {
      qreg[jj] = *(const float4 *)(qp + jj * 8);
      if (row >= rows_q) qreg[jj] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
  const int64_t lim = a.causal ? S - a.S_obs + (row % a.S_obs) : S - 1;
  const int64_t lim_min = a.causal ? S - a.S_obs : S - 1;
  const int64_t k0 = (int64_t)sp * a.rows_per_split;
  const int64_t k1 = (k0 + a.rows_per_split < S) ? k0 + a.rows_per_split : S;

  const unsigned char *kg = (const unsigned char *)a.k + (size_t)u * S * (kD * 4);
  const unsigned char *vg = (const unsigned char *)a.v + (size_t)u * S * (kD * 4);

  f32x16 o[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  float m_run = kNegBig, l_run = 0.f;

  const unsigned char *ka_p = Ks + n * kKstF + h * 16;
  const unsigned char *va_p = Vs + (h * 4) * kVstF + n * 4;

  for (int64_t kb = k0; kb < k1; kb += 32) {
    __syncthreads();   // the previous tile is no longer read
    // 32 rows of 512 bytes each: 1024 16-byte pieces per tensor
#pragma unroll 4
    for (int i = tid; i < 1024; i += NT) {
      const int r = i >> 5, c = (i & 31) * 16;
      int64_t gr = kb + r;
      gr = gr < S ? gr : S - 1;   // rows past the end repeat the last one; their weights are zero
      *(u32x4 *)(Ks + r * kKstF + c) = *(const u32x4 *)(kg + gr * (kD * 4) + c);
      *(u32x4 *)(Vs + r * kVstF + c) = *(const u32x4 *)(vg + gr * (kD * 4) + c);
    }
    __syncthreads();
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int jj = 0; jj < 16; ++jj) {
      const float4 ka = *(const float4 *)(ka_p + jj * 32);
      s = __builtin_amdgcn_mfma_f32_32x32x2f32(ka.x, qreg[jj].x, s, 0, 0, 0);
      s = __builtin_amdgcn_mfma_f32_32x32x2f32(ka.y, qreg[jj].y, s, 0, 0, 0);
      s = __builtin_amdgcn_mfma_f32_32x32x2f32(ka.z, qreg[jj].z, s, 0, 0, 0);
      s = __builtin_amdgcn_mfma_f32_32x32x2f32(ka.w, qreg[jj].w, s, 0, 0, 0);
    }
    softmax_step(s, kb, h, lim, lim_min, a.scale_log2, m_run, l_run, o);
#pragma unroll
    for (int r = 0; r < 16; ++r) l_run += s[r];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const unsigned char *vp = va_p + ((j >> 2) * 8 + (j & 3)) * kVstF;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        const float va = *(const float *)(vp + dt * 128);
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x2f32(va, s[j], o[dt], 0, 0, 0);
      }
    }
  }
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const int nqt = a.n_qblk * QT;
  write_record(a.part + (((size_t)u * a.n_split + sp) * nqt + qtile) * kRec, o, m_run, l_tot, n, h);
}

// Merge the partial records of one 32-row query tile of one unit and normalise.  A block of
// 256 threads covers DQ = 256 / PG value channels: thread (d, pg) sums the records p = pg,
// pg + PG, ... for channel d; the PG groups meet in LDS and are added in group order.  A unit
// with a single tile gets its score here (each thread holds all of its rows); otherwise the
// squared outputs go to sq[u][row][d] for k_value_norms.  PG = 2 for few records, 8 for many.
template <int PG>
__global__ __launch_bounds__(256) void k_value_merge(const float *part, float *sq, float *score, int G, int S_obs,
                                                     int n_part, int nqt, int nt) {
  constexpr int DQ = 256 / PG, NDB = kD / DQ;   // channels per block, blocks per (unit, tile)
  extern __shared__ float wts[];   // [n_part][32] merge weights, then [PG - 1][DQ][33] for the groups
  int64_t bid = blockIdx.x;
  const int db = (int)(bid % NDB);
  bid /= NDB;
  const int64_t u = bid / nt;
  const int t = (int)(bid % nt);
  const int dl = threadIdx.x % DQ, pg = threadIdx.x / DQ;
  const int d = db * DQ + dl;
  const int rows_q = G * S_obs;
  const float *pu = part + (size_t)u * n_part * nqt * kRec;
  if (threadIdx.x < 32) {
    const int q = threadIdx.x;
    float M = kNegBig;
    for (int p = 0; p < n_part; ++p) M = fmaxf(M, pu[((size_t)p * nqt + t) * kRec + 32 * kD + q]);
    float L = 0.f;
    for (int p = 0; p < n_part; ++p) {
      const float *r = pu + ((size_t)p * nqt + t) * kRec + 32 * kD;
      const float wv = __builtin_amdgcn_exp2f(r[q] - M);
      wts[p * 32 + q] = wv;
      L += wv * r[32 + q];
    }
    const float inv = L > 0.f ? 1.f / L : 0.f;
    for (int p = 0; p < n_part; ++p) wts[p * 32 + q] *= inv;
  }
  __syncthreads();
  float acc[32];
#pragma unroll
  for (int q = 0; q < 32; ++q) acc[q] = 0.f;
  for (int p = pg; p < n_part; p += PG) {
    const float4 *src = (const float4 *)(pu + ((size_t)p * nqt + t) * kRec + d * 32);
    const float *wp = wts + p * 32;
#pragma unroll
    for (int q4 = 0; q4 < 8; ++q4) {
      const float4 x = src[q4];
      acc[q4 * 4 + 0] += wp[q4 * 4 + 0] * x.x;
      acc[q4 * 4 + 1] += wp[q4 * 4 + 1] * x.y;
      acc[q4 * 4 + 2] += wp[q4 * 4 + 2] * x.z;
      acc[q4 * 4 + 3] += wp[q4 * 4 + 3] * x.w;
    }
  }
  __syncthreads();               // the weights are no longer read
  float *xch = wts;              // [PG - 1][DQ][33]
  if (pg > 0) {
#pragma unroll
    for (int q = 0; q < 32; ++q) xch[((pg - 1) * DQ + dl) * 33 + q] = acc[q];
  }
  __syncthreads();
  if (pg > 0) return;
#pragma unroll
  for (int g2 = 1; g2 < PG; ++g2)
#pragma unroll
    for (int q = 0; q < 32; ++q) acc[q] += xch[((g2 - 1) * DQ + dl) * 33 + q];
  if (nt == 1) {
    double ss = 0.0, total = 0.0;
#pragma unroll
    for (int q = 0; q < 32; ++q) {
      if (q < rows_q) {
        ss += (double)acc[q] * (double)acc[q];
        if ((q + 1) % S_obs == 0) {   // last window row of a head
          total += sqrt(ss);
          ss = 0.0;
        }
      }
    }
    score[(size_t)u * kD + d] = (float)total;
  } else {
    float *dst = sq + ((size_t)u * nt + t) * 32 * kD;
#pragma unroll
    for (int q = 0; q < 32; ++q) dst[q * kD + d] = acc[q] * acc[q];
  }
}

// Column norms per query head from the squared outputs.  1024 threads = 128 channels x 8 head
// groups: thread (d, hg) sums the squares of heads hg, hg + 8, ... (eight rows in flight), takes
// the roots, and the groups are added in group order.
__global__ __launch_bounds__(1024) void k_value_norms(const float *sq, float *score, int G, int S_obs, int nt) {
  __shared__ double tot[8][kD];
  const int64_t u = blockIdx.x;
  const int d = threadIdx.x & (kD - 1), hg = threadIdx.x >> 7;
  const float *src = sq + (size_t)u * nt * 32 * kD + d;
  double total = 0.0;
  for (int g = hg; g < G; g += 8) {
    const float *hs = src + (size_t)g * S_obs * kD;
    double ss = 0.0;
    for (int i0 = 0; i0 < S_obs; i0 += 8) {
      float x[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) x[j] = hs[(size_t)min(i0 + j, S_obs - 1) * kD];
#pragma unroll
      for (int j = 0; j < 8; ++j) ss += (i0 + j < S_obs) ? (double)x[j] : 0.0;
    }
    total += sqrt(ss);
  }
  tot[hg][d] = total;
  __syncthreads();
  if (hg == 0) {
    double t = tot[0][d];
#pragma unroll
    for (int g2 = 1; g2 < 8; ++g2) t += tot[g2][d];
    score[(size_t)u * kD + d] = (float)t;
  }
}

}  // namespace

int value_attn_qt(int G, int S_obs) {
  const int nqt = (G * S_obs + 31) / 32;
  return nqt >= 4 ? 4 : nqt >= 2 ? 2 : 1;
}

size_t value_part_bytes(int64_t U, int G, int S_obs, int n_split) {
  const int QT = value_attn_qt(G, S_obs);
  const int nqt = (G * S_obs + 31) / 32;
  const int n_qblk = (nqt + QT - 1) / QT;
  const size_t sq = nqt > 1 ? (size_t)U * nqt * 32 * kD * sizeof(float) : 0;
  return (size_t)U * n_split * n_qblk * QT * kRec * sizeof(float) + sq;
}

hipError_t launch_value_score(int dtype, const void *q_obs, const void *k, const void *v, float *part,
                              float *score, int64_t U, int64_t S, int G, int S_obs, int causal,
                              int n_split, int64_t rows_per_split, hipStream_t st) {
  clear_stale_hip_error();
  const int QT = value_attn_qt(G, S_obs);
  const int nqt_real = (G * S_obs + 31) / 32;
  ValueAttnArgs a;
  a.q_obs = q_obs; a.k = k; a.v = v; a.part = part;
  a.S = S; a.rows_per_split = rows_per_split;
  a.G = G; a.S_obs = S_obs; a.n_split = n_split; a.causal = causal;
  a.n_qblk = (nqt_real + QT - 1) / QT;
  a.scale_log2 = (float)(1.4426950408889634 / sqrt((double)kD));
  a.U = U;
  // several query blocks per (unit, piece): pieces rounded up to a multiple of the XCD count
  // (value_block_work; the surplus workgroups return at once)
  const int64_t pieces = a.n_qblk == 1 ? U * n_split : (U * n_split + kXcds - 1) / kXcds * kXcds;
  const unsigned grid = (unsigned)(pieces * a.n_qblk);
  const void *fn;
  int threads = 256;
  if (dtype == THK_BF16) {
    fn = QT == 4 ? (const void *)k_value_attn_bf16<4> : QT == 2 ? (const void *)k_value_attn_bf16<2> : (const void *)k_value_attn_bf16<1>;
  } else {
    fn = QT == 4 ? (const void *)k_value_attn_f32<4> : QT == 2 ? (const void *)k_value_attn_f32<2> : (const void *)k_value_attn_f32<1>;
    threads = QT == 4 ? 256 : QT == 2 ? 128 : 64;
  }
  void *kargs[] = {(void *)&a};
  hipError_t e = launch_main_kernel(fn, dim3(grid), dim3(threads), kargs, 0, st);
  if (e == hipSuccess) e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int n_part = n_split;
  const int nqt = a.n_qblk * QT;
  float *sq = part + (size_t)U * n_part * nqt * kRec;   // behind the partial records
  // few records: 2 groups x 128 channels per block; many: 8 groups x 32 channels, 4 blocks
  const int PG = n_part > 8 ? 8 : 2;
  const int DQ = 256 / PG;
  size_t lds = (size_t)n_part * 32 * sizeof(float);
  const size_t xch = (size_t)(PG - 1) * DQ * 33 * sizeof(float);
  if (lds < xch) lds = xch;
  const dim3 mg((unsigned)(U * nqt_real * (kD / DQ)));
  if (PG == 8)
    hipLaunchKernelGGL(k_value_merge<8>, mg, dim3(256), lds, st, part, sq, score, G, S_obs, n_part, nqt, nqt_real);
  else
    hipLaunchKernelGGL(k_value_merge<2>, mg, dim3(256), lds, st, part, sq, score, G, S_obs, n_part, nqt, nqt_real);
  e = hipGetLastError();
  if (e != hipSuccess || nqt_real == 1) return e;
  hipLaunchKernelGGL(k_value_norms, dim3((unsigned)U), dim3(1024), 0, st, sq, score, G, S_obs, nqt_real);
  return hipGetLastError();
}

}  // namespace thk
