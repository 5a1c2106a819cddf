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
// (4 / QT) * 32 rows, so wave w works on query tile w % QT and key sub-tile w / QT of every
// chunk.  Per 32-key sub-tile a wave computes
//   S^T = K_sub Q^T        8 x v_mfma_f32_32x32x16_bf16 (A = keys from LDS, B = queries in VGPRs)
//   P^T = exp2(S^T - m)    in the accumulator layout, which already is the B-operand layout
//   O^T += V_sub^T P^T     8 x MFMA; the A operand (values transposed) comes from row-major LDS
//                          through ds_read_b64_tr_b16
// so neither the softmax maximum (a query is a lane column: 16 registers and one cross-half
// exchange) nor the probabilities ever move between lanes.
#include "thk_internal.h"

namespace thk {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int kRec = 32 * kD + 64;   // floats per partial record: O^T [128][32], m [32], l [32]
constexpr float kNegBig = -1.0e30f;  // finite stand-in for "no key seen yet"

// ---------------------------------------------------------------- bf16 ----
constexpr int kKst = 272;  // LDS bytes per key row: 16-lane b128 reads of 16 rows hit 64 distinct banks
constexpr int kVst = 320;  // LDS bytes per value row: the 4-row x 32-byte transposing reads of a
                           // half-wave cover all 64 banks once

template <int QT>
__global__ __launch_bounds__(256, 2) void k_value_attn_bf16(ValueAttnArgs a) {
  constexpr int KW = 4 / QT;     // key sub-tiles per chunk
  constexpr int CR = KW * 32;    // rows per chunk
  constexpr int NP = 2 * KW;     // 16-row staging passes per chunk
  __shared__ __attribute__((aligned(16))) unsigned char Ks[CR * kKst];
  __shared__ __attribute__((aligned(16))) unsigned char Vs[CR * kVst];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int qt = w % QT, ksub = w / QT;
  const int n = lane & 31, h = lane >> 5;

  int64_t bid = blockIdx.x;
  const int qb = (int)(bid % a.n_qblk);
  bid /= a.n_qblk;
  const int sp = (int)(bid % a.n_split);
  const int64_t u = bid / a.n_split;

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
  auto fetch = [&](int c) {
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      int64_t gr = k0 + (int64_t)c * CR + p * 16 + srow;
      gr = gr < S ? gr : S - 1;   // rows past the end repeat the last one; their weights are zero
      pk[p] = *(const u32x4 *)(kg + gr * (kD * 2) + scol);
      pv[p] = *(const u32x4 *)(vg + gr * (kD * 2) + scol);
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
  const unsigned char *ka_p = Ks + (ksub * 32 + n) * kKst + h * 16;
  const int j = lane & 15, gsub = (lane >> 4) & 1;
  const unsigned char *va_p = Vs + (ksub * 32 + h * 4 + (j >> 2)) * kVst + (gsub * 16 + 4 * (j & 3)) * 2;

  if (nchunks > 0) {
    fetch(0);
    stash();
  }
  __syncthreads();
  for (int c = 0; c < nchunks; ++c) {
    if (c + 1 < nchunks) fetch(c + 1);
    const int64_t kb = k0 + (int64_t)c * CR + ksub * 32;   // first key of this wave's sub-tile
    if (kb < k1) {
      f32x16 s;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 ka = *(const bf16x8 *)(ka_p + ks * 32);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[ks], s, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] *= a.scale_log2;
      if (kb + 31 > lim_min) {   // wave-uniform: only the chunks that reach the window or the end
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
      const float m_new = fmaxf(m_run, mt);
      if (__any(m_new > m_run)) {
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        l_run *= alpha;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
        m_run = m_new;
      }
      // probabilities, rounded to bf16 once; the same rounded values feed the row sum
      bf16x8 pb[2];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(s[r] - m_run);
        const __bf16 pr = (__bf16)p;
        pb[r >> 3][r & 7] = pr;
        l_run += (float)pr;
      }
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) {
          const unsigned char *vp = va_p + (k2 * 16) * kVst + dt * 64;
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4 *)(vp));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4 *)(vp + 8 * kVst));
          const bf16x8 va = __builtin_bit_cast(
              bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[k2], o[dt], 0, 0, 0);
        }
      }
    }
    __syncthreads();
    if (c + 1 < nchunks) stash();
    __syncthreads();
  }

  // partial record of (unit, split, key sub-tile lane, query tile)
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const int n_part = a.n_split * KW;
  const int nqt = a.n_qblk * QT;
  float *rec = a.part + (((size_t)u * n_part + (size_t)sp * KW + ksub) * nqt + qtile) * kRec;
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

// Merge the partial records of one unit, normalise, and take the column norms per query head.
// 128 threads = the 128 value channels.
__global__ __launch_bounds__(128) void k_value_finalize(const float *part, float *score, int G, int S_obs,
                                                        int n_part, int nqt) {
  extern __shared__ float wts[];   // [n_part][32] merge weights of the current query tile
  const int64_t u = blockIdx.x;
  const int d = threadIdx.x;
  const int rows_q = G * S_obs;
  const float *pu = part + (size_t)u * n_part * nqt * kRec;
  double ss = 0.0, total = 0.0;   // running sum of squares of the current head; sum of finished heads
  for (int t = 0; t * 32 < rows_q; ++t) {
    __syncthreads();
    if (d < 32) {
      float M = kNegBig;
      for (int p = 0; p < n_part; ++p) M = fmaxf(M, pu[((size_t)p * nqt + t) * kRec + 32 * kD + d]);
      float L = 0.f;
      for (int p = 0; p < n_part; ++p) {
        const float *r = pu + ((size_t)p * nqt + t) * kRec + 32 * kD;
        const float wv = __builtin_amdgcn_exp2f(r[d] - M);
        wts[p * 32 + d] = wv;
        L += wv * r[32 + d];
      }
      const float inv = L > 0.f ? 1.f / L : 0.f;
      for (int p = 0; p < n_part; ++p) wts[p * 32 + d] *= inv;
    }
    __syncthreads();
    float acc[32];
#pragma unroll
    for (int q = 0; q < 32; ++q) acc[q] = 0.f;
    for (int p = 0; p < n_part; ++p) {
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
#pragma unroll
    for (int q = 0; q < 32; ++q) {
      const int row = t * 32 + q;
      if (row < rows_q) {
        ss += (double)acc[q] * (double)acc[q];
        if ((row + 1) % S_obs == 0) {   // last window row of a head
          total += sqrt(ss);
          ss = 0.0;
        }
      }
    }
  }
  score[(size_t)u * kD + d] = (float)total;
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
  return (size_t)U * n_split * (4 / QT) * n_qblk * QT * kRec * sizeof(float);
}

hipError_t launch_value_score(int dtype, const void *q_obs, const void *k, const void *v, float *part,
                              float *score, int64_t U, int64_t S, int G, int S_obs, int causal,
                              int n_split, int64_t rows_per_split, hipStream_t st) {
  if (dtype != THK_BF16) return hipErrorInvalidValue;
  const int QT = value_attn_qt(G, S_obs);
  const int nqt_real = (G * S_obs + 31) / 32;
  ValueAttnArgs a;
  a.q_obs = q_obs; a.k = k; a.v = v; a.part = part;
  a.S = S; a.rows_per_split = rows_per_split;
  a.G = G; a.S_obs = S_obs; a.n_split = n_split; a.causal = causal;
  a.n_qblk = (nqt_real + QT - 1) / QT;
  a.scale_log2 = (float)(1.4426950408889634 / sqrt((double)kD));
  const unsigned grid = (unsigned)(U * n_split * a.n_qblk);
  profile_mark(true, st);
  if (QT == 4) hipLaunchKernelGGL(k_value_attn_bf16<4>, dim3(grid), dim3(256), 0, st, a);
  else if (QT == 2) hipLaunchKernelGGL(k_value_attn_bf16<2>, dim3(grid), dim3(256), 0, st, a);
  else hipLaunchKernelGGL(k_value_attn_bf16<1>, dim3(grid), dim3(256), 0, st, a);
  profile_mark(false, st);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int n_part = n_split * (4 / QT);
  hipLaunchKernelGGL(k_value_finalize, dim3((unsigned)U), dim3(128), (size_t)n_part * 32 * sizeof(float), st,
                     part, score, G, S_obs, n_part, a.n_qblk * QT);
  return hipGetLastError();
}

}  // namespace thk
