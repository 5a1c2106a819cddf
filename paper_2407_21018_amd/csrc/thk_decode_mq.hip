// Decode attention over the pruned key cache for bf16 caches whose KV heads serve three or more
// query heads each (Sec. 3.3, Fig. 2; attention formula of Sec. 3.2) -- gfx950, wave64.
//
// With four query heads per key row the two products of a tile are skinny matrix products
// (4 x T by T x 32, then 4 x 32 by 32 x 128) and go to the matrix cores as batches of 4 x 4
// blocks (v_mfma_f32_4x4x4_16B_bf16: 16 independent blocks per instruction; lane 4 b + x holds
// row x of A_b, column x of B_b and column x of D_b).  Work split, tile size, staging of the key
// bytes, split records and the final merge are those of k_decode; what differs is one tile:
//
//   logits   block b <-> key rows 4 (b % 8) .. + 3 and one half (b / 8) of the kept channels.
//            A_b = four key rows x four channels, 8 bytes per lane straight from the staged
//            bytes in LDS; B_b = the four query heads' same four channels; D_b[i][j] is the
//            partial logit of row i and head j.  The blocks of one half walk the channel chunks
//            in rotated order so that the row reads spread over the LDS banks; the two halves
//            are added with one cross-half exchange.
//   softmax  lane 4 b + j owns head j and four rows: the running maximum is a per-lane scalar,
//            reduced over the lanes of equal j.  A probability is split into two bf16 terms
//            (p = hi + lo, exact to 2^-16), so that the matrix product loses nothing against
//            the fp32 arithmetic of the other kernels.
//   values   block b <-> output channels 4 b .. + 3 (two instructions cover 128 channels).
//            A_b = the four heads' probabilities of four rows, the same for every block (read
//            back from a 512-byte LDS line); B_b = four value rows x four channels, which is a
//            transposed read of the row-major value tile: ds_read_b64_tr_b16 out of LDS, where
//            the tile is staged with the two 128-byte halves of odd rows swapped (the four rows
//            of one read then cover all banks).  D_b[i][j] accumulates head i, channel 4 b + j:
//            lane l ends with channels l and 64 + l of all four heads.
//   VP = 1   channel-pruned value rows (T_v kept channels, rows ld_v elements apart): their bytes
//            are staged like the key bytes, as a flat range, and the same transposing reads walk
//            them with the row pitch ld_v; lane l then sums kept channels l and 64 + l, which
//            are scattered to their output channels at the end.  The tail keeps full-width rows.
//   NH = 2   eight query heads per KV head in one block: two groups of four share every key
//            and value operand read from LDS; queries, probabilities and accumulators double.
//
// The kernel streams at the rate of a plain read of the same bytes only while its instruction
// stream stays short (a wave64 instruction holds its SIMD for four cycles, and three or four
// waves share one): the wave index is made uniform so that tile counts, row counts and their
// branches live in scalar registers; a whole tile (32 rows, all but a block's last) takes
// straight-line paths -- value loads at fixed offsets without per-row clamps, the eight 4-row
// steps of the second product without a test between them so that later reads overlap earlier
// products; rows of whole 8-channel groups (T a multiple of 8) take a logit loop without masks or
// range checks; tiles of at most 4 KB of keys get a staging class of their own (no fifth,
// duplicate chunk).  Together: 805 MB (64 units x 32768 rows, G = 4) 130.4 -> 125.9 us, 403 MB
// (8 units x 131072 rows) 68.0 -> 65.0 us; with no arithmetic at all the same loads take 123 us.
#include <stdlib.h>

#include "thk_decode_impl.h"

namespace thk {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kMqRows = 32;                       // rows per tile
constexpr int kMqVBytes = kMqRows * kD * 2;       // a value tile in LDS
constexpr int kMqVChunks = kMqVBytes / 16 / kWave;   // 16-byte value chunks per lane and tile

struct MqState {
  float m;        // running maximum of this lane's head (lane % 4), log2 domain
  float l;        // this lane's share of its head's probability sum
  f32x4 acc[2];   // acc[h][i]: head i, channel 64 h + lane
  f32x4 accp[2];  // channel-pruned values only: accp[h][i]: head i, kept channel number 64 h + lane
};

__device__ __forceinline__ f32x4 mfma4(s16x4 a, s16x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a, b, c, 0, 0, 0);
}

// x combined over the lanes of equal lane % 4 inside each half of the wave (rotations by 4 and 8
// inside the 16-lane rows, then the neighbouring row).
template <bool MAX>
__device__ __forceinline__ float quad_column_reduce(float x) {
  float y = dpp_move<0x124, 0xf>(x, x);   // row_ror:4
  x = MAX ? max_nn(x, y) : x + y;
  y = dpp_move<0x128, 0xf>(x, x);         // row_ror:8
  x = MAX ? max_nn(x, y) : x + y;
  const LanePair p = pair16(x);
  return MAX ? max_nn(p.a, p.b) : p.a + p.b;
}

// Value rows of a tile into registers: chunk j * 64 + lane is 16 bytes of row 4 j + lane / 16.
// Rows past a ragged tile's end re-read its last row (their probability is 0).
__device__ __forceinline__ void mq_v_issue(u32x4 (&vr)[kMqVChunks], const u32x4 *__restrict__ vg, int nrows,
                                           int lane) {
  if (nrows == kMqRows) {   // a whole tile is one contiguous run: chunk j * 64 + lane as it lies in memory
#pragma unroll
    for (int j = 0; j < kMqVChunks; ++j) vr[j] = ld_stream(vg + j * kWave + lane);
    return;
  }
  const int rsub = lane >> 4, col = lane & 15;
#pragma unroll
  for (int j = 0; j < kMqVChunks; ++j) vr[j] = ld_stream(vg + (size_t)min(4 * j + rsub, nrows - 1) * 16 + col);
}

// ... and into the slab: rows 256 bytes apart, the two halves of odd rows swapped.
__device__ __forceinline__ void mq_v_commit(const u32x4 (&vr)[kMqVChunks], char *slab, int lane) {
  const int rsub = lane >> 4, col = (lane & 15) ^ ((rsub & 1) << 3);
#pragma unroll
  for (int j = 0; j < kMqVChunks; ++j) *(u32x4 *)(slab + (4 * j + rsub) * 256 + col * 16) = vr[j];
}

// Logits of a tile whose key bytes are in the slab, for NH groups of four heads.  nch =
// ceil(W / 4) 4-channel chunks per row; qrow: this lane's head of the first group as packed bf16, zero from
// chunk nch on (the same head of the next group follows 4 * kQS / 2 words later).  d[g] receives,
// in both halves of the wave, the dot products of rows 4 ((lane / 4) % 8) + r, r = 0 .. 3, with
// head 4 g + lane % 4: the key operand is read once for all groups.
// W: elements per key row; the elements the last chunk holds past W (row padding, or whatever
// follows the tile) are masked off, so their bytes never matter.
template <int NH>
__device__ __forceinline__ void mq_logits(const char *slab, int shift, int nrows, int W, int pitch_bytes,
                                          const uint32_t *qrow, int lane, f32x4 (&d)[NH]) {
  const int nch = (W + 3) >> 2;
  const uint32_t m0 = (W & 3) == 1 ? 0x0000ffffu : 0xffffffffu;
  const uint32_t m1 = (W & 3) == 0 ? 0xffffffffu : (W & 3) == 3 ? 0x0000ffffu : 0u;
  const int b = lane >> 2, x = lane & 3, half = b >> 3, bb = b & 7;
  const char *rowp = slab + shift + min(4 * bb + x, nrows - 1) * pitch_bytes;
  const int nst = (nch + 1) >> 1;          // chunks per half = matrix instructions per group
  int rel = bb % nst;
  f32x4 d0[NH], d1[NH];
#pragma unroll
  for (int g = 0; g < NH; ++g) {
    d0[g] = f32x4{0.f, 0.f, 0.f, 0.f};
    d1[g] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  auto step = [&](f32x4 (&acc)[NH]) {
    const int c = half * nst + rel;
    // a chunk past the row's end: the row's first chunk against the zero chunk of the query
    const bool valid = c < nch;
    const int ck = valid ? c : 0;
    uint2 kw = *(const uint2 *)(rowp + ck * 8);
    const bool last = ck == nch - 1;
    kw.x &= last ? m0 : 0xffffffffu;
    kw.y &= last ? m1 : 0xffffffffu;
    const s16x4 ka = __builtin_bit_cast(s16x4, kw);
    const char *qp = (const char *)qrow + (valid ? c : nch) * 8;
#pragma unroll
    for (int g = 0; g < NH; ++g) acc[g] = mfma4(ka, *(const s16x4 *)(qp + g * 4 * (kQS / 2) * 4), acc[g]);
    rel = rel + 1 == nst ? 0 : rel + 1;
  };
  if ((W & 7) == 0) {
    // Rows of whole chunks, an even number of them: every step of both halves is a real chunk
    // and nothing is masked.  off walks this lane's chunks as a byte offset, wrapping inside
    // the half's range.
    const int lo = half * nst * 8, hi = lo + nst * 8;
    int off = lo + rel * 8;
    const char *qb = (const char *)qrow;
    auto pstep = [&](f32x4 (&acc)[NH]) {
      const s16x4 ka = *(const s16x4 *)(rowp + off);
#pragma unroll
      for (int g = 0; g < NH; ++g) acc[g] = mfma4(ka, *(const s16x4 *)(qb + off + g * 4 * (kQS / 2) * 4), acc[g]);
      off = off + 8 == hi ? lo : off + 8;
    };
    int ks = 0;
    for (; ks + 4 <= nst; ks += 4) { pstep(d0); pstep(d1); pstep(d0); pstep(d1); }
    for (; ks + 2 <= nst; ks += 2) { pstep(d0); pstep(d1); }
    if (ks < nst) pstep(d0);
  } else {
    int ks = 0;
    for (; ks + 2 <= nst; ks += 2) { step(d0); step(d1); }
    if (ks < nst) step(d0);
  }
#pragma unroll
  for (int g = 0; g < NH; ++g)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const LanePair t = pair32(d0[g][r] + d1[g][r]);
      d[g][r] = t.a + t.b;
    }
}

// Running softmax over the tile's logits; the probabilities go to pline as two bf16 terms:
// bytes [0, 256) the leading terms, [256, 512) the remainders, entry 4 ks + head holding the
// four rows 4 ks .. 4 ks + 3.
template <int VP>
__device__ __forceinline__ void mq_softmax(const f32x4 &d, int nrows, float scale, MqState &st, char *pline,
                                           int lane) {
  const int bb = (lane >> 2) & 7;
  float zz[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) zz[r] = (nrows == kMqRows || 4 * bb + r < nrows) ? d[r] * scale : -INFINITY;
  const float mx = quad_column_reduce<true>(max_nn(max_nn(zz[0], zz[1]), max_nn(zz[2], zz[3])));
  const float m_new = max_nn(st.m, mx);             // finite: the tile has at least one row
  if (__builtin_amdgcn_ballot_w64(m_new != st.m) != 0) {   // rare after the first tiles
    const float corr = __builtin_amdgcn_exp2f(st.m - m_new);
    st.l *= corr;
    st.m = m_new;
    // every lane carries channels of all four heads: the heads' factors sit in the lane's quad
    const float c0 = dpp_move<0x00, 0xf>(corr, corr), c1 = dpp_move<0x55, 0xf>(corr, corr);
    const float c2 = dpp_move<0xAA, 0xf>(corr, corr), c3 = dpp_move<0xFF, 0xf>(corr, corr);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      st.acc[h][0] *= c0; st.acc[h][1] *= c1; st.acc[h][2] *= c2; st.acc[h][3] *= c3;
      if constexpr (VP) {
        st.accp[h][0] *= c0; st.accp[h][1] *= c1; st.accp[h][2] *= c2; st.accp[h][3] *= c3;
      }
    }
  }
  uint32_t hi[4], lo[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const float p = __builtin_amdgcn_exp2f(zz[r] - m_new);
    st.l += p;
    hi[r] = __float_as_uint(p) & 0xffff0000u;
    lo[r] = __float_as_uint(p - __uint_as_float(hi[r])) & 0xffff0000u;
  }
  // the lower half of the wave writes the leading terms, the upper half the remainders
  const bool up = lane >= 32;
  uint2 w;
  w.x = up ? ((lo[0] >> 16) | lo[1]) : ((hi[0] >> 16) | hi[1]);
  w.y = up ? ((lo[2] >> 16) | lo[3]) : ((hi[2] >> 16) | hi[3]);
  *(uint2 *)(pline + lane * 8) = w;
}

// acc += P . V for the tile whose value rows are in the slab; the probabilities of head group g
// are in the 512 bytes at pline + 512 g.  The value operand is read once for all groups.
template <int NH>
__device__ __forceinline__ void mq_values(const char *slab, const char *pline, int nrows, MqState (&st)[NH],
                                          int lane) {
  const int x = lane & 3, grp = lane >> 4, j = lane & 15, r = j >> 2, seg = j & 3;
  const int cc = 2 * grp + (seg >> 1), swz = (r & 1) << 3;
  const char *vb0 = slab + r * 256 + ((cc ^ swz) << 4) + (seg & 1) * 8;        // channels 0 .. 63
  const char *vb1 = slab + r * 256 + (((8 + cc) ^ swz) << 4) + (seg & 1) * 8;  // channels 64 .. 127
  const char *pa = pline + x * 8;
  auto rows4 = [&](const int ks) {
    const s16x4 b0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4 *)(vb0 + ks * 1024));
    const s16x4 b1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4 *)(vb1 + ks * 1024));
    s16x4 a_hi[NH], a_lo[NH];
#pragma unroll
    for (int g = 0; g < NH; ++g) {
      a_hi[g] = *(const s16x4 *)(pa + g * 512 + ks * 32);
      a_lo[g] = *(const s16x4 *)(pa + g * 512 + 256 + ks * 32);
    }
#pragma unroll
    for (int g = 0; g < NH; ++g) {
      st[g].acc[0] = mfma4(a_hi[g], b0, st[g].acc[0]);
      st[g].acc[1] = mfma4(a_hi[g], b1, st[g].acc[1]);
    }
#pragma unroll
    for (int g = 0; g < NH; ++g) {
      st[g].acc[0] = mfma4(a_lo[g], b0, st[g].acc[0]);
      st[g].acc[1] = mfma4(a_lo[g], b1, st[g].acc[1]);
    }
  };
  if (nrows == kMqRows) {   // a whole tile: straight-line code, the reads of later rows overlap the products
#pragma unroll
    for (int ks = 0; ks < kMqRows / 4; ++ks) rows4(ks);
    return;
  }
  const int nks = (nrows + 3) >> 2;
#pragma unroll
  for (int ks = 0; ks < kMqRows / 4; ++ks)
    if (ks < nks) rows4(ks);
}

// accp += P . V_pruned for the tile whose value bytes sit in the slab as staged (first row at
// byte `shift`, rows pitch_bytes apart).  A read past a row's T_v channels lands in the next row,
// or within the bytes that follow every slab, and only feeds kept-channel numbers >= T_v,
// which nobody collects; a row past a ragged tile's end is read as the tile's last row, with
// probability 0.
template <int NH>
__device__ __forceinline__ void mq_values_pruned(const char *slab, int shift, int pitch_bytes, int T_v,
                                                 const char *pline, int nrows, MqState (&st)[NH], int lane) {
  const int x = lane & 3, grp = lane >> 4, j = lane & 15, r = j >> 2, seg = j & 3;
  const char *vb = slab + shift + (16 * grp + 4 * seg) * 2;
  const char *pa = pline + x * 8;
  const int nks = (nrows + 3) >> 2;
  const bool wide = T_v > 64;
#pragma unroll
  for (int ks = 0; ks < kMqRows / 4; ++ks) {
    if (ks >= nks) break;
    const char *vrow = vb + min(4 * ks + r, nrows - 1) * pitch_bytes;
    const s16x4 b0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(vrow));
    s16x4 a_hi[NH], a_lo[NH];
#pragma unroll
    for (int g = 0; g < NH; ++g) {
      a_hi[g] = *(const s16x4 *)(pa + g * 512 + ks * 32);
      a_lo[g] = *(const s16x4 *)(pa + g * 512 + 256 + ks * 32);
      st[g].accp[0] = mfma4(a_hi[g], b0, st[g].accp[0]);
    }
    if (wide) {
      const s16x4 b1 =
          __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(vrow + 128));
#pragma unroll
      for (int g = 0; g < NH; ++g) st[g].accp[1] = mfma4(a_hi[g], b1, st[g].accp[1]);
#pragma unroll
      for (int g = 0; g < NH; ++g) {
        st[g].accp[0] = mfma4(a_lo[g], b0, st[g].accp[0]);
        st[g].accp[1] = mfma4(a_lo[g], b1, st[g].accp[1]);
      }
    } else {
#pragma unroll
      for (int g = 0; g < NH; ++g) st[g].accp[0] = mfma4(a_lo[g], b0, st[g].accp[0]);
    }
  }
}

// KB: 16-byte key chunks a lane may have to stage for one tile.  slab_bytes: the wave's LDS slab,
// which holds a tile's key bytes and, once the logits are done, its value rows.
// VP = 1: the value rows of the pruned segment are channel-pruned (a.v = V_pruned, a.ld_v, a.idx_v).
// NH: groups of four query heads served by one block (1, or 2 when N_q / N_kv is a multiple of 8:
// the key and value operands are then read from LDS once for eight heads).
template <int KB, int WPE, int VP, int NH>
__global__ __launch_bounds__(256, WPE) void k_decode_mq(DecodeArgs a, int groups, int slab_bytes) {
  constexpr int DT = THK_BF16, GT = 4 * NH, EB = 2, TR = kMqRows, LPR = 16;
  constexpr int KBT = kTailRows * kD * EB / 16 / kWave;   // chunks per lane of a tail tile
  extern __shared__ uint4 smem[];
  uint32_t *qkp = (uint32_t *)smem;                 // [GT][kQS/2] kept query channels, packed bf16, 0 beyond T
  uint32_t *qfp = qkp + GT * (kQS / 2);             // [GT][kQS/2] full query
  char *wbase = (char *)(qfp + GT * (kQS / 2));
  const int tid = threadIdx.x, lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);   // uniform: tile counts and branches stay scalar
  char *slab = wbase + (size_t)wave * (slab_bytes + 512 * NH);
  char *pline = slab + slab_bytes;               // 512 bytes of probabilities per head group
  __shared__ int s_last;

  const int sp = (int)(blockIdx.x % a.n_split);
  const int64_t ug = blockIdx.x / a.n_split;
  const int gi = (int)(ug % groups);
  const int64_t u = ug / groups;             // (layer, batch, KV head)
  const int G = a.N_q / a.N_kv;
  const int64_t bn0 = u * G + (int64_t)gi * GT;
  const int hb = min(GT, G - gi * GT);   // head slots in use; the others carry a zero query

  const int64_t s0 = min(a.S, (int64_t)sp * a.rows_per_split);
  const int64_t s1 = min(a.S, s0 + a.rows_per_split);
  const int nt_p = (int)((s1 - s0 + TR - 1) / TR);
  const int nt_t = (a.s_tail + kTailRows - 1) / kTailRows;   // tail tiles of the unit: tile j goes to split j % n_split
  const char *kpg = (const char *)a.kp;
  const size_t krow0 = (size_t)u * a.unit_rows + s0;     // first K_pruned / V row of this block
  const u32x4 *vbase = (const u32x4 *)a.v + krow0 * LPR;

  // the first tile's key and value bytes start moving before anything else happens
  u32x4 kr[KB];
  u32x4 vr[kMqVChunks];
  u32x4 vrp[VP ? KB : 1];
  int shift_next = 0, vshift = 0;
  if (wave < nt_p) {
    const int nr = (int)min((int64_t)TR, s1 - s0 - (int64_t)wave * TR);
    shift_next = k_issue<DT, KB>(kr, kpg, (krow0 + (size_t)wave * TR) * a.ldk * EB, nr, a.T, a.ldk, lane);
    if constexpr (VP)
      vshift = k_issue<DT, KB>(vrp, (const char *)a.v, (krow0 + (size_t)wave * TR) * a.ld_v * EB, nr, a.T_v, a.ld_v,
                               lane);
    else
      mq_v_issue(vr, vbase + (size_t)wave * TR * LPR, nr, lane);
  }

  // query: gather the kept channels (Sec. 3.3: the query is pruned with the stored mask)
  {
    const int16_t *uidx = a.idx + (size_t)u * a.T;
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
  __syncthreads();

  MqState st[NH];
#pragma unroll
  for (int g = 0; g < NH; ++g) {
    st[g].m = -INFINITY;
    st[g].l = 0.f;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      st[g].acc[h] = f32x4{0.f, 0.f, 0.f, 0.f};
      st[g].accp[h] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
  }
  const int x = lane & 3;
  const int pitch_bytes = a.ldk * EB;

  // ---- pruned segment: the bytes of this wave's next tile are in flight while the current
  // one is computed
  for (int ti = wave; ti < nt_p; ti += 4) {
    const int nrows = (int)min((int64_t)TR, s1 - s0 - (int64_t)ti * TR);
    const bool more = ti + 4 < nt_p;
    const int nr4 = more ? (int)min((int64_t)TR, s1 - s0 - (int64_t)(ti + 4) * TR) : 0;
    const int shift = shift_next;
    k_commit<KB>(kr, slab, lane);
    if (more)
      shift_next = k_issue<DT, KB>(kr, kpg, (krow0 + (size_t)(ti + 4) * TR) * a.ldk * EB, nr4, a.T, a.ldk, lane);
    wave_sync_lds();
    f32x4 d[NH];
    mq_logits<NH>(slab, shift, nrows, a.T, pitch_bytes, qkp + x * (kQS / 2), lane, d);
#pragma unroll
    for (int g = 0; g < NH; ++g) mq_softmax<VP>(d[g], nrows, a.scale_log2, st[g], pline + 512 * g, lane);
    wave_sync_lds();   // the key bytes are consumed: the slab takes the value rows
    if constexpr (VP) {
      const int vs = vshift;
      k_commit<KB>(vrp, slab, lane);
      if (more)
        vshift = k_issue<DT, KB>(vrp, (const char *)a.v, (krow0 + (size_t)(ti + 4) * TR) * a.ld_v * EB, nr4, a.T_v,
                                 a.ld_v, lane);
      wave_sync_lds();
      mq_values_pruned<NH>(slab, vs, a.ld_v * EB, a.T_v, pline, nrows, st, lane);
    } else {
      mq_v_commit(vr, slab, lane);
      if (more) mq_v_issue(vr, vbase + (size_t)(ti + 4) * TR * LPR, nr4, lane);
      wave_sync_lds();
      mq_values<NH>(slab, pline, nrows, st, lane);
    }
    wave_sync_lds();   // slab and pline are rewritten by the next tile
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
    mq_v_issue(vr, vg, nrows, lane);
    k_commit<KBT>(kt, slab, lane);
    wave_sync_lds();
    f32x4 d[NH];
    mq_logits<NH>(slab, 0, nrows, kD, kD * EB, qfp + x * (kQS / 2), lane, d);
#pragma unroll
    for (int g = 0; g < NH; ++g) mq_softmax<VP>(d[g], nrows, a.scale_log2, st[g], pline + 512 * g, lane);
    wave_sync_lds();
    mq_v_commit(vr, slab, lane);
    wave_sync_lds();
    mq_values<NH>(slab, pline, nrows, st, lane);
    wave_sync_lds();
  }

  // ---- wave state -> LDS: [GT][130] floats at the start of the wave's own slab -------------
  {
    float *mrg = (float *)slab;
#pragma unroll
    for (int g = 0; g < NH; ++g) {
      const float lt = quad_column_reduce<false>(st[g].l);   // both halves of the wave saw every row
      if (lane < 4) {
        float *rec = mrg + (4 * g + lane) * (kD + 2);
        rec[0] = st[g].m;
        rec[1] = lt;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float *rec = mrg + (4 * g + i) * (kD + 2) + 2;
        rec[lane] = st[g].acc[0][i];
        rec[64 + lane] = st[g].acc[1][i];
      }
    }
    if constexpr (VP) {
      // the sums over the pruned rows go to their channels (distinct for distinct kept numbers)
      wave_sync_lds();
      const int16_t *uidv = a.idx_v + (size_t)u * a.T_v;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int t = 64 * h + lane;
        if (t < a.T_v) {
          const int c = uidv[t];
#pragma unroll
          for (int g = 0; g < NH; ++g)
#pragma unroll
            for (int i = 0; i < 4; ++i) mrg[(4 * g + i) * (kD + 2) + 2 + c] += st[g].accp[h][i];
        }
      }
    }
  }
  __syncthreads();
  block_merge_store<DT, GT>((const float *)wbase, (slab_bytes + 512 * NH) / 4, a, bn0, sp, hb, ug, &s_last);
}

// Four blocks per compute unit with the narrow staging class and four heads per block (37 KB of
// LDS and at most 128 registers per lane each), two with the wide class and eight heads, three
// otherwise.
template <int KB, int VP, int NH>
static hipError_t mq_launch(const DecodeArgs &a, int groups, hipStream_t st) {
  constexpr int WPE = (KB <= 5 && NH == 1) ? 4 : (KB > 5 && NH == 2) ? 2 : 3;
  const int slab = KB * kWave * 16 > kMqVBytes ? KB * kWave * 16 : kMqVBytes;
  const size_t lds = (size_t)(2 * 4 * NH * (kQS / 2)) * 4 + 4 * ((size_t)slab + 512 * NH);
  const dim3 grid((unsigned)(a.units * groups * a.n_split)), block(256);
  {
    static DynLds set;   // one per instantiation
    const hipError_t e = ensure_dyn_lds((const void *)k_decode_mq<KB, WPE, VP, NH>, lds, set);
    if (e != hipSuccess) return e;
  }
  void *kargs[] = {(void *)&a, (void *)&groups, (void *)&slab};
  const hipError_t e = launch_main_kernel((const void *)k_decode_mq<KB, WPE, VP, NH>, grid, block, kargs, lds, st);
  return e != hipSuccess ? e : hipGetLastError();
}

// Staged 16-byte chunks per lane for one tile: the wider of the key rows and, when they are
// channel-pruned, the value rows.
static int mq_chunks(const DecodeArgs &a) {
  int kb = decode_launch_params<THK_BF16>(a, kMqRows).kb;
  if (a.T_v > 0) {
    const int kbv = (int)((kMqRows * (size_t)a.ld_v * 2 + 15 + 15) / 16 + kWave - 1) / kWave;
    if (kbv > kb) kb = kbv;
  }
  return kb;
}

// True when the shape is one this kernel serves: bf16, at least three query heads per KV head
// (one or two share a key row cheaply enough on the vector units), and rows (keys, and values
// when they are channel-pruned) whose pitch is a multiple of four elements, so that every operand
// is an aligned 8 bytes (T itself is free: dense rows qualify when T is a multiple of 4, other T
// with a padded pitch).  THK_DECODE_MFMA=0 in the environment keeps such shapes on k_decode.
bool decode_mq_serves(const DecodeArgs &a) {
  if (a.dtype != THK_BF16 || a.N_kv <= 0) return false;
  const int G = a.N_q / a.N_kv;
  if (G < 3 || a.ldk % 4 != 0) return false;
  if (a.T_v > 0 && a.ld_v % 4 != 0) return false;
  if (mq_chunks(a) > 9) return false;
  return !env_switches().decode_mfma_off;
}

// Head slots per block: four for three or four query heads per KV head, else eight; a unit
// takes ceil(G / slots) blocks per split and the last one may leave slots empty.
int decode_mq_heads(const DecodeArgs &a) { return (a.N_q / a.N_kv) <= 4 ? 4 : 8; }

// Staging classes: 4 chunks per lane (a 32-row tile of at most 4 KB: T <= 64 with 16-byte rows),
// 5 (T <= 79) and 9 (up to 128 kept channels).
template <int VP, int NH>
static hipError_t mq_launch_class(const DecodeArgs &a, int groups, hipStream_t st) {
  const int kb = mq_chunks(a);
  if (kb <= 4) return mq_launch<4, VP, NH>(a, groups, st);
  if (kb <= 5) return mq_launch<5, VP, NH>(a, groups, st);
  return mq_launch<9, VP, NH>(a, groups, st);
}

hipError_t decode_mq_launch(const DecodeArgs &a, hipStream_t st) {
  const int G = a.N_q / a.N_kv;
  if (decode_mq_heads(a) == 8) {
    const int groups = (G + 7) / 8;
    return a.T_v > 0 ? mq_launch_class<1, 2>(a, groups, st) : mq_launch_class<0, 2>(a, groups, st);
  }
  const int groups = (G + 3) / 4;
  return a.T_v > 0 ? mq_launch_class<1, 1>(a, groups, st) : mq_launch_class<0, 1>(a, groups, st);
}

}  // namespace thk
