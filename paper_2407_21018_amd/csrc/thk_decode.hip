// Decode attention: dispatch to the per-(dtype, group width) kernels and the
// merge of the per-split softmax states (gfx950, wave64).
#include "thk_decode_impl.h"

namespace thk {

constexpr int kMaxSplitDev = 4096;   // largest n_split the API accepts
static_assert(kFuseMaxSplit == kDecodeFuseMaxSplit, "the host and the kernels must agree on the fused merge's reach");

hipError_t decode_launch_bf16_g1(const DecodeArgs &, int, hipStream_t);
hipError_t decode_launch_bf16_g2(const DecodeArgs &, int, hipStream_t);
hipError_t decode_launch_bf16_g4(const DecodeArgs &, int, hipStream_t);
hipError_t decode_launch_f32_g1(const DecodeArgs &, int, hipStream_t);
hipError_t decode_launch_f32_g2(const DecodeArgs &, int, hipStream_t);
hipError_t decode_launch_f32_g4(const DecodeArgs &, int, hipStream_t);
hipError_t decode_kv_launch_bf16_g1(const DecodeArgs &, int, hipStream_t);
hipError_t decode_kv_launch_bf16_g2(const DecodeArgs &, int, hipStream_t);
hipError_t decode_kv_launch_bf16_g4(const DecodeArgs &, int, hipStream_t);
hipError_t decode_kv_launch_f32_g1(const DecodeArgs &, int, hipStream_t);
hipError_t decode_kv_launch_f32_g2(const DecodeArgs &, int, hipStream_t);
hipError_t decode_kv_launch_f32_g4(const DecodeArgs &, int, hipStream_t);
// four query heads per KV head on the matrix cores (bf16, full-width values)
hipError_t decode_mq_launch(const DecodeArgs &, hipStream_t);

// Merge of the per-split states: m = max m_i, l = sum l_i 2^(m_i - m),
// acc = sum acc_i 2^(m_i - m), out = acc / l.  One block of 128 * PG threads per query head:
// thread (c, g) owns channel c and the g-th contiguous share of the splits.  The (m_i, l_i)
// pairs are read once per block, turned into weights kept in LDS, and the acc_i[c] loads of
// eight splits are in flight together; the PG shares are then added in share order, so the
// result does not depend on timing.  PG = 4 when there are many splits (few heads, long S).
template <int DT, int PG>
__global__ __launch_bounds__(128 * PG) void k_decode_merge(const float *__restrict__ ws,
                                                           void *__restrict__ out, int n_split) {
  using E = Elem<DT>;
  constexpr int NW = 2 * PG;   // wavefronts per block
  __shared__ float wgt[kMaxSplitDev];
  __shared__ float red[NW];
  __shared__ float part_l[PG], part_a[PG][kD];
  const int tid = threadIdx.x, c = tid & (kD - 1), g = tid >> 7;
  const int lane = tid % kWave, wave = tid / kWave;
  const size_t bn = blockIdx.x;
  const float *rec0 = ws + bn * n_split * (kD + 2);
  float mloc = -INFINITY;
  for (int i = tid; i < n_split; i += 128 * PG) mloc = fmaxf(mloc, rec0[(size_t)i * (kD + 2)]);
  mloc = wave_max(mloc);
  if (lane == 0) red[wave] = mloc;
  __syncthreads();
  float M = red[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) M = fmaxf(M, red[w]);
  for (int i = tid; i < n_split; i += 128 * PG) {
    const float mi = rec0[(size_t)i * (kD + 2)];
    wgt[i] = mi == -INFINITY ? 0.f : exp2f(mi - M);
  }
  __syncthreads();
  const int per = (n_split + PG - 1) / PG;
  const int i0 = g * per, i1 = min(n_split, i0 + per);
  float Lsum = 0.f, A = 0.f;
  int i = i0;
  for (; i + 8 <= i1; i += 8) {
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
  for (; i < i1; ++i) {
    const float *rec = rec0 + (size_t)i * (kD + 2);
    Lsum = fmaf(rec[1], wgt[i], Lsum);
    A = fmaf(rec[2 + c], wgt[i], A);
  }
  if constexpr (PG > 1) {
    part_a[g][c] = A;
    if (c == 0) part_l[g] = Lsum;
    __syncthreads();
    if (g != 0) return;
    A = part_a[0][c];
    Lsum = part_l[0];
#pragma unroll
    for (int k = 1; k < PG; ++k) {
      A += part_a[k][c];
      Lsum += part_l[k];
    }
  }
  E::store1(out, bn * kD + c, A / Lsum);
}

hipError_t launch_decode(const DecodeArgs &a, hipStream_t st) {
  clear_stale_hip_error();
  const int G = a.N_q / a.N_kv;
  // query heads per block of the general kernel: 1, 2, or 4 with the unit's last block partly
  // filled when G is not a multiple of 4 (every block of a unit streams the unit's K and V)
  const int gt = G <= 2 ? G : 4;
  const int groups = (G + gt - 1) / gt;
  hipError_t e;
  if (decode_mq_serves(a))
    e = decode_mq_launch(a, st);
  else if (a.T_v > 0 && a.dtype == THK_BF16)
    e = gt == 4 ? decode_kv_launch_bf16_g4(a, groups, st)
                : gt == 2 ? decode_kv_launch_bf16_g2(a, groups, st) : decode_kv_launch_bf16_g1(a, groups, st);
  else if (a.T_v > 0)
    e = gt == 4 ? decode_kv_launch_f32_g4(a, groups, st)
                : gt == 2 ? decode_kv_launch_f32_g2(a, groups, st) : decode_kv_launch_f32_g1(a, groups, st);
  else if (a.dtype == THK_BF16)
    e = gt == 4 ? decode_launch_bf16_g4(a, groups, st)
                : gt == 2 ? decode_launch_bf16_g2(a, groups, st) : decode_launch_bf16_g1(a, groups, st);
  else
    e = gt == 4 ? decode_launch_f32_g4(a, groups, st)
                : gt == 2 ? decode_launch_f32_g2(a, groups, st) : decode_launch_f32_g1(a, groups, st);
  if (e != hipSuccess) return e;
  if (a.n_split > 1 && a.arrive == nullptr) {
    const int64_t heads = a.units / a.N_kv * a.N_q;
    const bool wide = a.n_split >= 32;   // many splits: four thread groups share them
    if (a.dtype == THK_BF16) {
      if (wide) hipLaunchKernelGGL((k_decode_merge<THK_BF16, 4>), dim3((unsigned)heads), dim3(512), 0, st, a.ws, a.out, a.n_split);
      else hipLaunchKernelGGL((k_decode_merge<THK_BF16, 1>), dim3((unsigned)heads), dim3(128), 0, st, a.ws, a.out, a.n_split);
    } else {
      if (wide) hipLaunchKernelGGL((k_decode_merge<THK_F32, 4>), dim3((unsigned)heads), dim3(512), 0, st, a.ws, a.out, a.n_split);
      else hipLaunchKernelGGL((k_decode_merge<THK_F32, 1>), dim3((unsigned)heads), dim3(128), 0, st, a.ws, a.out, a.n_split);
    }
    e = hipGetLastError();
  }
  return e;
}

}  // namespace thk
