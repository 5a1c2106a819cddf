// Plain memory streams for benchmarks: what the chip gives a kernel that does nothing but read,
// copy or write the bytes of a prune or decode call -- the ceiling those calls are measured
// against at the call's own size (a launch of a few hundred MB pays its start and its end, so
// the rate of a long stream is not its ceiling).  Not part of the method.  gfx950, wave64.
//
// A block of 256 threads owns 128 KiB of the source (32 chunks of 16 bytes per thread, all
// loads in flight at once, non-temporal like the library's own streams) and w x 4 KiB of the
// destination (w chunks per thread, non-temporal stores):
//   read   the chunks are folded into one value that the compiler must produce; nothing is stored
//   copy   the block keeps its 32 chunks in registers and then stores the first w of them -- the
//          traffic of a prune block (w / 32 = T / 128) without any exchange between blocks
//   write  w chunks per thread of a constant
#include "thk_internal.h"

namespace thk {
namespace {

constexpr int kProbeChunks = 32;   // 16-byte chunks per thread = 128 KiB per block

// The value has to exist in registers here: the loads it was folded from cannot be dropped.
__device__ __forceinline__ void keep_alive(const u32x4 &x) {
  asm volatile("" ::"v"(x.x), "v"(x.y), "v"(x.z), "v"(x.w));
}

template <int MODE>   // 0 read, 1 copy, 2 write
__global__ __launch_bounds__(256) void k_bench_stream(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int w) {
  const size_t b = blockIdx.x;
  u32x4 r[kProbeChunks];
  if constexpr (MODE != 2) {
    const u32x4 *p = src + b * (kProbeChunks * 256) + threadIdx.x;
#pragma unroll
    for (int j = 0; j < kProbeChunks; ++j) r[j] = ld_stream(p + j * 256);
  }
  if constexpr (MODE == 0) {
    u32x4 x = r[0];
#pragma unroll
    for (int j = 1; j < kProbeChunks; ++j) x ^= r[j];
    keep_alive(x);
  } else {
    u32x4 *q = dst + b * ((size_t)w * 256) + threadIdx.x;
    if constexpr (MODE == 1) {
      // every chunk is really read, also those that are not written (a prune block reads whole
      // rows): they are folded into a value the compiler must produce
      u32x4 x = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int j = 0; j < kProbeChunks; ++j) x ^= r[j];
      keep_alive(x);
    }
#pragma unroll
    for (int j = 0; j < kProbeChunks; ++j) {
      if (j < w) {   // uniform
        const u32x4 fill = {(uint32_t)b, (uint32_t)j, 0x74686bu, threadIdx.x};
        st_stream(q + j * 256, MODE == 1 ? r[j] : fill);
      }
    }
  }
}

}  // namespace

hipError_t launch_bench_stream(int mode, const void *src, void *dst, int64_t n_blocks, int w, hipStream_t st) {
  const dim3 grid((unsigned)n_blocks), block(256);
  const u32x4 *s = (const u32x4 *)src;
  u32x4 *d = (u32x4 *)dst;
  void *kargs[] = {(void *)&s, (void *)&d, (void *)&w};
  const void *fn = mode == 0 ? (const void *)k_bench_stream<0>
                             : mode == 1 ? (const void *)k_bench_stream<1> : (const void *)k_bench_stream<2>;
  const hipError_t e = launch_main_kernel(fn, grid, block, kargs, 0, st);
  return e != hipSuccess ? e : hipGetLastError();
}

}  // namespace thk
