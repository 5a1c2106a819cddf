// Decode kernels over channel-pruned keys AND values, bf16 inputs, 2 query head(s) per block.
#include "thk_decode_impl.h"

namespace thk {
hipError_t decode_kv_launch_bf16_g2(const DecodeArgs &a, int groups, hipStream_t st) {
  return decode_launch_gt<THK_BF16, 2, 1>(a, groups, st);
}
}  // namespace thk
