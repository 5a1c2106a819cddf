// Decode kernels over channel-pruned keys AND values, f32 inputs, 4 query head(s) per block.
#include "thk_decode_impl.h"

namespace thk {
hipError_t decode_kv_launch_f32_g4(const DecodeArgs &a, int groups, hipStream_t st) {
  return decode_launch_gt<THK_F32, 4, 1>(a, groups, st);
}
}  // namespace thk
