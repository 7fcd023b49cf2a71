// Top-level dispatch of the bf16 attention path.
#include <cstring>
#include "attn_bf16_launch.h"
namespace seka {
hipError_t launch_attention_bf16(const AttnArgs& a, const SteerArgs* steer, hipStream_t s) {
  return a.D == 128 ? launch_attention_bf16_d128(a, steer, s) : launch_attention_bf16_d64(a, steer, s);
}
}  // namespace seka
