// bf16 attention kernels for head dimension 64.
#include <cstring>
#include "attn_bf16_launch.h"
namespace seka {
hipError_t launch_attention_bf16_d64(const AttnArgs& a, const SteerArgs* steer, hipStream_t s) {
  return launch_attention_bf16_d<64>(a, steer, s);
}
}  // namespace seka
