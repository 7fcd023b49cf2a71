// Top-level dispatch of the bf16 attention path.
#include <cstring>
#include "attn_bf16_launch.h"
namespace seka {
bool attention_bf16_variant_ok(int variant) {
#ifdef SEKA_TUNING_VARIANTS
  return variant >= 0 && variant < kNumAttnVariants;
#else
  return variant == 0;
#endif
}
hipError_t launch_attention_bf16(const AttnArgs& a, const SteerArgs* steer, int variant, hipStream_t s) {
  return a.D == 128 ? launch_attention_bf16_d128(a, steer, variant, s) : launch_attention_bf16_d64(a, steer, variant, s);
}
}  // namespace seka
