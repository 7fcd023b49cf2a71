// Software-pipelined bf16 attention, head dimension 128: steered kernels for a concatenated rank of at most 128.
#include "attn_bf16_pipe_launch.h"
namespace seka {
hipError_t launch_attention_bf16_pipe_r128(const AttnArgs& a, const SteerArgs* steer, hipStream_t s) {
  return launch_attention_bf16_pipe_group<true, 4>(a, steer, s);
}
}  // namespace seka
