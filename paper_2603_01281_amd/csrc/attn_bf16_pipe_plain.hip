// Software-pipelined bf16 attention, head dimension 128: unsteered kernels.
#include "attn_bf16_pipe_launch.h"
namespace seka {
hipError_t launch_attention_bf16_pipe_plain(const AttnArgs& a, hipStream_t s) {
  return launch_attention_bf16_pipe_group<false, 1>(a, nullptr, s);
}
}  // namespace seka
