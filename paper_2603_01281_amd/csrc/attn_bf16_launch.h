// Launch-side dispatch of the bf16 attention kernel for one head dimension (instantiated per D in its own
// translation unit so the variants compile in parallel).
#pragma once
#include "attn_bf16_kernel.h"

namespace seka {

template <int D, int HPW, int RB, bool STEER, int VMODE>
hipError_t launch_attention_bf16_cfg(const AttnArgs& a, const SteerArgs* steer, hipStream_t s) {
  constexpr int BQ = 32 * RB;
  const int Rpad = STEER ? (steer->M * steer->r + 31) / 32 * 32 : 0;
  const size_t smem = attention_bf16_smem_bytes(D, VMODE, STEER, Rpad);
  auto kernel = attention_bf16_kernel<D, HPW, RB, STEER, VMODE>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  const int nQB = (a.S + BQ - 1) / BQ;
  const long long blocks = (long long)nQB * (a.Hq / HPW) * a.B;
  if (blocks > 0x7fffffffLL) return hipErrorNotSupported;
  SteerArgs sa;
  if (STEER) sa = *steer; else memset(&sa, 0, sizeof(sa));
  hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(64 * HPW * RB), smem, s, a, sa, Rpad);
  return hipGetLastError();
}

template <int D, bool STEER, int VMODE>
hipError_t launch_attention_bf16_group(const AttnArgs& a, const SteerArgs* steer, hipStream_t s) {
  const int G = a.Hq / a.Hkv;
  if (G % 4 == 0) return launch_attention_bf16_cfg<D, 4, 2, STEER, VMODE>(a, steer, s);
  if (G % 7 == 0) return launch_attention_bf16_cfg<D, 7, 1, STEER, VMODE>(a, steer, s);
  if (G % 2 == 0) return launch_attention_bf16_cfg<D, 2, 4, STEER, VMODE>(a, steer, s);
  return launch_attention_bf16_cfg<D, 1, 8, STEER, VMODE>(a, steer, s);
}

template <int D>
hipError_t launch_attention_bf16_d(const AttnArgs& a, const SteerArgs* steer, int variant, hipStream_t s) {
  const bool tr = (variant == 0);
  if (steer) return tr ? launch_attention_bf16_group<D, true, 0>(a, steer, s) : launch_attention_bf16_group<D, true, 1>(a, steer, s);
  return tr ? launch_attention_bf16_group<D, false, 0>(a, steer, s) : launch_attention_bf16_group<D, false, 1>(a, steer, s);
}

hipError_t launch_attention_bf16_d128(const AttnArgs& a, const SteerArgs* steer, int variant, hipStream_t s);
hipError_t launch_attention_bf16_d64(const AttnArgs& a, const SteerArgs* steer, int variant, hipStream_t s);

}  // namespace seka
