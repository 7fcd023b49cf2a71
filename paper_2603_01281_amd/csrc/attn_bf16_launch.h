// Launch-side dispatch of the bf16 attention kernels for one head dimension (instantiated per D in its own
// translation unit so that the instantiations compile in parallel).
#pragma once
#include <cstring>
#include "attn_bf16_kernel.h"

namespace seka {

constexpr int kAttnVPad = 32;    // row padding of the register-staged kernel's V tile (elements)

template <int D, int HPW, int RB, bool STEER>
hipError_t launch_attention_bf16_cfg(const AttnArgs& a, const SteerArgs* steer, hipStream_t s) {
  constexpr int BQ = 32 * RB;
  const int Rpad = STEER ? (steer->M * steer->r + 31) / 32 * 32 : 0;
  const size_t smem = attention_bf16_smem_bytes(D, kAttnVPad, STEER, Rpad, 64 * HPW * RB);
  auto kernel = attention_bf16_kernel<D, HPW, RB, STEER, kAttnVPad>;
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

// software-pipelined direct-to-LDS kernels (head dimension 128 only; defined in attn_bf16_pipe_*.hip)
hipError_t launch_attention_bf16_pipe_plain(const AttnArgs& a, hipStream_t s);
hipError_t launch_attention_bf16_pipe_r32(const AttnArgs& a, const SteerArgs* steer, hipStream_t s);
hipError_t launch_attention_bf16_pipe_r64(const AttnArgs& a, const SteerArgs* steer, hipStream_t s);
hipError_t launch_attention_bf16_pipe_r128(const AttnArgs& a, const SteerArgs* steer, hipStream_t s);

inline hipError_t launch_attention_bf16_pipe(const AttnArgs& a, const SteerArgs* steer, hipStream_t s) {
  if (!steer) return launch_attention_bf16_pipe_plain(a, s);
  const int R = steer->M * steer->r;
  // The rank <= 32 kernel applies the edit to the scores and has no place for a key scale other than 1 (Eq. 4's
  // negative-side gain): such calls take the dense form, which edits the keys themselves.
  bool unit_scale = true;
  for (int h = 0; h < a.Hkv; ++h) unit_scale = unit_scale && (steer->gain[h] == 0.f || steer->kscale[h] == 1.f);
  if (R <= 32 && unit_scale) return launch_attention_bf16_pipe_r32(a, steer, s);
  if (R <= 64) return launch_attention_bf16_pipe_r64(a, steer, s);
  return launch_attention_bf16_pipe_r128(a, steer, s);
}

template <int D, bool STEER>
hipError_t launch_attention_bf16_group(const AttnArgs& a, const SteerArgs* steer, hipStream_t s) {
  const int G = a.Hq / a.Hkv;
  if (G % 4 == 0) return launch_attention_bf16_cfg<D, 4, 2, STEER>(a, steer, s);
  if (G % 7 == 0) return launch_attention_bf16_cfg<D, 7, 1, STEER>(a, steer, s);
  if (G % 2 == 0) return launch_attention_bf16_cfg<D, 2, 4, STEER>(a, steer, s);
  return launch_attention_bf16_cfg<D, 1, 8, STEER>(a, steer, s);
}

template <int D, bool STEER>
hipError_t launch_attention_bf16_any(const AttnArgs& a, const SteerArgs* steer, hipStream_t s) {
  if (D == 128) {
    const hipError_t e = launch_attention_bf16_pipe(a, steer, s);
    if (e != hipErrorNotSupported) return e;     // highlight bitmap too large for LDS at this S: register-staged kernel
  }
  return launch_attention_bf16_group<D, STEER>(a, steer, s);
}

template <int D>
hipError_t launch_attention_bf16_d(const AttnArgs& a, const SteerArgs* steer, hipStream_t s) {
  return steer ? launch_attention_bf16_any<D, true>(a, steer, s) : launch_attention_bf16_any<D, false>(a, steer, s);
}

hipError_t launch_attention_bf16_d128(const AttnArgs& a, const SteerArgs* steer, hipStream_t s);
hipError_t launch_attention_bf16_d64(const AttnArgs& a, const SteerArgs* steer, hipStream_t s);

}  // namespace seka
