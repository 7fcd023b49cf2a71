// Launch-side dispatch of the software-pipelined bf16 attention kernel (head dimension 128).  The plain kernels
// and the steered kernels of each compile-time rank are instantiated in translation units of their own.
#pragma once
#include <cstring>

#include "attn_bf16_pipe_kernel.h"

namespace seka {

template <int HPW, int RBW, bool STEER, int NKR>
hipError_t launch_attention_bf16_pipe_cfg(const AttnArgs& a, const SteerArgs* steer, hipStream_t s) {
  constexpr int BQ = 32 * RBW;
  const size_t smem = attention_bf16_pipe_smem_bytes(a.S, STEER, NKR, HPW * RBW);
  if (smem > 160 * 1024) return hipErrorNotSupported;
  auto kernel = attention_bf16_pipe_kernel<HPW, RBW, 1, STEER, NKR>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  const int nQB = (a.S + BQ - 1) / BQ;
  const long long blocks = (long long)((nQB + 1) / 2) * (a.Hq / HPW) * a.B;     // two blocks of query rows per workgroup
  if (blocks > 0x7fffffffLL) return hipErrorNotSupported;
  SteerArgs sa;
  if (STEER) sa = *steer; else memset(&sa, 0, sizeof(sa));
  hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(64 * HPW * RBW), smem, s, a, sa);
  return hipGetLastError();
}

// Compute units of the current device (256 on MI355X), asked once.
inline int pipe_compute_units() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
      n = 256;
    cus = n;
  }
  return cus;
}

// Workgroup shape by GQA group size: HPW query heads of one KV head x RBW blocks of 32 query rows.
template <bool STEER, int NKR>
hipError_t launch_attention_bf16_pipe_group(const AttnArgs& a, const SteerArgs* steer, hipStream_t s) {
  const int G = a.Hq / a.Hkv;
  if (G % 4 == 0) return launch_attention_bf16_pipe_cfg<4, 2, STEER, NKR>(a, steer, s);
  if (G % 7 == 0) {
    // Seven heads x 32 rows gives many small workgroups, each of which repeats the edit of every highlighted
    // tile; 256 rows of one or two heads per workgroup is faster (Hq=28, Hkv=4: +5 % plain, +8 % steered at
    // S=32768) once its grid still fills the chip several times over, and slower below that.
    const int hpw = G % 2 == 0 ? 2 : 1, bq = 256 / hpw;    // the shape the group falls to below
    const long long big = (long long)(((a.S + bq - 1) / bq + 1) / 2) * (a.Hq / hpw) * a.B;
    if (big < 6LL * pipe_compute_units()) return launch_attention_bf16_pipe_cfg<7, 1, STEER, NKR>(a, steer, s);
  }
  if (G % 2 == 0) return launch_attention_bf16_pipe_cfg<2, 4, STEER, NKR>(a, steer, s);
  return launch_attention_bf16_pipe_cfg<1, 8, STEER, NKR>(a, steer, s);
}

}  // namespace seka
