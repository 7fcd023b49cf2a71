// Internal declarations shared by the HIP translation units of libseka (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "seka.h"

namespace seka {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;

// Per-launch steering parameters passed by value (gains live in kernel arguments so that a
// zero gain can skip work without a device-side lookup).
struct SteerArgs {
  const void* U;        // dev [Hkv, M, D, r]
  const float* w;       // dev [B, Hkv, M] or nullptr
  const uint8_t* mask;  // dev [B, S]
  int M, r;
  float gain[SEKA_MAX_KV_HEADS];
  float kscale[SEKA_MAX_KV_HEADS];   // a of k' = a k + g P k (1 unless Eq. 4's negative-side gain is used)
};

struct AttnArgs {
  const void* Q;
  const void* K;
  const void* V;
  void* O;
  float* lse;  // may be nullptr
  const int* lens;  // dev [B] valid tokens per prompt (clamped to [0, S]), or nullptr for S everywhere
  const int* cu;    // packed layout: dev [B + 1] token offsets (prompt b = tokens [cu[b], cu[b+1]) of `total`), else nullptr
  int total;        // packed layout: tokens in the tensors
  int B, S, Hq, Hkv, D;   // S: tokens per prompt in memory (padded layout) / longest prompt (packed layout)
  float scale;
};

// Launchers (defined one per .hip file).  `steer` may be nullptr for plain attention.
hipError_t launch_attention_f32(const AttnArgs& a, const SteerArgs* steer, hipStream_t s);
hipError_t launch_attention_bf16(const AttnArgs& a, const SteerArgs* steer, hipStream_t s);
hipError_t launch_edit_keys(const void* K_in, void* K_out, int B, int S, int Hkv, int D, int dtype,
                            const SteerArgs& steer, hipStream_t s, const int* cu = nullptr, int total = 0);
size_t route_workspace_bytes(int B, int Hkv, int D, int t0, int t1);
size_t project_route_workspace_bytes(int B, int S, int Hq);
hipError_t launch_project_route(const void* X, const void* W, int E, void* Qout, int B, int S, int Hq, int Hkv,
                                const float* proto, int M, int mode, float tau, float* w_out, void* workspace,
                                hipStream_t s);
hipError_t launch_route(const void* Q, int B, int S, int Hq, int Hkv, int D, int dtype, const float* proto,
                        int M, int t0, int t1, int mode, float tau, float* w_out, void* workspace,
                        hipStream_t s, const int* lens = nullptr, const int* cu = nullptr, int total = 0,
                        int window = 0);

size_t decode_workspace_bytes(int B, int S, int Hq, int Hkv, int D, int dtype);
constexpr size_t kDecodeStaticScratchBytes = (size_t)SEKA_DECODE_STATIC_MAX_BYTES;   // the library-owned buffer
// Device address of the library-owned partial-state buffer on the current device (resolved once per device).
hipError_t decode_static_scratch(void** out);
hipError_t launch_decode(const void* q, const void* K, const void* V, void* O, float* lse, const int* lens, int B, int S,
                         int Hq, int Hkv, int D, int dtype, float scale, void* workspace, hipStream_t s);

size_t learn_workspace_bytes(int Hkv, int D, int n);
hipError_t launch_learn(const void* hn, const void* hs, int n, int Hkv, int D, int dtype, float gamma, float* U_out,
                        float* sigma_out, int* k_out, void* U_packed, int r_pad, void* workspace, hipStream_t s);
hipError_t launch_head_distance(const void* hp, const void* hm, int n, int Hkv, int D, int dtype, float* D_out,
                                void* workspace, hipStream_t s);

// Where prompt b starts (in tokens) and how many tokens it has.  Packed layout: read from cu, clamped so that every
// access derived from them stays inside the tensors whatever cu holds.
__device__ __forceinline__ void prompt_extent(const AttnArgs& a, int b, size_t& tok0, int& len) {
  if (a.cu) {
    const int c0 = min(max(a.cu[b], 0), a.total);
    tok0 = (size_t)c0;
    len = min(max(a.cu[b + 1] - c0, 0), min(a.S, a.total - c0));
  } else {
    tok0 = (size_t)b * a.S;
    len = a.lens ? min(max(a.lens[b], 0), a.S) : a.S;
  }
}
// lse[(b, hq, token i of the prompt)]: [B, Hq, S] in the padded layout, [Hq, total] in the packed one
__device__ __forceinline__ size_t lse_index(const AttnArgs& a, int b, int hq, size_t tok0, int i) {
  return a.cu ? (size_t)hq * a.total + tok0 + i : ((size_t)b * a.Hq + hq) * a.S + i;
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

}  // namespace seka
