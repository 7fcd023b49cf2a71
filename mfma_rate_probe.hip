// Stand-alone probe (not part of libseka.so): the rate a loop of nothing but v_mfma_f32_32x32x16_bf16 sustains on
// this device, once with constant operands and once with random N(0,1) bf16 operands.  The chip is power-limited:
// with operands that toggle like real data the shader clock settles well below its maximum, so this rate, not the
// published peak, is what a dense bf16 kernel on such data can approach.  Prints one JSON line.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#define PROBE_CHECK(x)                                                                  \
  do {                                                                                  \
    hipError_t e_ = (x);                                                                \
    if (e_ != hipSuccess) {                                                             \
      fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);  \
      return 1;                                                                         \
    }                                                                                   \
  } while (0)

// ops: [16 operand sets][64 lanes][8] bf16 (8 A operands, then 8 B operands), read once into registers.
__global__ __launch_bounds__(512) void mfma_only_kernel(const uint16_t* __restrict__ ops, float* __restrict__ out,
                                                        unsigned long long* __restrict__ clk, int iters) {
  const int lane = threadIdx.x & 63;
  bf16x8 a[8], b[8];
  for (int s = 0; s < 8; ++s) {
    a[s] = *reinterpret_cast<const bf16x8*>(ops + ((size_t)s * 64 + lane) * 8);
    b[s] = *reinterpret_cast<const bf16x8*>(ops + ((size_t)(8 + s) * 64 + lane) * 8);
  }
  f32x16 acc[4];
  for (int k = 0; k < 4; ++k)
    for (int r = 0; r < 16; ++r) acc[k][r] = 0.f;
  const unsigned long long t0 = __builtin_amdgcn_s_memtime();        // shader clock
  const unsigned long long r0 = __builtin_amdgcn_s_memrealtime();    // 100 MHz
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i)
      acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 7], b[(i + (i >> 3)) & 7], acc[i & 3], 0, 0, 0);
    if ((it & 63) == 63) {   // keeps the sums of random products in range
      for (int k = 0; k < 4; ++k)
        for (int r = 0; r < 16; ++r) acc[k][r] *= 0.001f;
    }
  }
  const unsigned long long t1 = __builtin_amdgcn_s_memtime();
  const unsigned long long r1 = __builtin_amdgcn_s_memrealtime();
  float s = 0.f;
  for (int k = 0; k < 4; ++k)
    for (int r = 0; r < 16; ++r) s += acc[k][r];
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    clk[0] = t1 - t0;
    clk[1] = r1 - r0;
  }
}

static uint16_t bf16_bits(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

int main() {
  const int iters = 20000, blocks = 1024, threads = 512, reps = 12;
  float* out = nullptr;
  unsigned long long* clk = nullptr;
  uint16_t* ops = nullptr;
  PROBE_CHECK(hipMalloc(&out, (size_t)blocks * threads * sizeof(float)));
  PROBE_CHECK(hipMalloc(&clk, 2 * sizeof(unsigned long long)));
  PROBE_CHECK(hipMalloc(&ops, 16 * 64 * 8 * sizeof(uint16_t)));
  std::mt19937 rng(1);
  std::normal_distribution<float> nd(0.f, 1.f);
  double tflops[2], mhz[2];
  for (int mode = 0; mode < 2; ++mode) {
    std::vector<uint16_t> h(16 * 64 * 8);
    for (auto& x : h) x = mode == 0 ? bf16_bits(1.0f) : bf16_bits(nd(rng));
    PROBE_CHECK(hipMemcpy(ops, h.data(), h.size() * sizeof(uint16_t), hipMemcpyHostToDevice));
    hipEvent_t e0, e1;
    PROBE_CHECK(hipEventCreate(&e0));
    PROBE_CHECK(hipEventCreate(&e1));
    for (int w = 0; w < 3; ++w) hipLaunchKernelGGL(mfma_only_kernel, dim3(blocks), dim3(threads), 0, 0, ops, out, clk, iters);
    PROBE_CHECK(hipEventRecord(e0));
    for (int w = 0; w < reps; ++w) hipLaunchKernelGGL(mfma_only_kernel, dim3(blocks), dim3(threads), 0, 0, ops, out, clk, iters);
    PROBE_CHECK(hipEventRecord(e1));
    PROBE_CHECK(hipEventSynchronize(e1));
    PROBE_CHECK(hipGetLastError());
    float ms = 0.f;
    PROBE_CHECK(hipEventElapsedTime(&ms, e0, e1));
    unsigned long long hc[2];
    PROBE_CHECK(hipMemcpy(hc, clk, sizeof(hc), hipMemcpyDeviceToHost));
    const double flops = (double)blocks * (threads / 64) * iters * 16.0 * 32768.0 * reps;
    tflops[mode] = flops / (ms * 1e-3) / 1e12;
    mhz[mode] = (double)hc[0] / ((double)hc[1] / 100.0);
  }
  printf("{\"instruction\": \"v_mfma_f32_32x32x16_bf16\", \"constant_operands_tflops\": %.1f, \"constant_operands_mhz\": %.0f, "
         "\"random_operands_tflops\": %.1f, \"random_operands_mhz\": %.0f}\n",
         tflops[0], mhz[0], tflops[1], mhz[1]);
  return 0;
}
