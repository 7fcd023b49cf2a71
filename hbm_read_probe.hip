// Stand-alone probe (not part of libseka.so): how fast this device reads a key/value cache of a given shape when a
// kernel does nothing else.  The generation step and the stand-alone key edit move 17 MB to 134 MB per call at the
// benchmark configurations; at those sizes launch, ramp-up and the tail of the last workgroups are a large share
// of the call, so the published 8 TB/s is not what such a call can reach.  This probe gives the reference: the
// time of a kernel that only loads the same bytes (xor-reduced so that the loads are not removed), once with the
// access pattern of the generation step (a workgroup per (token range, KV head, prompt) reads 256-byte rows at a
// stride of Hkv * D * 2 bytes) and once as one linear stream, every call on buffers that are not in any cache
// (rotated over > 1.5 GB).  Usage: hbm_read_probe.bin B S Hkv [splits]; D = 128, bf16.  Prints one JSON line.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <vector>

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

#define PROBE_CHECK(x)                                                                  \
  do {                                                                                  \
    hipError_t e_ = (x);                                                                \
    if (e_ != hipSuccess) {                                                             \
      fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);  \
      return 1;                                                                         \
    }                                                                                   \
  } while (0)

constexpr int kD = 128, kThreads = 256, kBlockRows = 32;

// grid (splits, Hkv, B): the workgroup's four waves take the 32-row blocks of its token range in turn; a lane
// loads 16 bytes of 8 rows of K and of V per block (rows clamped into the range).
__global__ __launch_bounds__(kThreads) void read_rows_kernel(const unsigned short* __restrict__ K,
                                                             const unsigned short* __restrict__ V, int S, int Hkv,
                                                             int splits, unsigned* __restrict__ out) {
  const int b = blockIdx.z, h = blockIdx.y, split = blockIdx.x;
  const int per = (S + splits - 1) / splits, k0 = split * per, k1 = min(S, k0 + per);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const size_t rowstride = (size_t)Hkv * kD;
  const unsigned short* Kb = K + ((size_t)b * S * Hkv + h) * kD;
  const unsigned short* Vb = V + ((size_t)b * S * Hkv + h) * kD;
  u32x4 acc = {0, 0, 0, 0};
  for (int kb = k0 + wave * kBlockRows; kb < k1; kb += 4 * kBlockRows) {
    u32x4 r[16];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const size_t rv = (size_t)min(kb + 4 * i + lane / 16, k1 - 1) * rowstride + 8 * (lane % 16);
      r[i] = *reinterpret_cast<const u32x4*>(Kb + rv);
      r[8 + i] = *reinterpret_cast<const u32x4*>(Vb + rv);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) acc ^= r[i];
  }
  const unsigned v = acc.x ^ acc.y ^ acc.z ^ acc.w;
  if (v == 0x12345678u) out[0] = v;        // (keeps the loads alive; the buffers hold other values)
}

// grid (n): workgroup w reads elements [w * per, (w + 1) * per) of both buffers, per a multiple of 16384
__global__ __launch_bounds__(kThreads) void read_linear_kernel(const unsigned short* __restrict__ K,
                                                               const unsigned short* __restrict__ V, size_t per,
                                                               unsigned* __restrict__ out) {
  const unsigned short* Kb = K + (size_t)blockIdx.x * per;
  const unsigned short* Vb = V + (size_t)blockIdx.x * per;
  u32x4 acc = {0, 0, 0, 0};
  for (size_t o = 0; o < per; o += (size_t)kThreads * 64) {
    u32x4 r[16];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      r[i] = *reinterpret_cast<const u32x4*>(Kb + o + (size_t)(i * kThreads + threadIdx.x) * 8);
      r[8 + i] = *reinterpret_cast<const u32x4*>(Vb + o + (size_t)(i * kThreads + threadIdx.x) * 8);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) acc ^= r[i];
  }
  const unsigned v = acc.x ^ acc.y ^ acc.z ^ acc.w;
  if (v == 0x12345678u) out[0] = v;
}

int main(int argc, char** argv) {
  if (argc < 4) {
    fprintf(stderr, "usage: %s B S Hkv [splits]\n", argv[0]);
    return 2;
  }
  const int B = atoi(argv[1]), S = atoi(argv[2]), Hkv = atoi(argv[3]);
  if (B < 1 || B > 65535 || S < 1 || Hkv < 1 || Hkv > 65535 || (size_t)B * S * Hkv * kD > ((size_t)1 << 31)) {
    fprintf(stderr, "shape out of range\n");
    return 2;
  }
  int splits = argc > 4 ? atoi(argv[4]) : std::max(1, std::min(64, std::min(S / 512, (4096 + B * Hkv - 1) / (B * Hkv))));
  if (splits < 1 || splits > 65535) return 2;
  const size_t elems = (size_t)B * S * Hkv * kD, bytes = elems * 2;
  // linear pattern: whole chunks of 16384 elements per workgroup; the remainder (< one chunk per workgroup) is
  // left unread and the byte count says so
  const size_t chunk = (size_t)kThreads * 64;
  int nwg = 2048;
  while (nwg > 1 && elems / nwg < chunk) nwg /= 2;
  const size_t per = elems / nwg / chunk * chunk;
  if (per == 0) {
    fprintf(stderr, "tensor smaller than one chunk\n");
    return 2;
  }
  const int nrot = (int)std::max<size_t>(2, (size_t)1600000000 / (2 * bytes) + 1);
  std::vector<unsigned short*> Ks(nrot), Vs(nrot);
  for (int i = 0; i < nrot; ++i) {
    PROBE_CHECK(hipMalloc(&Ks[i], bytes));
    PROBE_CHECK(hipMalloc(&Vs[i], bytes));
    PROBE_CHECK(hipMemset(Ks[i], 1 + i % 200, bytes));
    PROBE_CHECK(hipMemset(Vs[i], 7 + i % 200, bytes));
  }
  unsigned* out;
  PROBE_CHECK(hipMalloc(&out, 4));
  hipEvent_t e0, e1;
  PROBE_CHECK(hipEventCreate(&e0));
  PROBE_CHECK(hipEventCreate(&e1));
  float med[2] = {0.f, 0.f};
  for (int mode = 0; mode < 2; ++mode) {
    auto launch = [&](int i) {
      if (mode == 0)
        hipLaunchKernelGGL(read_rows_kernel, dim3(splits, Hkv, B), dim3(kThreads), 0, 0, Ks[i], Vs[i], S, Hkv, splits, out);
      else
        hipLaunchKernelGGL(read_linear_kernel, dim3(nwg), dim3(kThreads), 0, 0, Ks[i], Vs[i], per, out);
    };
    for (int i = 0; i < nrot; ++i) launch(i);
    PROBE_CHECK(hipDeviceSynchronize());
    std::vector<float> ts;
    const int reps = std::max(3 * nrot, 9);
    for (int r = 0; r < reps; ++r) {
      PROBE_CHECK(hipEventRecord(e0, 0));
      launch(r % nrot);
      PROBE_CHECK(hipEventRecord(e1, 0));
      PROBE_CHECK(hipEventSynchronize(e1));
      float ms = 0.f;
      PROBE_CHECK(hipEventElapsedTime(&ms, e0, e1));
      ts.push_back(ms);
    }
    PROBE_CHECK(hipGetLastError());
    std::sort(ts.begin(), ts.end());
    med[mode] = ts[ts.size() / 2];
  }
  const double rows_bytes = 2.0 * bytes, lin_bytes = 2.0 * (double)per * nwg * 2;
  printf("{\"B\": %d, \"S\": %d, \"Hkv\": %d, \"D\": %d, \"bytes\": %.0f, \"buffer_pairs\": %d, \"splits\": %d, "
         "\"rows_per_head_us\": %.2f, \"rows_per_head_GBps\": %.0f, \"linear_us\": %.2f, \"linear_GBps\": %.0f}\n",
         B, S, Hkv, kD, rows_bytes, nrot, splits, med[0] * 1e3, rows_bytes / med[0] / 1e6, med[1] * 1e3,
         lin_bytes / med[1] / 1e6);
  for (int i = 0; i < nrot; ++i) {
    (void)hipFree(Ks[i]);
    (void)hipFree(Vs[i]);
  }
  (void)hipFree(out);
  return 0;
}
