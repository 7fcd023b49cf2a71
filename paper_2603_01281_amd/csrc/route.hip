// seka_route: AdaSEKA expert coefficients (paper Sec. 3.3, Eq. 6; benchmark rule softmax of cosines).
//
// HBM-bound: one pass over Q[B, t0:t1, Hq, D].  Stage 1 splits the token range of every
// (batch, KV head) into chunks so that the launch has enough workgroups to fill 256 CUs; each
// workgroup streams its chunk with 16-byte loads (the G query heads of a KV head are contiguous,
// so a token contributes one contiguous G*D run) and writes D fp32 partial sums to the
// workspace.  Stage 2 (one small workgroup per (batch, KV head)) adds the partials in a fixed
// order, so the result is deterministic, then forms the M alignments and normalises them.
#include "common.h"

namespace seka {

namespace {

constexpr int kRouteThreads = 256;
constexpr int kMaxChunks = 256;
constexpr int kFinishThreads = 512;

// Chunks per (batch, KV head): enough workgroups for the whole chip (about 2048) even when B * Hkv is small,
// at least 32 tokens per chunk, at most kMaxChunks partial sums for the second stage to add.
__host__ __device__ inline int route_chunks(int T, int BH) {
  int want = (2048 + BH - 1) / BH;
  if (want < 16) want = 16;
  if (want > kMaxChunks) want = kMaxChunks;
  int c = (T + 31) / 32;
  return c < 1 ? 1 : (c > want ? want : c);
}

template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  __device__ static void load(const float* p, float (&out)[4]) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
  }
};
template <> struct Vec16<uint16_t> {
  static constexpr int N = 8;
  __device__ static void load(const uint16_t* p, float (&out)[8]) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[2 * i] = __uint_as_float(w[i] << 16);
      out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};

// grid = (chunks, B*Hkv); workspace[(bh*chunks + c)*D + d] = sum over the chunk's tokens and the G heads.
template <typename T, int D>
__global__ __launch_bounds__(kRouteThreads) void route_partial_kernel(const T* __restrict__ Q, int S, int Hq, int Hkv,
                                                                       int t0, int t1, int chunks,
                                                                       const int* __restrict__ lens,
                                                                       const int* __restrict__ cu, int total, int window,
                                                                       float* __restrict__ workspace) {
  constexpr int VE = Vec16<T>::N;
  constexpr int VPR = D / VE;                    // 16-byte vectors per (token, head) row
  constexpr int RPP = kRouteThreads / VPR;       // rows per pass
  __shared__ float red[RPP][D];
  const int G = Hq / Hkv;
  const int bh = blockIdx.y, b = bh / Hkv, h = bh % Hkv;
  const int c = blockIdx.x;
  size_t row_base = (size_t)b * S;               // first token row of the prompt
  if (lens != nullptr || cu != nullptr) {        // per-prompt range: the last `window` tokens of the prompt
    int len;
    if (cu != nullptr) {
      const int start = min(max(cu[b], 0), total);
      len = min(cu[b + 1] - start, total - start);
      row_base = (size_t)start;
    } else {
      len = lens[b];
    }
    len = min(max(len, 0), S);
    t1 = len;
    t0 = max(0, len - window);
  }
  const int T_total = t1 - t0;
  const int per = (T_total + chunks - 1) / chunks;
  const int ta = t0 + c * per;
  const int tb = min(t1, ta + per);
  const int col = threadIdx.x % VPR, lane_row = threadIdx.x / VPR;
  float acc[VE];
#pragma unroll
  for (int i = 0; i < VE; ++i) acc[i] = 0.f;
  const int nrows = max(0, tb - ta) * G;
  // four independent 16-byte loads per thread and turn keep enough bytes in flight
  for (int row0 = lane_row; row0 < nrows; row0 += 4 * RPP) {
    float v[4][VE];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int row = row0 + u * RPP;
      if (row < nrows) {
        const int t = ta + row / G, g = row % G;
        Vec16<T>::load(Q + ((row_base + t) * Hq + (size_t)h * G + g) * D + col * VE, v[u]);
      } else {
#pragma unroll
        for (int i = 0; i < VE; ++i) v[u][i] = 0.f;
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int i = 0; i < VE; ++i) acc[i] += v[u][i];
  }
#pragma unroll
  for (int i = 0; i < VE; ++i) red[lane_row][col * VE + i] = acc[i];
  __syncthreads();
  if (threadIdx.x < D) {
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < RPP; ++r) s += red[r][threadIdx.x];
    workspace[((size_t)bh * chunks + c) * D + threadIdx.x] = s;
  }
}

// grid = B*Hkv, block = kFinishThreads: thread (j, d) adds the partials of chunks j, j + NJ, ... in that order, then
// the NJ sums are added in index order: a fixed order, whatever the launch.
template <int D>
__global__ __launch_bounds__(kFinishThreads) void route_finish_kernel(const float* __restrict__ workspace, int chunks, float inv_count,
                                                           const float* __restrict__ proto, int Hkv, int M, int mode,
                                                           float tau, const int* __restrict__ lens, const int* __restrict__ cu,
                                                           int total, int S, int window, int G, float* __restrict__ w_out) {
  __shared__ float qbar[D];
  __shared__ float dots[SEKA_MAX_EXPERTS];
  __shared__ float pnorm2[SEKA_MAX_EXPERTS];
  constexpr int NJ = kFinishThreads / D;
  __shared__ float part[NJ][D];
  const int bh = blockIdx.x, h = bh % Hkv;
  if (lens != nullptr || cu != nullptr) {        // tokens this prompt contributed (the partial kernel's range)
    const int b = bh / Hkv;
    int len;
    if (cu != nullptr) {
      const int start = min(max(cu[b], 0), total);
      len = min(cu[b + 1] - start, total - start);
    } else {
      len = lens[b];
    }
    len = min(max(len, 0), S);
    const int count = (len - max(0, len - window)) * G;
    inv_count = count > 0 ? 1.0f / (float)count : 0.f;
  }
  {
    const int d = threadIdx.x % D, j = threadIdx.x / D;
    float s = 0.f;
    for (int c = j; c < chunks; c += NJ) s += workspace[((size_t)bh * chunks + c) * D + d];
    part[j][d] = s;
  }
  __syncthreads();
  if (threadIdx.x < D) {
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < NJ; ++j) s += part[j][threadIdx.x];
    qbar[threadIdx.x] = s * inv_count;
  }
  __syncthreads();
  if (threadIdx.x < M) {
    const float* p = proto + ((size_t)h * M + threadIdx.x) * D;
    float d = 0.f, n2 = 0.f;
    for (int i = 0; i < D; ++i) {
      d += qbar[i] * p[i];
      n2 += p[i] * p[i];
    }
    dots[threadIdx.x] = d;
    pnorm2[threadIdx.x] = n2;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float* out = w_out + (size_t)bh * M;
    if (mode == SEKA_ROUTE_SOFTMAX_COS) {
      float q2 = 0.f;
      for (int i = 0; i < D; ++i) q2 += qbar[i] * qbar[i];
      const float qn = sqrtf(q2);
      float z[SEKA_MAX_EXPERTS];
      float zmax = -INFINITY;
      for (int m = 0; m < M; ++m) {
        const float nn = qn * sqrtf(pnorm2[m]);
        const float c = nn >= 1e-30f ? dots[m] / nn : 0.f;
        z[m] = tau * c;
        zmax = fmaxf(zmax, z[m]);
      }
      float den = 0.f;
      for (int m = 0; m < M; ++m) {
        z[m] = expf(z[m] - zmax);
        den += z[m];
      }
      for (int m = 0; m < M; ++m) out[m] = z[m] / den;
    } else {
      float big = 0.f;
      for (int m = 0; m < M; ++m) big = fmaxf(big, fabsf(dots[m]));
      for (int m = 0; m < M; ++m) out[m] = big >= 1e-30f ? dots[m] / big : 0.f;
    }
  }
}

}  // namespace

size_t route_workspace_bytes(int B, int Hkv, int D, int t0, int t1) {
  return (size_t)B * Hkv * route_chunks(t1 - t0, B * Hkv) * D * sizeof(float);
}

hipError_t launch_route(const void* Q, int B, int S, int Hq, int Hkv, int D, int dtype, const float* proto, int M,
                        int t0, int t1, int mode, float tau, float* w_out, void* workspace, hipStream_t s,
                        const int* lens, const int* cu, int total, int window) {
  const bool ragged = lens != nullptr || cu != nullptr;
  if (ragged) { t0 = 0; t1 = window < S ? window : S; }      // the longest range a prompt can have
  const int chunks = route_chunks(t1 - t0, B * Hkv);
  const dim3 grid(chunks, B * Hkv);
  float* ws = static_cast<float*>(workspace);
  const float inv_count = 1.0f / ((float)(t1 - t0) * (float)(Hq / Hkv));
#define SEKA_ROUTE_CASE(T, DD)                                                                                       \
  do {                                                                                                               \
    hipLaunchKernelGGL((route_partial_kernel<T, DD>), grid, dim3(kRouteThreads), 0, s, static_cast<const T*>(Q), S,  \
                       Hq, Hkv, t0, t1, chunks, lens, cu, total, window, ws);                                        \
    hipLaunchKernelGGL((route_finish_kernel<DD>), dim3(B * Hkv), dim3(kFinishThreads), 0, s, ws, chunks, inv_count, proto, Hkv, \
                       M, mode, tau, lens, cu, total, S, window, Hq / Hkv, w_out);                                   \
  } while (0)
  if (dtype == SEKA_BF16) {
    if (D == 128) SEKA_ROUTE_CASE(uint16_t, 128); else SEKA_ROUTE_CASE(uint16_t, 64);
  } else {
    if (D == 128) SEKA_ROUTE_CASE(float, 128); else SEKA_ROUTE_CASE(float, 64);
  }
#undef SEKA_ROUTE_CASE
  return hipGetLastError();
}

}  // namespace seka
