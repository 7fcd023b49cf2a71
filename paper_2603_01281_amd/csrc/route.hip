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


// ---- query projection with the routing sums in its epilogue (Sec. 3.3: the routing query is a by-product of the
// projection that produces Q, so it need not be read back) ----
//
// Q[t, n] = sum_e X[t, e] W[n, e]  (bf16 in, fp32 accumulate, bf16 out; W is the projection weight with one row per
// output feature, the layout of a linear layer).  One workgroup = 128 tokens x 128 output features (one head at
// D = 128), four waves of 64 x 64, v_mfma_f32_32x32x16_bf16; 64-wide slices of E go through two LDS stages, the
// next slice's global loads are in flight while the current one is multiplied.  ROUTE: every wave also sums the
// rounded outputs of its 64 tokens per feature and writes them as one partial sum of seka_route's first stage, so
// route_finish_kernel completes the routing without a pass over Q.
constexpr int kProjTile = 128, kProjK = 64, kProjLd = kProjK + 8;     // LDS row stride in elements (144 bytes: conflict-free 16-byte reads)

template <bool ROUTE>
__global__ __launch_bounds__(256) void project_route_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ W,
                                                            uint16_t* __restrict__ Qout, int E, int N, int S, int G,
                                                            int Hkv, float* __restrict__ workspace) {
  __shared__ __attribute__((aligned(16))) uint16_t lds[2 * 2 * kProjTile * kProjLd];   // [stage][A | B][128][72]; reused for the output tile
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, hf = lane >> 5;
  const size_t row0 = (size_t)blockIdx.y * kProjTile;     // first token of the tile (B*S is a multiple of 128)
  const int col0 = blockIdx.x * kProjTile;                // first output feature
  // global -> registers: thread t takes 64 contiguous bytes of row t / 2 of both operand tiles
  const int lrow = tid >> 1, lhalf = tid & 1;
  const uint16_t* xa = X + (row0 + lrow) * (size_t)E + 32 * lhalf;
  const uint16_t* wb = W + ((size_t)col0 + lrow) * (size_t)E + 32 * lhalf;
  // Two register sets: a slice is requested two turns before it is multiplied (one turn in flight, written to
  // LDS at the end of the next), so a turn of 16 MFMAs per wave does not have to cover the whole memory latency.
  typedef unsigned int proj_u32x4 __attribute__((ext_vector_type(4)));
  struct Slice { proj_u32x4 a0, a1, a2, a3, b0, b1, b2, b3; };
  Slice r0, r1;
#define SEKA_PROJ_GLOAD(r, kt)                                                                \
  {                                                                                           \
    const int kt_ = (kt) < nk ? (kt) : nk - 1;            /* past the end: a slice nobody uses */ \
    const proj_u32x4* pa_ = reinterpret_cast<const proj_u32x4*>(xa + (size_t)kt_ * kProjK);   \
    const proj_u32x4* pb_ = reinterpret_cast<const proj_u32x4*>(wb + (size_t)kt_ * kProjK);   \
    r.a0 = pa_[0]; r.a1 = pa_[1]; r.a2 = pa_[2]; r.a3 = pa_[3];                               \
    r.b0 = pb_[0]; r.b1 = pb_[1]; r.b2 = pb_[2]; r.b3 = pb_[3];                               \
  }
#define SEKA_PROJ_LSTORE(r, stage)                                                            \
  {                                                                                           \
    proj_u32x4* A_ = reinterpret_cast<proj_u32x4*>(lds + (stage) * (2 * kProjTile * kProjLd) + lrow * kProjLd + 32 * lhalf); \
    proj_u32x4* B_ = reinterpret_cast<proj_u32x4*>(lds + (stage) * (2 * kProjTile * kProjLd) + kProjTile * kProjLd + lrow * kProjLd + 32 * lhalf); \
    A_[0] = r.a0; A_[1] = r.a1; A_[2] = r.a2; A_[3] = r.a3;                                   \
    B_[0] = r.b0; B_[1] = r.b1; B_[2] = r.b2; B_[3] = r.b3;                                   \
  }
  // Tokens are the MFMA's rows and features its columns, so that a lane owns one feature column and its 16
  // registers are 16 tokens: the routing sum over tokens is a sum over registers.
#define SEKA_PROJ_COMPUTE(stage)                                                              \
  {                                                                                           \
    const uint16_t* A_ = lds + (stage) * (2 * kProjTile * kProjLd);                           \
    const uint16_t* B_ = A_ + kProjTile * kProjLd;                                            \
    _Pragma("unroll") for (int ks = 0; ks < kProjK / 16; ++ks) {                              \
      bf16x8 a_[2], b_[2];                                                                    \
      _Pragma("unroll") for (int i = 0; i < 2; ++i)                                           \
        a_[i] = *reinterpret_cast<const bf16x8*>(A_ + (64 * wm + 32 * i + l32) * kProjLd + 16 * ks + 8 * hf); \
      _Pragma("unroll") for (int j = 0; j < 2; ++j)                                           \
        b_[j] = *reinterpret_cast<const bf16x8*>(B_ + (64 * wn + 32 * j + l32) * kProjLd + 16 * ks + 8 * hf); \
      _Pragma("unroll") for (int i = 0; i < 2; ++i)                                           \
        _Pragma("unroll") for (int j = 0; j < 2; ++j)                                         \
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_[i], b_[j], acc[i][j], 0, 0, 0); \
    }                                                                                         \
  }
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  const int nk = E / kProjK;
  SEKA_PROJ_GLOAD(r0, 0)
  SEKA_PROJ_LSTORE(r0, 0)
  __syncthreads();
  SEKA_PROJ_GLOAD(r0, 1)
  int kt = 0;
  for (; kt + 1 < nk; kt += 2) {
    // even turn: stage 0 holds slice kt, set 0 holds slice kt + 1
    SEKA_PROJ_GLOAD(r1, kt + 2)
    SEKA_PROJ_COMPUTE(0)
    SEKA_PROJ_LSTORE(r0, 1)
    __syncthreads();
    // odd turn: stage 1 holds slice kt + 1, set 1 holds slice kt + 2 (past the end: a copy of the last slice)
    SEKA_PROJ_GLOAD(r0, kt + 3)
    SEKA_PROJ_COMPUTE(1)
    SEKA_PROJ_LSTORE(r1, 0)
    __syncthreads();
  }
  if (kt < nk) SEKA_PROJ_COMPUTE(0)                        // an odd number of slices: the last one sits in stage 0
  __syncthreads();
#undef SEKA_PROJ_GLOAD
#undef SEKA_PROJ_LSTORE
#undef SEKA_PROJ_COMPUTE
  // ---- epilogue: round, sum for the routing, stage the tile in LDS, store 16 bytes per lane ----
  constexpr int OLD = kProjTile + 8;                      // output tile row stride in elements
  uint16_t* Ct = lds;                                     // [128][136] = 34816 B <= the operand stages
  float colsum[2] = {0.f, 0.f};
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const __bf16 v = (__bf16)acc[i][j][r];
        colsum[j] += (float)v;
        const int m = 64 * wm + 32 * i + 8 * (r >> 2) + 4 * hf + (r & 3);
        Ct[m * OLD + 64 * wn + 32 * j + l32] = __builtin_bit_cast(uint16_t, v);
      }
  if (ROUTE) {
    // this wave's 64 tokens lie in one prompt (S is a multiple of 128); feature column -> (head, d)
    const size_t tok = row0 + 64 * wm;
    const int b = (int)(tok / S), tchunk = (int)(tok % S) / 64;
    const int hq = col0 / 128, h = hq / G, g = hq % G;            // D = 128: one tile column block = one head
    const int chunks = (S / 64) * G;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const float tot = colsum[j] + __shfl_xor(colsum[j], 32);    // the other 32 tokens of the wave
      if (hf == 0)
        workspace[(((size_t)b * Hkv + h) * chunks + (size_t)tchunk * G + g) * 128 + 64 * wn + 32 * j + l32] = tot;
    }
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < (kProjTile * kProjTile / 8) / 256; ++it) {
    const int idx = tid + 256 * it, m = idx / (kProjTile / 8), c8 = idx % (kProjTile / 8);
    const uint4 v = *reinterpret_cast<const uint4*>(Ct + m * OLD + 8 * c8);
    *reinterpret_cast<uint4*>(Qout + (row0 + m) * (size_t)N + col0 + 8 * c8) = v;
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


size_t project_route_workspace_bytes(int B, int S, int Hq) {
  return (size_t)B * Hq * (S / 64) * 128 * sizeof(float);
}

hipError_t launch_project_route(const void* X, const void* W, int E, void* Qout, int B, int S, int Hq, int Hkv,
                                const float* proto, int M, int mode, float tau, float* w_out, void* workspace,
                                hipStream_t s) {
  const int N = Hq * 128, G = Hq / Hkv;
  const dim3 grid(N / kProjTile, (unsigned)(((size_t)B * S) / kProjTile));
  float* ws = static_cast<float*>(workspace);
  if (w_out != nullptr) {
    hipLaunchKernelGGL((project_route_kernel<true>), grid, dim3(256), 0, s, static_cast<const uint16_t*>(X),
                       static_cast<const uint16_t*>(W), static_cast<uint16_t*>(Qout), E, N, S, G, Hkv, ws);
    const float inv_count = 1.0f / ((float)S * (float)G);
    hipLaunchKernelGGL((route_finish_kernel<128>), dim3(B * Hkv), dim3(kFinishThreads), 0, s, ws, (S / 64) * G, inv_count,
                       proto, Hkv, M, mode, tau, static_cast<const int*>(nullptr), static_cast<const int*>(nullptr), 0, S, 0, G,
                       w_out);
  } else {
    hipLaunchKernelGGL((project_route_kernel<false>), grid, dim3(256), 0, s, static_cast<const uint16_t*>(X),
                       static_cast<const uint16_t*>(W), static_cast<uint16_t*>(Qout), E, N, S, G, Hkv, ws);
  }
  return hipGetLastError();
}

}  // namespace seka
