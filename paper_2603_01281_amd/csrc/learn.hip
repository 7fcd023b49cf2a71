// Offline stage of SEKA for one layer (paper Sec. 3.1 and 3.4): per KV head, the cross-covariance
// Omega = h^T h_signal / n of token key embeddings, its left singular vectors and singular values, the rank k
// that keeps a fraction gamma of the singular-value mass (Eq. 3), and the head score D_h = mean ||h+ - h-||_2.
//
// Not on the inference path: written for clarity and determinism, not speed.
//   cov_partial_kernel   Omega in 16-row strips, the token range split into chunks (fp32 accumulation); bf16
//                        tensors take cov_partial_mfma_kernel (exact products on the matrix cores, one pass).
//   jacobi_svd_kernel    one workgroup per head, Omega (d x d, column-major, padded) resident in LDS.  One-sided
//                        (Hestenes) Jacobi: plane rotations applied from the right make the columns mutually
//                        orthogonal, Omega V = U Sigma, so at convergence column j is sigma_j u_j: the left singular
//                        vectors come out directly, which is what Eq. 2 needs.  d/2 disjoint column pairs per
//                        step (round-robin tournament), d - 1 steps per sweep, until a sweep rotates nothing.
//   head_distance_*      token ranges per workgroup, 16-byte loads, partial sums merged in a fixed order.
#include "common.h"

namespace seka {

namespace {

constexpr int kLearnThreads = 256;
constexpr int kCovTokens = 32;          // tokens staged per turn
constexpr int kMaxSweeps = 30;
constexpr float kRotateTol = 2e-6f;     // rotate while |a_p . a_q| > tol |a_p| |a_q| (fp32 dot products of length d)
constexpr float kZeroSigma = 1e-5f;     // sigma_c <= this share of sigma_1 is rounding noise: its direction is not determined

__host__ __device__ inline int learn_token_splits(int n) {
  int s = n / 256;
  return s < 1 ? 1 : (s > 32 ? 32 : s);
}

template <typename T> __device__ __forceinline__ float learn_load(const T* p);
template <> __device__ __forceinline__ float learn_load<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float learn_load<uint16_t>(const uint16_t* p) { return bf16_bits_to_float(*p); }

// grid (D/16, Hkv, splits); part[((split * Hkv + h) * D + i) * D + j] = sum over the split's tokens of hn[t,h,i] hs[t,h,j]
template <typename T, int D>
__global__ __launch_bounds__(kLearnThreads) void cov_partial_kernel(const T* __restrict__ hn, const T* __restrict__ hs,
                                                                    int n, int Hkv, int splits, float* __restrict__ part) {
  constexpr int RPT = 16 * D / kLearnThreads;        // strip rows per thread (one column each)
  __shared__ float a_s[kCovTokens][16];
  __shared__ float b_s[kCovTokens][D];
  const int i0 = 16 * blockIdx.x, h = blockIdx.y, split = blockIdx.z;
  const int per = (n + splits - 1) / splits;
  const int t0 = split * per, t1 = min(n, t0 + per);
  const int j = threadIdx.x % D, rgrp = threadIdx.x / D;
  float acc[RPT];
#pragma unroll
  for (int r = 0; r < RPT; ++r) acc[r] = 0.f;
  for (int tb = t0; tb < t1; tb += kCovTokens) {
    for (int idx = threadIdx.x; idx < kCovTokens * 16; idx += kLearnThreads) {
      const int tt = idx / 16, ii = idx % 16, t = tb + tt;
      a_s[tt][ii] = t < t1 ? learn_load(hn + ((size_t)t * Hkv + h) * D + i0 + ii) : 0.f;
    }
    for (int idx = threadIdx.x; idx < kCovTokens * D; idx += kLearnThreads) {
      const int tt = idx / D, jj = idx % D, t = tb + tt;
      b_s[tt][jj] = t < t1 ? learn_load(hs + ((size_t)t * Hkv + h) * D + jj) : 0.f;
    }
    __syncthreads();
#pragma unroll 4
    for (int tt = 0; tt < kCovTokens; ++tt) {
      const float bv = b_s[tt][j];
#pragma unroll
      for (int r = 0; r < RPT; ++r) acc[r] = fmaf(a_s[tt][RPT * rgrp + r], bv, acc[r]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int r = 0; r < RPT; ++r)
    part[(((size_t)split * Hkv + h) * D + i0 + RPT * rgrp + r) * D + j] = acc[r];
}

// The same partial sums for bf16 tensors on the matrix cores.  A product of two bf16 values is exact in fp32, so
// v_mfma_f32_32x32x16_bf16 with its fp32 accumulation computes what the fp32 kernel above computes (up to the
// order of the additions) and the kernel becomes a single pass over both views: grid (splits, Hkv), a workgroup
// stages 64 tokens x D of both views in LDS with 16-byte loads and every wave owns D*D/4096 blocks of 32 x 32 of
// Omega.  Both MFMA operands run along the token axis, the strided one of the row-major [token][d] tiles, hence
// the transposing LDS reads (rows padded by 64 bytes: four consecutive rows, of which 16 lanes read 32 bytes each, fall
// into different banks).
typedef __attribute__((address_space(3))) s16x4* learn_lds_s16x4_ptr;
template <int D>
__global__ __launch_bounds__(kLearnThreads) void cov_partial_mfma_kernel(const uint16_t* __restrict__ hn,
                                                                         const uint16_t* __restrict__ hs, int n, int Hkv,
                                                                         int splits, float* __restrict__ part) {
  constexpr int TOK = 64, LD = D + 32, NB = D / 32, NBW = NB * NB / 4, CPR = D / 8;
  static_assert(NBW >= 1, "at least one block per wave");
  __shared__ __attribute__((aligned(16))) uint16_t a_s[TOK * LD];
  __shared__ __attribute__((aligned(16))) uint16_t b_s[TOK * LD];
  const int split = blockIdx.x, h = blockIdx.y;
  const int per = (n + splits - 1) / splits;
  const int t0 = split * per, t1 = min(n, t0 + per);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, hf = lane >> 5, li = lane & 15, grp = lane >> 4;
  f32x16 acc[NBW];
#pragma unroll
  for (int q = 0; q < NBW; ++q)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[q][r] = 0.f;
  // transposing read of an operand fragment: lanes address row 4 hf + li / 4 (+ 8) of a 16-token slab, columns
  // 16 (grp & 1) + 4 (li & 3) of a 32-column block; the result is lane (column l32, tokens 8 hf .. 8 hf + 7)
  const int frag_off = (4 * hf + (li >> 2)) * LD + 16 * (grp & 1) + 4 * (li & 3);
  auto frag = [&](const uint16_t* tile, int slab, int blk) __attribute__((always_inline)) -> bf16x8 {
    const uint16_t* p = tile + frag_off + (16 * slab) * LD + 32 * blk;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((learn_lds_s16x4_ptr)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((learn_lds_s16x4_ptr)(p + 8 * LD));
    return __builtin_shufflevector(__builtin_bit_cast(bf16x4, lo), __builtin_bit_cast(bf16x4, hi), 0, 1, 2, 3, 4, 5, 6, 7);
  };
  // the next 64 tokens travel through registers while the current ones are multiplied
  constexpr int NLD = TOK * CPR / kLearnThreads;
  static_assert(TOK * CPR % kLearnThreads == 0, "whole turns");
  typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
  u32x4 ra[NLD], rb[NLD];
  auto fetch = [&](int tb) __attribute__((always_inline)) {
#pragma unroll
    for (int k = 0; k < NLD; ++k) {
      const int idx = threadIdx.x + k * kLearnThreads, tt = idx / CPR, c = idx % CPR, t = tb + tt;
      ra[k] = u32x4{0, 0, 0, 0};
      rb[k] = u32x4{0, 0, 0, 0};
      if (t < t1) {
        ra[k] = *reinterpret_cast<const u32x4*>(hn + ((size_t)t * Hkv + h) * D + 8 * c);
        rb[k] = *reinterpret_cast<const u32x4*>(hs + ((size_t)t * Hkv + h) * D + 8 * c);
      }
    }
  };
  if (t0 < t1) fetch(t0);
  for (int tb = t0; tb < t1; tb += TOK) {
#pragma unroll
    for (int k = 0; k < NLD; ++k) {
      const int idx = threadIdx.x + k * kLearnThreads, tt = idx / CPR, c = idx % CPR;
      *reinterpret_cast<u32x4*>(a_s + tt * LD + 8 * c) = ra[k];
      *reinterpret_cast<u32x4*>(b_s + tt * LD + 8 * c) = rb[k];
    }
    __syncthreads();
    if (tb + TOK < t1) fetch(tb + TOK);
#pragma unroll
    for (int slab = 0; slab < TOK / 16; ++slab) {
#pragma unroll
      for (int q = 0; q < NBW; ++q) {
        const int blk = wave * NBW + q, ib = blk / NB, jb = blk % NB;
        acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a_s, slab, ib), frag(b_s, slab, jb), acc[q], 0, 0, 0);
      }
    }
    __syncthreads();
  }
  // accumulator element r of lane (l32, hf): row 8 (r / 4) + 4 hf + r % 4 of the block, column l32
#pragma unroll
  for (int q = 0; q < NBW; ++q) {
    const int blk = wave * NBW + q, ib = blk / NB, jb = blk % NB;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int i = 32 * ib + 8 * (r >> 2) + 4 * hf + (r & 3), j = 32 * jb + l32;
      part[(((size_t)split * Hkv + h) * D + i) * D + j] = acc[q][r];
    }
  }
}

// grid (Hkv); dynamic LDS: D columns of D + 1 floats, then D floats (sigma), then D ints (rank).
template <typename T, int D>
__global__ __launch_bounds__(8 * D) void jacobi_svd_kernel(const float* __restrict__ part, int Hkv, int splits,
                                                                   float inv_n, float gamma, float* __restrict__ U_out,
                                                                   float* __restrict__ sigma_out, int* __restrict__ k_out,
                                                                   T* __restrict__ U_packed, int r_pad) {
  constexpr int LD = D + 1;
  constexpr int NP = D / 2;                       // column pairs per step
  constexpr int TPP = 16;                         // threads per pair (a pair never straddles a wave)
  constexpr int NT = NP * TPP;                    // = blockDim.x
  extern __shared__ float lds[];
  float* A = lds;                                 // A[j * LD + i] = Omega[i][j]
  float* sig = lds + D * LD;
  int* rank = reinterpret_cast<int*>(sig + D);
  const int h = blockIdx.x, tid = threadIdx.x;

  for (int idx = tid; idx < D * D; idx += NT) {
    const int i = idx / D, j = idx % D;
    float s = 0.f;
    for (int sp = 0; sp < splits; ++sp) s += part[(((size_t)sp * Hkv + h) * D + i) * D + j];     // fixed order
    A[j * LD + i] = s * inv_n;
  }
  __syncthreads();

  const int pr = tid / TPP, sub = tid % TPP;
  for (int sweep = 0; sweep < kMaxSweeps; ++sweep) {
    int rotated = 0;
    for (int step = 0; step < D - 1; ++step) {
      // round-robin tournament: position 0 stays, the others rotate; positions k and D - 1 - k meet
      auto at = [&](int pos) {                    // pos - 1 + step < 2 (D - 1)
        if (pos == 0) return 0;
        const int x = pos - 1 + step;
        return (x >= D - 1 ? x - (D - 1) : x) + 1;
      };
      int p = at(pr), q = at(D - 1 - pr);
      if (p > q) { const int t = p; p = q; q = t; }
      float* ap = A + p * LD;
      float* aq = A + q * LD;
      float alpha = 0.f, beta = 0.f, gam = 0.f;
#pragma unroll
      for (int i = sub; i < D; i += TPP) {
        const float x = ap[i], y = aq[i];
        alpha = fmaf(x, x, alpha);
        beta = fmaf(y, y, beta);
        gam = fmaf(x, y, gam);
      }
#pragma unroll
      for (int d = 1; d < TPP; d *= 2) {
        alpha += __shfl_xor(alpha, d);
        beta += __shfl_xor(beta, d);
        gam += __shfl_xor(gam, d);
      }
      if (fabsf(gam) > kRotateTol * sqrtf(alpha * beta)) {        // the same decision in all TPP lanes of the pair
        rotated = 1;
        const float zeta = (beta - alpha) / (2.f * gam);
        const float t = copysignf(1.f, zeta) / (fabsf(zeta) + sqrtf(1.f + zeta * zeta));
        const float c = 1.f / sqrtf(1.f + t * t), s = c * t;
#pragma unroll
        for (int i = sub; i < D; i += TPP) {
          const float x = ap[i], y = aq[i];
          ap[i] = c * x - s * y;
          aq[i] = s * x + c * y;
        }
      }
      __syncthreads();
    }
    if (!__syncthreads_or(rotated)) break;
  }

  // singular values = column norms; order them (descending, ties by column index)
  if (tid < D) {
    float s2 = 0.f;
    for (int i = 0; i < D; ++i) s2 = fmaf(A[tid * LD + i], A[tid * LD + i], s2);
    sig[tid] = sqrtf(s2);
  }
  __syncthreads();
  if (tid < D) {
    const float me = sig[tid];
    int r = 0;
    for (int k = 0; k < D; ++k) r += (sig[k] > me) || (sig[k] == me && k < tid);
    rank[tid] = r;
    sigma_out[(size_t)h * D + r] = me;
  }
  __syncthreads();
  // rank rule of Eq. 3 (one thread; d additions)
  __shared__ int k_sel;
  __shared__ float sorted_s[D];
  __shared__ float sig_floor;
  if (tid < D) sorted_s[rank[tid]] = sig[tid];
  __syncthreads();
  if (tid == 0) {
    float total = 0.f;
    for (int k = 0; k < D; ++k) total += sorted_s[k];
    float run = 0.f;
    int ks = D;
    for (int k = 0; k < D; ++k) {
      run += sorted_s[k];
      if (run >= gamma * total) { ks = k + 1; break; }
    }
    k_sel = ks;
    k_out[h] = ks;
    sig_floor = kZeroSigma * sorted_s[0];
  }
  __syncthreads();
  for (int idx = tid; idx < D * D; idx += NT) {
    const int j = idx / D, i = idx % D;                 // column j of A, element i
    const float s = sig[j];
    const float u = s > sig_floor ? A[j * LD + i] / s : 0.f;     // s > 0 here
    const int r = rank[j];
    U_out[((size_t)h * D + i) * D + r] = u;
    if (U_packed && r < r_pad) {
      const float v = r < k_sel ? u : 0.f;
      if (sizeof(T) == 2) {
        const __bf16 bv = (__bf16)v;
        reinterpret_cast<uint16_t*>(U_packed)[((size_t)h * D + i) * r_pad + r] = __builtin_bit_cast(uint16_t, bv);
      } else {
        reinterpret_cast<float*>(U_packed)[((size_t)h * D + i) * r_pad + r] = v;
      }
    }
  }
}

// grid (splits, Hkv): part[h * splits + split] = sum over the split's tokens of || hp[t,h,:] - hm[t,h,:] ||_2.
// A row is D / 8 (bf16) or D / 4 (fp32) consecutive lanes with one 16-byte load each; fixed-order merges throughout.
template <typename T, int D>
__global__ __launch_bounds__(kLearnThreads) void head_distance_partial_kernel(const T* __restrict__ hp, const T* __restrict__ hm,
                                                                              int n, int Hkv, int splits, float* __restrict__ part) {
  constexpr int EPL = 16 / sizeof(T);               // elements per lane
  constexpr int LPR = D / EPL;                      // lanes per row (8, 16 or 32)
  constexpr int RPT = kLearnThreads / LPR;          // rows per workgroup turn
  __shared__ float wsum[kLearnThreads / 64];
  const int split = blockIdx.x, h = blockIdx.y;
  const int per = (n + splits - 1) / splits;
  const int t0 = split * per, t1 = min(n, t0 + per);
  const int c = threadIdx.x % LPR, rr = threadIdx.x / LPR;
  float acc = 0.f;
  for (int tb = t0; tb < t1; tb += RPT) {           // workgroup-uniform trip count
    const int t = tb + rr;
    const bool ok = t < t1;
    const size_t off = ((size_t)(ok ? t : t1 - 1) * Hkv + h) * D + c * EPL;      // clamped: loads stay inside the tensors
    const uint4 a = *reinterpret_cast<const uint4*>(hp + off), b = *reinterpret_cast<const uint4*>(hm + off);
    const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
    float s2 = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (sizeof(T) == 2) {
        const float d0 = __uint_as_float(aw[i] << 16) - __uint_as_float(bw[i] << 16);
        const float d1 = __uint_as_float(aw[i] & 0xffff0000u) - __uint_as_float(bw[i] & 0xffff0000u);
        s2 = fmaf(d0, d0, s2);
        s2 = fmaf(d1, d1, s2);
      } else {
        const float d0 = __uint_as_float(aw[i]) - __uint_as_float(bw[i]);
        s2 = fmaf(d0, d0, s2);
      }
    }
#pragma unroll
    for (int d = 1; d < LPR; d *= 2) s2 += __shfl_xor(s2, d);
    if (ok && c == 0) acc += sqrtf(s2);
  }
#pragma unroll
  for (int d = 1; d < 64; d *= 2) acc += __shfl_xor(acc, d);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    float s = 0.f;
    for (int w = 0; w < kLearnThreads / 64; ++w) s += wsum[w];
    part[(size_t)h * splits + split] = s;
  }
}

// grid (Hkv), one wave: D_h = (sum of the head's partials, in order) / n
__global__ void head_distance_finish_kernel(const float* __restrict__ part, int splits, float inv_n, float* __restrict__ D_out) {
  if (threadIdx.x == 0) {
    float s = 0.f;
    for (int i = 0; i < splits; ++i) s += part[(size_t)blockIdx.x * splits + i];
    D_out[blockIdx.x] = s * inv_n;
  }
}

template <typename T, int D>
hipError_t launch_learn_td(const void* hn, const void* hs, int n, int Hkv, float gamma, float* U_out, float* sigma_out,
                           int* k_out, void* U_packed, int r_pad, float* part, hipStream_t s) {
  const int splits = learn_token_splits(n);
  if constexpr (sizeof(T) == 2)
    hipLaunchKernelGGL((cov_partial_mfma_kernel<D>), dim3(splits, Hkv), dim3(kLearnThreads), 0, s,
                       static_cast<const uint16_t*>(hn), static_cast<const uint16_t*>(hs), n, Hkv, splits, part);
  else
    hipLaunchKernelGGL((cov_partial_kernel<T, D>), dim3(D / 16, Hkv, splits), dim3(kLearnThreads), 0, s,
                       static_cast<const T*>(hn), static_cast<const T*>(hs), n, Hkv, splits, part);
  const size_t smem = ((size_t)D * (D + 1) + 2 * D) * sizeof(float);
  auto kernel = jacobi_svd_kernel<T, D>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kernel, dim3(Hkv), dim3(8 * D), smem, s, part, Hkv, splits, 1.0f / (float)n, gamma, U_out,
                     sigma_out, k_out, static_cast<T*>(U_packed), r_pad);
  return hipGetLastError();
}

}  // namespace

// token ranges of the head-distance pass: about 2048 workgroups in all, at least 256 tokens each
static inline int distance_splits(int n, int Hkv) {
  int want = (2048 + Hkv - 1) / Hkv;
  const int cap = n / 256 > 1 ? n / 256 : 1;
  if (want > cap) want = cap;
  return want > 1024 ? 1024 : want;
}

size_t learn_workspace_bytes(int Hkv, int D, int n) {
  const size_t cov = (size_t)learn_token_splits(n) * Hkv * D * D * sizeof(float);
  const size_t dist = ((size_t)distance_splits(n, Hkv) * Hkv * sizeof(float) + 15) / 16 * 16;
  return cov > dist ? cov : dist;
}

hipError_t launch_learn(const void* hn, const void* hs, int n, int Hkv, int D, int dtype, float gamma, float* U_out,
                        float* sigma_out, int* k_out, void* U_packed, int r_pad, void* workspace, hipStream_t s) {
  float* part = static_cast<float*>(workspace);
  if (dtype == SEKA_BF16)
    return D == 128 ? launch_learn_td<uint16_t, 128>(hn, hs, n, Hkv, gamma, U_out, sigma_out, k_out, U_packed, r_pad, part, s)
                    : launch_learn_td<uint16_t, 64>(hn, hs, n, Hkv, gamma, U_out, sigma_out, k_out, U_packed, r_pad, part, s);
  return D == 128 ? launch_learn_td<float, 128>(hn, hs, n, Hkv, gamma, U_out, sigma_out, k_out, U_packed, r_pad, part, s)
                  : launch_learn_td<float, 64>(hn, hs, n, Hkv, gamma, U_out, sigma_out, k_out, U_packed, r_pad, part, s);
}

hipError_t launch_head_distance(const void* hp, const void* hm, int n, int Hkv, int D, int dtype, float* D_out,
                                void* workspace, hipStream_t s) {
  const int splits = distance_splits(n, Hkv);
  float* part = static_cast<float*>(workspace);
#define SEKA_HD_CASE(T, DD) \
  hipLaunchKernelGGL((head_distance_partial_kernel<T, DD>), dim3(splits, Hkv), dim3(kLearnThreads), 0, s, \
                     static_cast<const T*>(hp), static_cast<const T*>(hm), n, Hkv, splits, part)
  if (dtype == SEKA_BF16) { if (D == 128) SEKA_HD_CASE(uint16_t, 128); else SEKA_HD_CASE(uint16_t, 64); }
  else { if (D == 128) SEKA_HD_CASE(float, 128); else SEKA_HD_CASE(float, 64); }
#undef SEKA_HD_CASE
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(head_distance_finish_kernel, dim3(Hkv), dim3(64), 0, s, part, splits, 1.0f / (float)n, D_out);
  return hipGetLastError();
}

}  // namespace seka
