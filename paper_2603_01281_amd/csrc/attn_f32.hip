// fp32 causal GQA attention with the key edit fused in (paper Sec. 2: scores q.k'/sqrt(d_k); k' = k + g P k
// on highlighted tokens).  This is the exact-arithmetic path for small problems: plain fp32 FMAs,
// no matrix cores.  One workgroup = 64 query rows of one query head; keys/values are visited in tiles
// of 32 staged in LDS; the tile's highlighted keys are edited in LDS before scoring, so edited keys
// never reach HBM.  Four threads share a query row (8 keys of the tile each, then a quarter of D each).
#include "common.h"

namespace seka {

namespace {

constexpr int kThreads = 256;
constexpr int BQ = 64;
constexpr int BK = 32;

template <int D, bool STEER>
__global__ __launch_bounds__(kThreads) void attention_f32_kernel(AttnArgs a, SteerArgs st) {
  __shared__ float Ks[BK][D + 1];
  __shared__ float Vs[BK][D];
  __shared__ float Ps[BQ][BK + 1];
  __shared__ float Zs[STEER ? BK : 1][STEER ? SEKA_MAX_RANK : 1];
  __shared__ int Ms[BK];

  const float* __restrict__ Q = static_cast<const float*>(a.Q);
  const float* __restrict__ K = static_cast<const float*>(a.K);
  const float* __restrict__ V = static_cast<const float*>(a.V);
  float* __restrict__ O = static_cast<float*>(a.O);

  const int b = blockIdx.z, hq = blockIdx.y;
  const int G = a.Hq / a.Hkv, h = hq / G;
  const int q0 = (gridDim.x - 1 - blockIdx.x) * BQ;      // longest rows first
  const int row = threadIdx.x >> 2, part = threadIdx.x & 3;
  const int i = q0 + row;
  size_t tok0;                                           // first token of this prompt in the tensors
  int Sb;                                                // this prompt's length
  prompt_extent(a, b, tok0, Sb);
  if (q0 >= Sb) return;                                  // block beyond the prompt's end (uniform, before any barrier)
  const bool row_ok = i < Sb;

  float q[D];
  {
    const float* qp = Q + ((tok0 + (row_ok ? i : 0)) * a.Hq + hq) * D;
#pragma unroll
    for (int d = 0; d < D; ++d) q[d] = row_ok ? qp[d] : 0.f;
  }
  constexpr int DP = D / 4;
  float o[DP];
#pragma unroll
  for (int d = 0; d < DP; ++d) o[d] = 0.f;
  float m_run = -1e30f, l_run = 0.f;

  const float gain = STEER ? st.gain[h] : 0.f;
  const float kscale = STEER ? st.kscale[h] : 1.f;
  const int R = STEER ? st.M * st.r : 0;
  const float* Uh = STEER ? static_cast<const float*>(st.U) + (size_t)h * st.M * D * st.r : nullptr;

  const int last_key = min(Sb, q0 + BQ) - 1;
  for (int k0 = 0; k0 <= last_key; k0 += BK) {
    for (int idx = threadIdx.x; idx < BK * D; idx += kThreads) {
      const int jj = idx / D, d = idx % D, t = k0 + jj;
      const size_t off = ((tok0 + t) * a.Hkv + h) * D + d;
      Ks[jj][d] = t < Sb ? K[off] : 0.f;
      Vs[jj][d] = t < Sb ? V[off] : 0.f;
    }
    int any = 0;
    if (STEER) {
      if (threadIdx.x < BK) {
        const int t = k0 + threadIdx.x;
        const int mk = (t < Sb && gain != 0.f) ? st.mask[tok0 + t] : 0;
        Ms[threadIdx.x] = mk;
        any = mk != 0;
      }
    }
    const bool edit_tile = __syncthreads_or(any) != 0;
    if (STEER && edit_tile) {
      for (int idx = threadIdx.x; idx < BK * R; idx += kThreads) {
        const int jj = idx / R, r = idx % R, m = r / st.r, rr = r % st.r;
        float acc = 0.f;
        if (Ms[jj]) {
          const float* u = Uh + (size_t)m * D * st.r + rr;
          for (int d = 0; d < D; ++d) acc = fmaf(u[(size_t)d * st.r], Ks[jj][d], acc);
          acc *= gain * (st.w ? st.w[((size_t)b * a.Hkv + h) * st.M + m] : 1.f);
        }
        Zs[jj][r] = acc;
      }
      __syncthreads();
      for (int idx = threadIdx.x; idx < BK * D; idx += kThreads) {
        const int jj = idx / D, d = idx % D;
        if (!Ms[jj]) continue;
        float acc = 0.f;
        for (int r = 0; r < R; ++r) {
          const int m = r / st.r, rr = r % st.r;
          acc = fmaf(Uh[((size_t)m * D + d) * st.r + rr], Zs[jj][r], acc);
        }
        Ks[jj][d] = fmaf(kscale, Ks[jj][d], acc);
      }
      __syncthreads();
    }

    float s[BK / 4];
    float mx = -INFINITY;
#pragma unroll
    for (int jj = 0; jj < BK / 4; ++jj) {
      const int j = part + 4 * jj;
      float acc = 0.f;
#pragma unroll
      for (int d = 0; d < D; ++d) acc = fmaf(q[d], Ks[j][d], acc);
      acc *= a.scale;
      if (k0 + j > i) acc = -INFINITY;
      s[jj] = acc;
      mx = fmaxf(mx, acc);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 1));
    mx = fmaxf(mx, __shfl_xor(mx, 2));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = expf(m_run - m_new);
    float lsum = 0.f;
#pragma unroll
    for (int jj = 0; jj < BK / 4; ++jj) {
      const float p = expf(s[jj] - m_new);
      Ps[row][part + 4 * jj] = p;
      lsum += p;
    }
    l_run = l_run * alpha + lsum;
    m_run = m_new;
    __syncthreads();
#pragma unroll
    for (int d = 0; d < DP; ++d) o[d] *= alpha;
    for (int j = 0; j < BK; ++j) {
      const float p = Ps[row][j];
#pragma unroll
      for (int d = 0; d < DP; ++d) o[d] = fmaf(p, Vs[j][part * DP + d], o[d]);
    }
    __syncthreads();
  }

  l_run += __shfl_xor(l_run, 1);
  l_run += __shfl_xor(l_run, 2);
  if (row_ok) {
    float* op = O + ((tok0 + i) * a.Hq + hq) * D + part * DP;
    const float inv = 1.f / l_run;
#pragma unroll
    for (int d = 0; d < DP; ++d) op[d] = o[d] * inv;
    if (a.lse && part == 0) a.lse[lse_index(a, b, hq, tok0, i)] = m_run + logf(l_run);
  }
}

}  // namespace

hipError_t launch_attention_f32(const AttnArgs& a, const SteerArgs* steer, hipStream_t s) {
  const dim3 grid((a.S + BQ - 1) / BQ, a.Hq, a.B);
  SteerArgs none;
  none.U = nullptr; none.w = nullptr; none.mask = nullptr; none.M = 0; none.r = 0;
  if (steer) {
    if (a.D == 128) hipLaunchKernelGGL((attention_f32_kernel<128, true>), grid, dim3(kThreads), 0, s, a, *steer);
    else hipLaunchKernelGGL((attention_f32_kernel<64, true>), grid, dim3(kThreads), 0, s, a, *steer);
  } else {
    if (a.D == 128) hipLaunchKernelGGL((attention_f32_kernel<128, false>), grid, dim3(kThreads), 0, s, a, none);
    else hipLaunchKernelGGL((attention_f32_kernel<64, false>), grid, dim3(kThreads), 0, s, a, none);
  }
  return hipGetLastError();
}

}  // namespace seka
