// seka_attention_decode: the generation step that follows a steered prefill.  The edited keys persist in the
// KV cache (the hook of Algorithm 1 ran at prefill, seka_edit_keys in place), so one new query per (prompt,
// head) attends to the cached keys as they are: logits q . k'_j / sqrt(d_k) over the first len[b] tokens,
// softmax, weighted sum of V (paper Sec. 2).
//
// HBM-bound: every cached key and value is read once (2 * B * S * Hkv * D elements), a few flops per byte.
// Stage 1: grid (splits, KV head x head chunk, prompt); a workgroup streams its range of cached tokens with
// 16-byte loads (a row is 16 consecutive lanes for bf16 at D = 128, so one wave instruction fetches whole
// rows), scores them against the GP query heads of its KV head that it keeps in registers (the GQA group
// shares every byte read), and keeps one online-softmax state per head and lane group with a lazily raised
// reference exponent.  Partial states are merged across lanes, waves (LDS) and splits (stage 2, fixed order, so
// the result does not depend on scheduling).
#include <mutex>

#include "common.h"

namespace seka {

namespace {

// Library-owned partial-state buffer of seka_attention_decode_static (callers that cannot allocate).  One copy per
// GPU that loads the library, held until the process ends; host code never uses this name as an address (it is
// a host-side stand-in there): decode_static_scratch() resolves the device address once per device.
static __device__ __align__(256) unsigned char scratch[kDecodeStaticScratchBytes];

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / 64;
constexpr float kDecSlack = 8.f;        // a head's reference exponent trails its maximum by at most this
constexpr float kNegBig = -1e30f;
// split policy (measured on MI355X: more, smaller splits lose to the merge stage; fewer leave CUs idle)
constexpr int kDecTargetWG = 4096, kDecMinRows = 512, kDecMaxSplits = 64;

__host__ __device__ inline int decode_heads_per_group(int G) {
  if (G <= 8) return G;
  for (int gp = 8; gp > 1; --gp)
    if (G % gp == 0) return gp;
  return 1;
}

// Splits of the cached range per (prompt, head group): about kDecTargetWG workgroups in all, at least kDecMinRows tokens each.
__host__ __device__ inline int decode_splits(int B, int Hkv, int G, int S) {
  const int groups = B * Hkv * (G / decode_heads_per_group(G));
  int want = (kDecTargetWG + groups - 1) / groups;
  const int cap = S / kDecMinRows > 1 ? S / kDecMinRows : 1;
  if (want > cap) want = cap;
  if (want > kDecMaxSplits) want = kDecMaxSplits;
  return want < 1 ? 1 : want;
}

template <typename T> struct DecElem;
template <> struct DecElem<uint16_t> {
  static constexpr int EPL = 8;         // elements per 16-byte load
  __device__ static void load(const uint16_t* p, float (&out)[8]) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[2 * i] = __uint_as_float(w[i] << 16);
      out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  __device__ static void store(uint16_t* p, float v) {
    const __bf16 b = (__bf16)v;
    *p = __builtin_bit_cast(uint16_t, b);
  }
};
__device__ __forceinline__ float dec_dot2(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}

template <> struct DecElem<float> {
  static constexpr int EPL = 4;
  __device__ static void load(const float* p, float (&out)[4]) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
  }
  __device__ static void store(float* p, float v) { *p = v; }
};

// Sum over the LPR consecutive lanes that hold one row; every one of them receives the total.
template <int LPR>
__device__ __forceinline__ float row_sum(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xf, 0xf, true));    // lane ^ 1
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xf, 0xf, true));    // lane ^ 2
  if (LPR >= 8)
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xf, 0xf, true)); // mirror in 8
  if (LPR >= 16)
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xf, 0xf, true)); // mirror in 16
  if (LPR >= 32) v += __shfl_xor(v, 16);
  return v;
}

// Merge online-softmax state (m2, l2, o2) into (m, l, o); exponents are base 2.
template <int N>
__device__ __forceinline__ void merge_state(float& m, float& l, float (&o)[N], float m2, float l2, const float (&o2)[N]) {
  const float mm = fmaxf(m, m2);
  const float a1 = __builtin_amdgcn_exp2f(m - mm), a2 = __builtin_amdgcn_exp2f(m2 - mm);
  m = mm;
  l = l * a1 + l2 * a2;
#pragma unroll
  for (int i = 0; i < N; ++i) o[i] = o[i] * a1 + o2[i] * a2;
}

// partial state of one (prompt, query head, split): D unnormalised outputs, then m (base-2 exponent), then l
template <typename T, int D, int GP>
__global__ __launch_bounds__(kDecThreads) void decode_partial_kernel(const T* __restrict__ q, const T* __restrict__ K,
                                                                     const T* __restrict__ V, const int* __restrict__ lens,
                                                                     int S, int Hq, int Hkv, float c2, int splits,
                                                                     float* __restrict__ part) {
  constexpr int EPL = DecElem<T>::EPL;
  constexpr int LPR = D / EPL;            // lanes per cached row
  constexpr int KPW = 64 / LPR;           // rows per wave load
  constexpr int UNR = 4;                  // row groups in flight per lane
  __shared__ float sm_o[kDecWaves][GP][D];
  __shared__ float sm_ml[kDecWaves][GP][2];

  const int G = Hq / Hkv;
  const int chunks = G / GP;
  const int b = blockIdx.z, h = blockIdx.y / chunks, hq0 = h * G + (blockIdx.y % chunks) * GP;
  const int split = blockIdx.x;
  const int n = lens ? min(max(lens[b], 0), S) : S;
  const int per = (S + splits - 1) / splits;
  const int k0 = split * per, k1 = min(n, k0 + per);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane % LPR, kk = lane / LPR;

  float qv[GP][EPL];
#pragma unroll
  for (int g = 0; g < GP; ++g) DecElem<T>::load(q + ((size_t)b * Hq + hq0 + g) * D + c * EPL, qv[g]);

  float m[GP], l[GP], o[GP][EPL];
#pragma unroll
  for (int g = 0; g < GP; ++g) {
    m[g] = kNegBig;
    l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[g][e] = 0.f;
  }

  const size_t rowstride = (size_t)Hkv * D;
  const T* Kb = K + ((size_t)b * S * Hkv + h) * D + c * EPL;
  const T* Vb = V + ((size_t)b * S * Hkv + h) * D + c * EPL;
  const int step = kDecWaves * KPW;                      // rows per workgroup turn
  constexpr bool PACKED = sizeof(T) == 2;      // bf16: both products on the packed dot-product instruction
  uint32_t qw[GP][4];                          // PACKED: the query chunk as it is stored (pairs of bf16)
  if (PACKED) {
#pragma unroll
    for (int g = 0; g < GP; ++g) {
      const uint4 t4 = *reinterpret_cast<const uint4*>(q + ((size_t)b * Hq + hq0 + g) * D + c * EPL);
      qw[g][0] = t4.x; qw[g][1] = t4.y; qw[g][2] = t4.z; qw[g][3] = t4.w;
    }
  }
  for (int turn = k0; turn < k1; turn += UNR * step) {      // workgroup-uniform trip count
    const int base = turn + wave * KPW + kk;
    bool ok[UNR];
    float sc[UNR][GP];
    if (PACKED) {
      uint4 kr[UNR], vr[UNR];
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int row = base + u * step;
        ok[u] = row < k1;
        const size_t r = (size_t)(ok[u] ? row : k1 - 1) * rowstride;      // clamped: loads stay inside the cache
        kr[u] = *reinterpret_cast<const uint4*>(Kb + r);
        vr[u] = *reinterpret_cast<const uint4*>(Vb + r);
      }
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
#pragma unroll
        for (int g = 0; g < GP; ++g) {
          float t = dec_dot2(qw[g][0], kr[u].x, 0.f);
          t = dec_dot2(qw[g][1], kr[u].y, t);
          t = dec_dot2(qw[g][2], kr[u].z, t);
          t = dec_dot2(qw[g][3], kr[u].w, t);
          t = row_sum<LPR>(t) * c2;
          sc[u][g] = ok[u] ? t : -INFINITY;
        }
      }
      // one reference check per head and turn; probabilities are rounded to bf16 and that rounded value feeds both
      // the row sum and the PV product (two cached rows per packed instruction)
      uint32_t pp[UNR / 2][GP];
#pragma unroll
      for (int g = 0; g < GP; ++g) {
        float smax = sc[0][g];
#pragma unroll
        for (int u = 1; u < UNR; ++u) smax = fmaxf(smax, sc[u][g]);
        if (smax > m[g] + kDecSlack) {                     // rare after the first rows
          const float alpha = __builtin_amdgcn_exp2f(m[g] - smax);
          m[g] = smax;
          l[g] *= alpha;
#pragma unroll
          for (int e = 0; e < EPL; ++e) o[g][e] *= alpha;
        }
#pragma unroll
        for (int pr = 0; pr < UNR / 2; ++pr) {
          const bf16x2 p2 = {(__bf16)__builtin_amdgcn_exp2f(sc[2 * pr][g] - m[g]),
                             (__bf16)__builtin_amdgcn_exp2f(sc[2 * pr + 1][g] - m[g])};
          pp[pr][g] = __builtin_bit_cast(uint32_t, p2);
          l[g] = dec_dot2(pp[pr][g], 0x3f803f80u, l[g]);
        }
      }
#pragma unroll
      for (int pr = 0; pr < UNR / 2; ++pr) {
        const uint32_t va[4] = {vr[2 * pr].x, vr[2 * pr].y, vr[2 * pr].z, vr[2 * pr].w};
        const uint32_t vb[4] = {vr[2 * pr + 1].x, vr[2 * pr + 1].y, vr[2 * pr + 1].z, vr[2 * pr + 1].w};
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const uint32_t lo = __builtin_amdgcn_perm(vb[w], va[w], 0x05040100u);   // (row a, row b) of element 2 w
          const uint32_t hi = __builtin_amdgcn_perm(vb[w], va[w], 0x07060302u);   // ... of element 2 w + 1
#pragma unroll
          for (int g = 0; g < GP; ++g) {
            o[g][2 * w] = dec_dot2(lo, pp[pr][g], o[g][2 * w]);
            o[g][2 * w + 1] = dec_dot2(hi, pp[pr][g], o[g][2 * w + 1]);
          }
        }
      }
    } else {
      float kf[UNR][EPL], vf[UNR][EPL];
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int row = base + u * step;
        ok[u] = row < k1;
        const size_t r = (size_t)(ok[u] ? row : k1 - 1) * rowstride;
        DecElem<T>::load(Kb + r, kf[u]);
        DecElem<T>::load(Vb + r, vf[u]);
      }
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
#pragma unroll
        for (int g = 0; g < GP; ++g) {
          float s = 0.f;
#pragma unroll
          for (int e = 0; e < EPL; ++e) s = fmaf(qv[g][e], kf[u][e], s);
          s = row_sum<LPR>(s) * c2;
          if (!ok[u]) s = -INFINITY;
          if (s > m[g] + kDecSlack) {                      // raise the reference exponent (rare after the first rows)
            const float alpha = __builtin_amdgcn_exp2f(m[g] - s);
            m[g] = s;
            l[g] *= alpha;
#pragma unroll
            for (int e = 0; e < EPL; ++e) o[g][e] *= alpha;
          }
          const float p = __builtin_amdgcn_exp2f(s - m[g]);
          l[g] += p;
#pragma unroll
          for (int e = 0; e < EPL; ++e) o[g][e] = fmaf(p, vf[u][e], o[g][e]);
        }
      }
    }
  }

  // ---- merge the row groups of a wave (lanes c, c + LPR, ...), then the waves ----
#pragma unroll
  for (int g = 0; g < GP; ++g) {
#pragma unroll
    for (int d = LPR; d < 64; d *= 2) {
      float o2[EPL];
      const float m2 = __shfl_xor(m[g], d), l2 = __shfl_xor(l[g], d);
#pragma unroll
      for (int e = 0; e < EPL; ++e) o2[e] = __shfl_xor(o[g][e], d);
      merge_state(m[g], l[g], o[g], m2, l2, o2);
    }
    if (kk == 0) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) sm_o[wave][g][c * EPL + e] = o[g][e];
      if (c == 0) {
        sm_ml[wave][g][0] = m[g];
        sm_ml[wave][g][1] = l[g];
      }
    }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < GP * D; idx += kDecThreads) {
    const int g = idx / D, d = idx % D;
    float mm = sm_ml[0][g][0];
#pragma unroll
    for (int w = 1; w < kDecWaves; ++w) mm = fmaxf(mm, sm_ml[w][g][0]);
    float ll = 0.f, oo = 0.f;
#pragma unroll
    for (int w = 0; w < kDecWaves; ++w) {
      const float aw = __builtin_amdgcn_exp2f(sm_ml[w][g][0] - mm);
      ll += sm_ml[w][g][1] * aw;
      oo += sm_o[w][g][d] * aw;
    }
    float* dst = part + (((size_t)b * Hq + hq0 + g) * splits + split) * (D + 2);
    dst[d] = oo;
    if (d == 0) {
      dst[D] = mm;
      dst[D + 1] = ll;
    }
  }
}

// grid (Hq, B), block kFinThreads: thread (j, d) merges splits j, j + NJ, ... in that order, then the NJ partial
// states are merged in index order: a fixed order, whatever the launch.  The kernel is pure latency (a few tens of
// kilobytes per workgroup), so every load of a thread is issued before the first is used, and a thread has at most
// kDecMaxSplits / NJ of them.
constexpr int kFinThreads = 1024;
template <typename T, int D>
__global__ __launch_bounds__(kFinThreads) void decode_finish_kernel(const float* __restrict__ part, int Hq, int splits,
                                                                    T* __restrict__ O, float* __restrict__ lse) {
  constexpr int NJ = kFinThreads / D;
  constexpr int NI = (kDecMaxSplits + NJ - 1) / NJ;        // splits per thread, at most
  __shared__ float sm[NJ][D + 2];
  const int hq = blockIdx.x, b = blockIdx.y, d = threadIdx.x % D, j = threadIdx.x / D;
  const float* src = part + ((size_t)b * Hq + hq) * splits * (D + 2);
  float mv[NI], lv[NI], ov[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int s = j + NJ * i;
    const float* ps = src + (size_t)(s < splits ? s : 0) * (D + 2);     // clamped: the value is dropped below
    mv[i] = ps[D];
    lv[i] = ps[D + 1];
    ov[i] = ps[d];
  }
  float mm = kNegBig;
#pragma unroll
  for (int i = 0; i < NI; ++i)
    if (j + NJ * i < splits) mm = fmaxf(mm, mv[i]);
  float ll = 0.f, oo = 0.f;
#pragma unroll
  for (int i = 0; i < NI; ++i)
    if (j + NJ * i < splits) {
      const float aw = __builtin_amdgcn_exp2f(mv[i] - mm);
      ll += lv[i] * aw;
      oo += ov[i] * aw;
    }
  sm[j][d] = oo;
  if (d == 0) {
    sm[j][D] = mm;
    sm[j][D + 1] = ll;
  }
  __syncthreads();
  if (j == 0) {
    float m2 = sm[0][D];
#pragma unroll
    for (int k = 1; k < NJ; ++k) m2 = fmaxf(m2, sm[k][D]);
    float l2 = 0.f, o2 = 0.f;
#pragma unroll
    for (int k = 0; k < NJ; ++k) {
      const float aw = __builtin_amdgcn_exp2f(sm[k][D] - m2);
      l2 += sm[k][D + 1] * aw;
      o2 += sm[k][d] * aw;
    }
    DecElem<T>::store(O + ((size_t)b * Hq + hq) * D + d, l2 > 0.f ? o2 / l2 : 0.f);
    if (lse && d == 0) lse[(size_t)b * Hq + hq] = l2 > 0.f ? m2 * 0.6931471805599453f + logf(l2) : -INFINITY;
  }
}

template <typename T, int D, int GP>
hipError_t launch_decode_gp(const void* q, const void* K, const void* V, void* O, float* lse, const int* lens, int B,
                            int S, int Hq, int Hkv, float scale, float* part, int splits, hipStream_t s) {
  const int chunks = (Hq / Hkv) / GP;
  const float c2 = scale * 1.4426950408889634f;
  hipLaunchKernelGGL((decode_partial_kernel<T, D, GP>), dim3(splits, Hkv * chunks, B), dim3(kDecThreads), 0, s,
                     static_cast<const T*>(q), static_cast<const T*>(K), static_cast<const T*>(V), lens, S, Hq, Hkv, c2,
                     splits, part);
  hipLaunchKernelGGL((decode_finish_kernel<T, D>), dim3(Hq, B), dim3(kFinThreads), 0, s, part, Hq, splits, static_cast<T*>(O), lse);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_decode_td(const void* q, const void* K, const void* V, void* O, float* lse, const int* lens, int B,
                            int S, int Hq, int Hkv, float scale, float* part, int splits, hipStream_t s) {
  switch (decode_heads_per_group(Hq / Hkv)) {
#define SEKA_DEC_CASE(GP) \
    case GP: return launch_decode_gp<T, D, GP>(q, K, V, O, lse, lens, B, S, Hq, Hkv, scale, part, splits, s)
    SEKA_DEC_CASE(1); SEKA_DEC_CASE(2); SEKA_DEC_CASE(3); SEKA_DEC_CASE(4);
    SEKA_DEC_CASE(5); SEKA_DEC_CASE(6); SEKA_DEC_CASE(7); SEKA_DEC_CASE(8);
#undef SEKA_DEC_CASE
    default: return hipErrorNotSupported;
  }
}

}  // namespace

hipError_t decode_static_scratch(void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptrs[kMaxDevices] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptrs[dev]) {                         // first call on this device, with it current: its own copy's address
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    ptrs[dev] = p;
  }
  *out = ptrs[dev];
  return hipSuccess;
}

size_t decode_workspace_bytes(int B, int S, int Hq, int Hkv, int D) {
  return (size_t)B * Hq * decode_splits(B, Hkv, Hq / Hkv, S) * (D + 2) * sizeof(float);
}

hipError_t launch_decode(const void* q, const void* K, const void* V, void* O, float* lse, const int* lens, int B, int S,
                         int Hq, int Hkv, int D, int dtype, float scale, void* workspace, hipStream_t s) {
  const int splits = decode_splits(B, Hkv, Hq / Hkv, S);
  float* part = static_cast<float*>(workspace);
  if (dtype == SEKA_BF16)
    return D == 128 ? launch_decode_td<uint16_t, 128>(q, K, V, O, lse, lens, B, S, Hq, Hkv, scale, part, splits, s)
                    : launch_decode_td<uint16_t, 64>(q, K, V, O, lse, lens, B, S, Hq, Hkv, scale, part, splits, s);
  return D == 128 ? launch_decode_td<float, 128>(q, K, V, O, lse, lens, B, S, Hq, Hkv, scale, part, splits, s)
                  : launch_decode_td<float, 64>(q, K, V, O, lse, lens, B, S, Hq, Hkv, scale, part, splits, s);
}

}  // namespace seka
