// seka_attention_decode: the generation step that follows a steered prefill.  The edited keys persist in the
// KV cache (the hook of Algorithm 1 ran at prefill, seka_edit_keys in place), so one new query per (prompt,
// head) attends to the cached keys as they are: logits q . k'_j / sqrt(d_k) over the first len[b] tokens,
// softmax, weighted sum of V (paper Sec. 2).
//
// HBM-bound: every cached key and value is read once (2 * B * S * Hkv * D elements), a few flops per byte.
// Stage 1: grid (splits, KV head x head chunk, prompt); a workgroup streams its range of cached tokens with
// 16-byte loads (a row is 16 consecutive lanes for bf16 at D = 128, so one wave instruction fetches whole
// rows) and scores them against all the query heads of its KV head (the GQA group shares every byte read),
// keeping one online-softmax state per head with a lazily raised reference exponent: on the matrix cores for
// bf16 caches (decode_partial_mfma_kernel), on the vector unit for fp32 ones (decode_partial_kernel).  Partial
// states are merged across lanes, waves (LDS) and splits (stage 2, fixed order, so the result does not depend on
// scheduling).
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
__host__ __device__ inline int decode_splits(int B, int Hkv, int G, int S, int heads_per_wg) {
  const int groups = B * Hkv * (G / heads_per_wg);
  int want = (kDecTargetWG + groups - 1) / groups;
  const int cap = S / kDecMinRows > 1 ? S / kDecMinRows : 1;
  if (want > cap) want = cap;
  if (want > kDecMaxSplits) want = kDecMaxSplits;
  return want < 1 ? 1 : want;
}

template <typename T> struct DecElem;
template <> struct DecElem<uint16_t> {
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

// What a stage-1 workgroup does with the merged state (mm, ll, oo) of output element d of query head hq: with
// several splits it goes to the partial-state buffer for stage 2; with a single split it IS the result, and the
// workgroup writes the output and the log-sum-exp itself (the same arithmetic as stage 2 on one split, which is
// then not launched: short caches take one kernel instead of two).
template <typename T, int D>
__device__ __forceinline__ void decode_emit(float mm, float ll, float oo, int b, int hq, int d, int Hq, int splits,
                                            int split, float* __restrict__ part, T* __restrict__ O,
                                            float* __restrict__ lse) {
  if (splits == 1) {
    DecElem<T>::store(O + ((size_t)b * Hq + hq) * D + d, ll > 0.f ? oo / ll : 0.f);
    if (lse && d == 0) lse[(size_t)b * Hq + hq] = ll > 0.f ? mm * 0.6931471805599453f + logf(ll) : -INFINITY;
    return;
  }
  float* dst = part + (((size_t)b * Hq + hq) * splits + split) * (D + 2);
  dst[d] = oo;
  if (d == 0) {
    dst[D] = mm;
    dst[D + 1] = ll;
  }
}

// partial state of one (prompt, query head, split): D unnormalised outputs, then m (base-2 exponent), then l
// (fp32 caches: every product on the vector unit, exactness over speed)
template <typename T, int D, int GP>
__global__ __launch_bounds__(kDecThreads) void decode_partial_kernel(const T* __restrict__ q, const T* __restrict__ K,
                                                                     const T* __restrict__ V, const int* __restrict__ lens,
                                                                     int S, int Hq, int Hkv, float c2, int splits,
                                                                     float* __restrict__ part, T* __restrict__ O,
                                                                     float* __restrict__ lse) {
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
  for (int turn = k0; turn < k1; turn += UNR * step) {      // workgroup-uniform trip count
    const int base = turn + wave * KPW + kk;
    bool ok[UNR];
    {
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
    decode_emit<T, D>(mm, ll, oo, b, hq0 + g, d, Hq, splits, split, part, O, lse);
  }
}

// Stage 1 for bf16 caches on the matrix cores.  Same grid, split ranges and partial-state layout as the kernel
// above; what changes is who does the arithmetic.  The query heads of the group (HP <= 16 of them, padded to the 32
// columns of the instruction) take the place that a tile of queries has in the prefill kernel:
//   S^T (32 keys x heads)   = K (32 keys x D) q^T        D/16 x v_mfma_f32_32x32x16_bf16
//   O^T (D x heads)        += V^T (D x 32 keys) P^T      2 D/32 of them
// Keys and values are loaded as whole rows (every cache line requested once; fragments fetched straight from
// global memory, 32 bytes per lane pair, cost twice the time) and pass through a wave-private LDS tile with padded
// rows (no bank conflicts): K comes back with 16-byte reads, then V takes the tile over and comes back through transposing reads,
// so that the vector unit is left with the softmax alone (one fma, one exponential and half a conversion per key
// and lane) instead of every product, and a wave's next 32 keys and values (16 KB) are in flight while it works
// on the current ones.  Waves take the 32-key blocks of the workgroup's range in turn and never synchronise
// before the final merge.  Probabilities are rounded to bf16 once; that value feeds the row sum and the product.
typedef __attribute__((address_space(3))) s16x4* dec_lds_s16x4_ptr;
constexpr int kDecMfmaMaxHeads = 16;

__host__ __device__ inline int decode_heads_per_group_mfma(int G) {
  if (G <= kDecMfmaMaxHeads) return G;
  for (int hp = kDecMfmaMaxHeads; hp > 1; --hp)
    if (G % hp == 0) return hp;
  return 1;
}

template <int D>
__global__ __launch_bounds__(kDecThreads, 2) void decode_partial_mfma_kernel(const uint16_t* __restrict__ q,
                                                                          const uint16_t* __restrict__ K,
                                                                          const uint16_t* __restrict__ V,
                                                                          const int* __restrict__ lens, int S, int Hq,
                                                                          int Hkv, int HP, float c2, int splits,
                                                                          float* __restrict__ part, uint16_t* __restrict__ O,
                                                                          float* __restrict__ lse) {
  constexpr int BK = 32;                   // keys per block
  // LDS row strides (elements).  K rows are read back 16 bytes per lane by 16 consecutive rows: a stride of 16 bytes
  // mod 256 spreads them over all banks.  V rows come back through transposing reads, where 16 lanes take 32 bytes
  // of each of four consecutive rows: a stride of 64 bytes mod 256 keeps those apart.
  constexpr int LDK = D + 8, LD = D + 32;
  constexpr int OLD = D + 4;               // row stride of the merge area (floats)
  constexpr int KS = D / 16, NB = D / 32;
  constexpr int CPR = D / 8, RPI = 64 / CPR, NV = BK / RPI;   // V rows: 16-byte chunks per row, rows per load, loads
  constexpr int kTileBytes = BK * LD * 2;
  constexpr int kMergeBytes = kDecMfmaMaxHeads * OLD * 4;
  __shared__ __attribute__((aligned(16))) unsigned char smem[kDecWaves * (kTileBytes > kMergeBytes ? kTileBytes : kMergeBytes)];
  __shared__ float sm_ml[kDecWaves][kDecMfmaMaxHeads][2];

  const int G = Hq / Hkv;
  const int chunks = G / HP;
  const int b = blockIdx.z, h = blockIdx.y / chunks, hq0 = h * G + (blockIdx.y % chunks) * HP;
  const int split = blockIdx.x;
  const int n = lens ? min(max(lens[b], 0), S) : S;
  const int per = (S + splits - 1) / splits;
  const int k0 = split * per, k1 = min(n, k0 + per);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, hf = lane >> 5, li = lane & 15, grp = lane >> 4;
  uint16_t* vt = reinterpret_cast<uint16_t*>(smem + (size_t)wave * kTileBytes);

  typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;   // (a plain vector type: arrays of it stay in registers)
  // B operand of the score product: lane (head l32, hf) holds q[head][16 s + 8 hf ..][0..7]; padding heads are zero
  bf16x8 qf[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    u32x4 t = {0, 0, 0, 0};
    if (l32 < HP) t = *reinterpret_cast<const u32x4*>(q + ((size_t)b * Hq + hq0 + l32) * D + 16 * s + 8 * hf);
    qf[s] = __builtin_bit_cast(bf16x8, t);
  }

  const size_t rowstride = (size_t)Hkv * D;
  const uint16_t* Kb = K + ((size_t)b * S * Hkv + h) * D;
  const uint16_t* Vb = V + ((size_t)b * S * Hkv + h) * D;
  // both tiles arrive as whole rows (a row is CPR consecutive lanes: every cache line is requested once)
  u32x4 kr[NV], vr[NV];
  auto fetch = [&](int kb) __attribute__((always_inline)) {       // rows clamped into the range: loads stay inside the cache
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const size_t rv = (size_t)min(kb + RPI * i + lane / CPR, k1 - 1) * rowstride + 8 * (lane % CPR);
      kr[i] = *reinterpret_cast<const u32x4*>(Kb + rv);
      vr[i] = *reinterpret_cast<const u32x4*>(Vb + rv);
    }
  };
  // transposing read of a V^T fragment (32 values of d x 16 keys): lanes address key 4 hf + li / 4 (+ 8) of the
  // 16-key slab, columns 16 (grp & 1) + 4 (li & 3) of the 32-column block; lane (d l32, hf) receives the keys in
  // the order in which the score accumulator holds them (element e: key 8 (e / 4) + 4 hf + e % 4)
  const int frag_off = (4 * hf + (li >> 2)) * LD + 16 * (grp & 1) + 4 * (li & 3);
  auto vfrag = [&](int slab, int blk) __attribute__((always_inline)) -> bf16x8 {
    const uint16_t* p = vt + frag_off + (16 * slab) * LD + 32 * blk;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((dec_lds_s16x4_ptr)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((dec_lds_s16x4_ptr)(p + 8 * LD));
    return __builtin_shufflevector(__builtin_bit_cast(bf16x4, lo), __builtin_bit_cast(bf16x4, hi), 0, 1, 2, 3, 4, 5, 6, 7);
  };

  // state of head l32 (both halves hf keep the same m; l is this lane's share of the row sum)
  float m = kNegBig, l = 0.f;
  f32x16 oacc[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;

  int kb = k0 + wave * BK;
  if (kb < k1) fetch(kb);
  for (; kb < k1; kb += kDecWaves * BK) {
    // K rows to the wave's tile, back as A fragments (lane (key l32, hf): 16 bytes at d = 16 s + 8 hf); then the V
    // rows take the tile over.  A wave's LDS operations execute in program order; the fences are for the compiler.
#pragma unroll
    for (int i = 0; i < NV; ++i)
      *reinterpret_cast<u32x4*>(vt + (RPI * i + lane / CPR) * LDK + 8 * (lane % CPR)) = kr[i];
    asm volatile("" ::: "memory");
    f32x16 sacc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8*>(vt + l32 * LDK + 16 * s + 8 * hf);
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], sacc, 0, 0, 0);
    }
    asm volatile("" ::: "memory");
#pragma unroll
    for (int i = 0; i < NV; ++i)
      *reinterpret_cast<u32x4*>(vt + (RPI * i + lane / CPR) * LD + 8 * (lane % CPR)) = vr[i];
    asm volatile("" ::: "memory");
    const int kb_next = kb + kDecWaves * BK;
    const bool full = kb + BK <= k1;
    if (kb_next < k1) fetch(kb_next);      // the registers are free again: next block's loads fly during the softmax

    float t[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) t[r] = sacc[r] * c2;
    if (!full) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (kb + 16 * (r >> 3) + 8 * ((r >> 2) & 1) + 4 * hf + (r & 3) >= k1) t[r] = -INFINITY;
    }
    float bmax = t[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) bmax = fmaxf(bmax, t[r]);
    bmax = fmaxf(bmax, __shfl_xor(bmax, 32));
    const bool raise = bmax > m + kDecSlack;
    if (__any(raise)) {                    // rare after the first blocks
      const float alpha = raise ? __builtin_amdgcn_exp2f(m - bmax) : 1.f;
      if (raise) m = bmax;
      l *= alpha;
#pragma unroll
      for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
    }
    bf16x8 pb[2];
#pragma unroll
    for (int sl = 0; sl < 2; ++sl) {
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        const bf16x2 p2 = {(__bf16)__builtin_amdgcn_exp2f(t[8 * sl + e] - m), (__bf16)__builtin_amdgcn_exp2f(t[8 * sl + e + 1] - m)};
        pb[sl][e] = p2[0];
        pb[sl][e + 1] = p2[1];
        l = dec_dot2(__builtin_bit_cast(uint32_t, p2), 0x3f803f80u, l);
      }
    }
#pragma unroll
    for (int sl = 0; sl < 2; ++sl)
#pragma unroll
      for (int i = 0; i < NB; ++i) oacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfrag(sl, i), pb[sl], oacc[i], 0, 0, 0);
    asm volatile("" ::: "memory");         // the tile is rewritten only after these reads
  }

  // ---- merge the waves: lane (head l32, hf) holds O[head][32 i + 8 (r / 4) + 4 hf + r % 4] ----
  l += __shfl_xor(l, 32);
  __syncthreads();                         // every wave is done with its V tile: the area becomes the merge area
  float* sm_o = reinterpret_cast<float*>(smem) + (size_t)wave * kDecMfmaMaxHeads * OLD;
  if (l32 < HP) {
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4)
        *reinterpret_cast<f32x4*>(sm_o + l32 * OLD + 32 * i + 8 * r4 + 4 * hf) =
            f32x4{oacc[i][4 * r4], oacc[i][4 * r4 + 1], oacc[i][4 * r4 + 2], oacc[i][4 * r4 + 3]};
    if (hf == 0) {
      sm_ml[wave][l32][0] = m;
      sm_ml[wave][l32][1] = l;
    }
  }
  __syncthreads();
  const float* sm_all = reinterpret_cast<const float*>(smem);
  for (int idx = threadIdx.x; idx < HP * D; idx += kDecThreads) {
    const int g = idx / D, d = idx % D;
    float mm = sm_ml[0][g][0];
#pragma unroll
    for (int w = 1; w < kDecWaves; ++w) mm = fmaxf(mm, sm_ml[w][g][0]);
    float ll = 0.f, oo = 0.f;
#pragma unroll
    for (int w = 0; w < kDecWaves; ++w) {
      const float aw = __builtin_amdgcn_exp2f(sm_ml[w][g][0] - mm);
      ll += sm_ml[w][g][1] * aw;
      oo += sm_all[((size_t)w * kDecMfmaMaxHeads + g) * OLD + d] * aw;
    }
    decode_emit<uint16_t, D>(mm, ll, oo, b, hq0 + g, d, Hq, splits, split, part, O, lse);
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
                     splits, part, static_cast<T*>(O), lse);
  if (splits > 1)
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

// query heads that one stage-1 workgroup serves: the bf16 kernel takes up to 16 per KV head, the fp32 one up to 8
static int decode_heads_per_wg(int G, int dtype) {
  return dtype == SEKA_BF16 ? decode_heads_per_group_mfma(G) : decode_heads_per_group(G);
}

size_t decode_workspace_bytes(int B, int S, int Hq, int Hkv, int D, int dtype) {
  const int G = Hq / Hkv;
  return (size_t)B * Hq * decode_splits(B, Hkv, G, S, decode_heads_per_wg(G, dtype)) * (D + 2) * sizeof(float);
}

hipError_t launch_decode(const void* q, const void* K, const void* V, void* O, float* lse, const int* lens, int B, int S,
                         int Hq, int Hkv, int D, int dtype, float scale, void* workspace, hipStream_t s) {
  const int G = Hq / Hkv, hp = decode_heads_per_wg(G, dtype);
  const int splits = decode_splits(B, Hkv, G, S, hp);
  float* part = static_cast<float*>(workspace);
  if (dtype == SEKA_BF16) {
    const float c2 = scale * 1.4426950408889634f;
    const dim3 grid(splits, Hkv * (G / hp), B);
    const uint16_t *q16 = static_cast<const uint16_t*>(q), *K16 = static_cast<const uint16_t*>(K), *V16 = static_cast<const uint16_t*>(V);
    uint16_t* O16 = static_cast<uint16_t*>(O);
    if (D == 128) {
      hipLaunchKernelGGL(decode_partial_mfma_kernel<128>, grid, dim3(kDecThreads), 0, s, q16, K16, V16, lens, S, Hq, Hkv, hp, c2, splits, part, O16, lse);
      if (splits > 1)
        hipLaunchKernelGGL((decode_finish_kernel<uint16_t, 128>), dim3(Hq, B), dim3(kFinThreads), 0, s, part, Hq, splits, O16, lse);
    } else {
      hipLaunchKernelGGL(decode_partial_mfma_kernel<64>, grid, dim3(kDecThreads), 0, s, q16, K16, V16, lens, S, Hq, Hkv, hp, c2, splits, part, O16, lse);
      if (splits > 1)
        hipLaunchKernelGGL((decode_finish_kernel<uint16_t, 64>), dim3(Hq, B), dim3(kFinThreads), 0, s, part, Hq, splits, O16, lse);
    }
    return hipGetLastError();
  }
  return D == 128 ? launch_decode_td<float, 128>(q, K, V, O, lse, lens, B, S, Hq, Hkv, scale, part, splits, s)
                  : launch_decode_td<float, 64>(q, K, V, O, lse, lens, B, S, Hq, Hkv, scale, part, splits, s);
}

}  // namespace seka
