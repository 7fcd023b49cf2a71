// bf16 causal GQA prefill attention for gfx950 with the spectral key edit fused in
// (paper Sec. 2: logits q_i . k'_j / sqrt(d_k), k'_j = k_j + g P k_j for highlighted j; Sec. 3.3 for the
// blended P of AdaSEKA).  Flash-style: scores and edited keys never leave the CU.
//
// Work decomposition
//   workgroup = HPW query heads of one KV group x (32*RB) query rows; wave = 32 rows of one head.
//   All waves share the K/V tiles (64 keys) staged in LDS, so a KV head's tile is read from L2
//   once for HPW heads.  Workgroups with the longest causal extent are launched first.
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16, wave64)
//   S^T = K Q^T   : A = K tile rows from LDS, B = Q fragments held in registers for the whole kernel.
//                   A lane then owns ONE query row (column of S^T) and 32 of the tile's 64 keys,
//                   so the row max/sum are in-lane reductions plus one exchange with lane^32.
//   O^T = V^T P^T : B = P^T taken straight from the S^T accumulators (the contraction order over
//                   keys is permuted identically on the V side), A = V^T fragments fetched from the
//                   row-major V tile with the transposing LDS read (ds_read_b64_tr_b16).
// Key edit (STEER): one 64-bit highlight word per tile (bit k = key 64 t + k is highlighted) is kept in a ring in
//   LDS, written by one thread per tile at set-up and refilled as the tile loop advances; after a K tile with a
//   non-zero word lands in LDS, its 16-key blocks with highlights get
//   Z^T = U_cat^T K^T and K'^T = K^T + U_cat (c .* Z^T) on 16x16x32 MFMAs, written back to LDS as bf16.
#pragma once
#include "common.h"

namespace seka {

constexpr int ATT_BK = 64;   // keys per tile

__host__ __device__ constexpr int att_kld(int D) { return D + 8; }     // K tile row stride (elements)

inline size_t attention_bf16_smem_bytes(int D, int vpad, bool steer, int Rpad, int threads) {
  size_t n = ((size_t)2 * ATT_BK * att_kld(D) + 2 * (size_t)ATT_BK * (D + vpad)) * 2;
  if (steer) n += (size_t)D * (Rpad + 8) * 2 + (size_t)Rpad * 4 + (size_t)2 * threads * 8;
  return n;
}

typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

__device__ __forceinline__ bf16x8 lds_read_tr_pair(const uint16_t* p0, const uint16_t* p1) {
  // two transposing 64-bit LDS reads -> 8 contraction slots of an MFMA operand
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p0));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p1));
  const bf16x4 lo4 = __builtin_bit_cast(bf16x4, lo), hi4 = __builtin_bit_cast(bf16x4, hi);
  return __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
}

template <int D, int HPW, int RB, bool STEER, int VPAD>
__global__ __launch_bounds__(64 * HPW * RB, D == 64 ? 4 : 1) void attention_bf16_kernel(AttnArgs a, SteerArgs st, int Rpad) {
  constexpr int NW = HPW * RB;
  constexpr int NT = 64 * NW;
  constexpr int BQ = 32 * RB;
  constexpr int BK = ATT_BK;
  constexpr int KLD = att_kld(D);
  constexpr int VLD = D + VPAD;
  constexpr int K_ELEMS = BK * KLD;
  constexpr int V_ELEMS = BK * VLD;
  constexpr int NKB = 2;              // K buffers in LDS
  constexpr int KS = D / 16;          // contraction steps of S^T = K Q^T
  constexpr int DB = D / 32;          // 32-row blocks of O^T
  constexpr int CPR = D / 8;          // 16-byte chunks per tile row
  constexpr int CHUNKS = BK * CPR;
  constexpr int NCH = (CHUNKS + NT - 1) / NT;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* Kt = reinterpret_cast<uint16_t*>(smem);            // [NKB][BK][KLD]
  uint16_t* Vt = Kt + NKB * K_ELEMS;                           // [2][BK][VLD]
  uint16_t* UN = Vt + 2 * V_ELEMS;                             // [D][Rpad+8]   U_cat, row d, column r (STEER)
  const int ULD = Rpad + 8;
  float* cvec = reinterpret_cast<float*>(UN + (size_t)D * ULD);   // [Rpad]  c_r = g * w_m(r)
  // [2 NT] ring of highlight words: bit k of entry (t mod 2 NT) = key 64 t + k is highlighted (STEER)
  unsigned long long* hlring = reinterpret_cast<unsigned long long*>(cvec + Rpad);

  const uint16_t* __restrict__ Qg = static_cast<const uint16_t*>(a.Q);
  const uint16_t* __restrict__ Kg = static_cast<const uint16_t*>(a.K);
  const uint16_t* __restrict__ Vg = static_cast<const uint16_t*>(a.V);
  uint16_t* __restrict__ Og = static_cast<uint16_t*>(a.O);

  const int Scap = a.S;                      // tokens per prompt in memory (strides, launch grid)
  const int G = a.Hq / a.Hkv;
  const int nHC = a.Hq / HPW;
  const int nQB = (Scap + BQ - 1) / BQ;
  const int per_qb = nHC * a.B;
  const int qb = nQB - 1 - (int)(blockIdx.x / per_qb);
  const int rem = blockIdx.x % per_qb;
  const int b = rem / nHC, hc = rem % nHC;
  size_t tok0;                               // first token of this prompt in the tensors
  int S;                                     // this prompt's length
  prompt_extent(a, b, tok0, S);
  if (qb * BQ >= S) return;                  // block beyond the prompt's end (workgroup-uniform, before any barrier)
  const int hq0 = hc * HPW;
  const int h = hq0 / G;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hf = lane >> 5;
  const int hq = hq0 + wave / RB;
  const int qw = qb * BQ + 32 * (wave % RB);     // first query row of this wave
  const int qi = qw + l32;                       // this lane's query row

  const float gain = STEER ? st.gain[h] : 0.f;
  const float kscale = STEER ? st.kscale[h] : 1.f;
  const bool steer_on = STEER && gain != 0.f;

  // ---- Q fragments: B operand of S^T = K Q^T, lane (col = row qi, k = 16 ks + 8 hf + e) ----
  bf16x8 qf[KS];
  {
    const bool ok = qi < S;
    const uint16_t* qp = Qg + ((tok0 + (ok ? qi : 0)) * a.Hq + hq) * D + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (ok) v = *reinterpret_cast<const uint4*>(qp + 16 * ks);
      qf[ks] = __builtin_bit_cast(bf16x8, v);
    }
  }

  // ---- stage U_cat (as stored: row d, r contiguous) and the per-column coefficients ----
  if (STEER && steer_on) {
    const int R = st.M * st.r;
    if (R != Rpad) {
      for (int i = tid; i < D * ULD; i += NT) UN[i] = 0;
      __syncthreads();
    }
    const uint16_t* Uh = static_cast<const uint16_t*>(st.U) + (size_t)h * st.M * D * st.r;
    const int r8 = st.r / 8;
    const int total = st.M * D * r8;
    for (int idx = tid; idx < total; idx += NT) {
      const int m = idx / (D * r8), rm = idx % (D * r8);
      const int d = rm / r8, v = rm % r8;
      *reinterpret_cast<uint4*>(UN + (size_t)d * ULD + m * st.r + 8 * v) =
          *reinterpret_cast<const uint4*>(Uh + ((size_t)m * D + d) * st.r + 8 * v);
    }
    for (int r = tid; r < Rpad; r += NT) {
      float c = 0.f;
      if (r < R) c = gain * (st.w ? st.w[((size_t)b * a.Hkv + h) * st.M + r / st.r] : 1.f);
      cvec[r] = c;
    }
    // visibility of UN/cvec is ensured by the barrier that follows the first tile write
  }

  const int last_key = min(S, qb * BQ + BQ) - 1;
  const int ntiles = last_key / BK + 1;

  // ---- tile movement: global -> registers -> LDS (K and V separately) ----
  uint4 kpre[NCH], vpre[NCH];

  // A tile's rows: one base per tile that is the same for every lane (scalar registers) plus a per-lane 32-bit
  // offset that never changes (row * Hkv * D + chunk, under 64 rows), the same for K and V.
  const size_t head_off = (tok0 * a.Hkv + h) * D;
  const size_t tile_stride = (size_t)BK * a.Hkv * D;
  unsigned loff[NCH];
#pragma unroll
  for (int n = 0; n < NCH; ++n) {
    const int c = tid + NT * n;
    loff[n] = (unsigned)((c / CPR) * a.Hkv * D + 8 * (c % CPR));
  }
  auto load_rows = [&](const uint16_t* __restrict__ src, int t, uint4 (&dst)[NCH]) {
    const uint16_t* __restrict__ tb = src + head_off + (size_t)t * tile_stride;
#pragma unroll
    for (int n = 0; n < NCH; ++n) {
      const int c = tid + NT * n;
      const int key = t * BK + c / CPR;
      uint4 v = make_uint4(0, 0, 0, 0);
      if ((NCH * NT == CHUNKS || c < CHUNKS) && key < S) v = *reinterpret_cast<const uint4*>(tb + loff[n]);
      dst[n] = v;
    }
  };
  auto store_rows = [&](uint16_t* dst, int ld, const uint4 (&src)[NCH]) {
#pragma unroll
    for (int n = 0; n < NCH; ++n) {
      const int c = tid + NT * n;
      if (NCH * NT == CHUNKS || c < CHUNKS) {
        const int row = c / CPR, cc = c % CPR;
        *reinterpret_cast<uint4*>(dst + row * ld + 8 * cc) = src[n];
      }
    }
  };
  // Highlight words of the tiles [t0, t0 + NT), one thread per tile, into the ring.  Every NT-th iteration refills
  // the half of the ring that the tile loop has left behind, so no lane carries mask state through the loop.
  auto fill_ring = [&](int t0) {
    const int t = t0 + tid;
    if (t < ntiles) {
      const uint8_t* mrow = st.mask + tok0 + (size_t)t * BK;
      unsigned long long bits = 0ull;
      if (t * BK + BK <= S && (reinterpret_cast<uintptr_t>(mrow) & 15) == 0) {
        uint4 mv[BK / 16];
#pragma unroll
        for (int q = 0; q < BK / 16; ++q) mv[q] = reinterpret_cast<const uint4*>(mrow)[q];
#pragma unroll
        for (int q = 0; q < BK / 16; ++q) {
          const uint32_t x4[4] = {mv[q].x, mv[q].y, mv[q].z, mv[q].w};
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            // non-zero test of the four bytes of x, gathered into four adjacent bits
            const uint32_t x = x4[w];
            const uint32_t y = ((x | ((x & 0x7f7f7f7fu) + 0x7f7f7f7fu)) & 0x80808080u) >> 7;
            const uint32_t nib = ((y * 0x00204081u) >> 21) & 0xfu;
            bits |= (unsigned long long)nib << (16 * q + 4 * w);
          }
        }
      } else {
        for (int k = 0; k < BK; ++k)
          if (t * BK + k < S && mrow[k] != 0) bits |= 1ull << k;
      }
      hlring[t % (2 * NT)] = bits;
    }
  };
  auto ring_word = [&](int t) -> unsigned long long {   // the same word in every lane, held in scalar registers
    const unsigned long long v = hlring[t % (2 * NT)];
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);          // the builtin is signed:
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));  // no sign extension here
    return ((unsigned long long)hi << 32) | lo;
  };

  // Edit the highlighted 16-key blocks of the K tile at Kb (LDS); one wave per block.
  auto edit_tile = [&](uint16_t* Kb, unsigned long long bits) {
    const int j = lane & 15, g = lane >> 4;
    constexpr int KS2 = D / 32;
    constexpr int MAXKR = SEKA_MAX_RANK / 32;
    const int nkr = Rpad / 32;
    for (int kblk = wave; kblk < BK / 16; kblk += NW) {
      const unsigned bits16 = (unsigned)((bits >> (16 * kblk)) & 0xffffull);
      if (bits16 == 0) continue;
      uint16_t* krow = Kb + (16 * kblk + j) * KLD + 8 * g;
      bf16x8 kreg[KS2];   // K^T as B operand: lane (col = key j, k = d = 32 s + 8 g + e)
#pragma unroll
      for (int s = 0; s < KS2; ++s) kreg[s] = *reinterpret_cast<const bf16x8*>(krow + 32 * s);
      const float mbit = ((bits16 >> j) & 1u) ? 1.f : 0.f;
      // Z^T = U^T K^T: A = U^T (row r, k = d) read transposed from the row-d layout
      const uint16_t* ut = UN + (size_t)(8 * g + (j >> 2)) * ULD + 4 * (j & 3);
      bf16x8 zb[MAXKR];
#pragma unroll
      for (int kr = 0; kr < MAXKR; ++kr) {
        if (kr < nkr) {
          float zc[8];
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            const int rb = 2 * kr + half;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < KS2; ++s) {
              const uint16_t* p = ut + (size_t)(32 * s) * ULD + 16 * rb;
              const bf16x8 ua = lds_read_tr_pair(p, p + 4 * ULD);
              acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ua, kreg[s], acc, 0, 0, 0);
            }
            const f32x4 c4 = *reinterpret_cast<const f32x4*>(cvec + 16 * rb + 4 * g);
#pragma unroll
            for (int i = 0; i < 4; ++i) zc[4 * half + i] = acc[i] * c4[i] * mbit;
          }
          bf16x8 z;   // next B operand: slot e <-> r = 32 kr + 16 (e / 4) + 4 g + e % 4
#pragma unroll
          for (int e = 0; e < 8; ++e) z[e] = (__bf16)zc[e];
          zb[kr] = z;
        }
      }
      // C^T = U (c .* Z^T): rows of U visited so that lane (j, g) receives d = 32 s + 8 g + e
#pragma unroll
      for (int s = 0; s < KS2; ++s) {
        float outv[8];
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const int d_row = 32 * s + 8 * (j >> 2) + 4 * half + (j & 3);
          f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int kr = 0; kr < MAXKR; ++kr) {
            if (kr < nkr) {
              const uint16_t* p = UN + (size_t)d_row * ULD + 32 * kr + 4 * g;
              const bf16x4 u0 = *reinterpret_cast<const bf16x4*>(p);
              const bf16x4 u1 = *reinterpret_cast<const bf16x4*>(p + 16);
              const bf16x8 ua = __builtin_shufflevector(u0, u1, 0, 1, 2, 3, 4, 5, 6, 7);
              acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ua, zb[kr], acc, 0, 0, 0);
            }
          }
#pragma unroll
          for (int i = 0; i < 4; ++i) outv[4 * half + i] = (float)kreg[s][4 * half + i] * (1.f + mbit * (kscale - 1.f)) + acc[i];
        }
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (__bf16)outv[e];
        *reinterpret_cast<bf16x8*>(krow + 32 * s) = o;
      }
    }
  };

  // ---- math pieces ----
  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float m_run = -1e30f, l_run = 0.f;
  const float c2 = a.scale * 1.4426950408889634f;   // p = exp2(s * c2 - m): m_run is in units of s * c2

  // S^T (64 keys x 32 rows) = K tile . Q^T
  auto qk_tile = [&](const uint16_t* Kb, f32x16& s0, f32x16& s1) {
#pragma unroll
    for (int r = 0; r < 16; ++r) { s0[r] = 0.f; s1[r] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(Kb + l32 * KLD + 16 * ks + 8 * hf);
      const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(Kb + (32 + l32) * KLD + 16 * ks + 8 * hf);
      s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qf[ks], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qf[ks], s1, 0, 0, 0);
    }
  };
  // causal mask of tile t, only where the tile reaches past the wave's first row
  auto causal_mask = [&](int t, f32x16& s0, f32x16& s1) {
    if (t * BK + BK - 1 > qw) {
      const int jbase = t * BK + 4 * hf;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int j = jbase + 8 * (r >> 2) + (r & 3);
        if (j > qi) s0[r] = -INFINITY;
        if (j + 32 > qi) s1[r] = -INFINITY;
      }
    }
  };
  // Online softmax of one 32-key block: scores -> packed P^T (two operands), reference exponent / sum, rescale of O
  // when the reference moved.  No row maximum in the common case: the probabilities are formed against the row's
  // reference exponent as it stands and their sum over this lane's 16 keys tells whether that was safe; a sum beyond
  // kSumLimit (or one that is not a number) means some score ran more than 2^8 ahead of the reference, and only then
  // is the block's maximum taken, the reference raised and the probabilities formed again (a handful of times per
  // row; the first block of a row always takes this turn, its reference starts at -1e30).  The PV product of a
  // block is accumulated before the next block's softmax, so a raise rescales exactly what was formed before it.
  constexpr float kSumLimit = 4096.f;          // 16 probabilities of at most 2^8
  constexpr float kSlack = 8.f;
  auto softmax_block = [&](const f32x16& sv, bf16x8 (&pb)[2]) {
    float pv[16];
    float lsum = 0.f;
    const float mneg = -m_run;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      pv[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[r], c2, mneg));
      lsum += pv[r];
    }
    if (__builtin_expect(__any(!(lsum <= kSumLimit)), 0)) {
      float mx = sv[0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sv[r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32)) * c2;                 // the other 16 keys of this row live in lane ^ 32
      const bool need = mx > m_run + kSlack;
      const float m_new = need ? mx : m_run;
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      m_run = m_new;
      lsum = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        pv[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[r], c2, -m_new));
        lsum += pv[r];
      }
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    }
    l_run += lsum;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      pb[0][e] = (__bf16)pv[e];
      pb[1][e] = (__bf16)pv[8 + e];
    }
  };
  // O^T += V^T P^T for the 32-key block `half` of the tile
  auto pv_block = [&](const uint16_t* Vb, int half, const bf16x8 (&pb)[2]) {
    const int li = lane & 15, grp = lane >> 4;
    const uint16_t* vbase = Vb + (32 * half + 4 * hf + (li >> 2)) * VLD + 16 * (grp & 1) + 4 * (li & 3);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const uint16_t* p = vbase + (16 * kb) * VLD + 32 * db;
        const bf16x8 va = lds_read_tr_pair(p, p + 8 * VLD);
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[kb], oacc[db], 0, 0, 0);
      }
    }
  };

  const bool wave_rows_exist = qw < S;
  const int tw_last = wave_rows_exist ? min(ntiles - 1, (qw + 31) / BK) : -1;   // last tile this wave computes on
  unsigned long long hl = 0ull;

  // ---------------- simple loop: load(t+1) | S(t), softmax(t), PV(t) | store(t+1) ----------------
  load_rows(Kg, 0, kpre);
  load_rows(Vg, 0, vpre);
  if (STEER && steer_on) fill_ring(0);
  store_rows(Kt, KLD, kpre);
  store_rows(Vt, VLD, vpre);
  __syncthreads();
  if (STEER && steer_on) hl = ring_word(0);
  if (STEER && hl != 0ull) {
    edit_tile(Kt, hl);
    __syncthreads();
  }
  for (int t = 0; t < ntiles; ++t) {
    const int buf = t & 1;
    const bool more = t + 1 < ntiles;
    if (more) {
      load_rows(Kg, t + 1, kpre);
      load_rows(Vg, t + 1, vpre);
      if (STEER && steer_on) {
        hl = ring_word(t + 1);                    // written at least one barrier ago
        if (__builtin_expect(t % NT == 0, 0)) fill_ring(t + NT);       // tiles t + NT .. t + 2 NT - 1 replace t - NT .. t - 1
      }
    }
    if (t <= tw_last) {
      f32x16 s0, s1;
      bf16x8 pb[2];
      qk_tile(Kt + buf * K_ELEMS, s0, s1);
      causal_mask(t, s0, s1);
      softmax_block(s0, pb);
      pv_block(Vt + buf * V_ELEMS, 0, pb);
      softmax_block(s1, pb);
      pv_block(Vt + buf * V_ELEMS, 1, pb);
    }
    if (more) {
      store_rows(Kt + (buf ^ 1) * K_ELEMS, KLD, kpre);
      store_rows(Vt + (buf ^ 1) * V_ELEMS, VLD, vpre);
    }
    __syncthreads();
    if (STEER && more && __builtin_expect(hl != 0ull, 0)) {
      edit_tile(Kt + (buf ^ 1) * K_ELEMS, hl);
      __syncthreads();
    }
  }

  // ---- epilogue ----
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  if (qi < S) {
    const float inv = 1.f / l_tot;
    uint16_t* op = Og + ((tok0 + qi) * a.Hq + hq) * D + 4 * hf;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        bf16x4 o4;
#pragma unroll
        for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(oacc[db][4 * q4 + e] * inv);
        *reinterpret_cast<uint2*>(op + 32 * db + 8 * q4) = __builtin_bit_cast(uint2, o4);
      }
    }
    if (a.lse && hf == 0) a.lse[lse_index(a, b, hq, tok0, qi)] = m_run * 0.6931471805599453f + logf(l_tot);
  }
}

}  // namespace seka
