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
//                   keys is permuted identically on the V side), A = V^T fragments read from LDS
//                   either with the transposing LDS read (VMODE 0) or from a tile that was
//                   stored transposed (VMODE 1).
// Key edit (STEER): after a K tile lands in LDS, a wave ballot of its mask bytes tells whether it
//   holds highlighted tokens; if so, 16-key blocks with highlights get
//   Z^T = U_cat^T K^T and K'^T = K^T + U_cat (c .* Z^T) on 16x16x32 MFMAs, written back to LDS as bf16.
#pragma once
#include "common.h"

namespace seka {

constexpr int ATT_BK = 64;   // keys per tile

__host__ __device__ constexpr int att_kld(int D) { return D + 8; }                       // K tile row stride
__host__ __device__ constexpr int att_v_elems(int D, int vmode) { return vmode == 0 ? ATT_BK * (D + 8) : D * (ATT_BK + 8); }

inline size_t attention_bf16_smem_bytes(int D, int vmode, bool steer, int Rpad) {
  size_t n = 2 * ((size_t)ATT_BK * att_kld(D) + att_v_elems(D, vmode)) * 2;
  if (steer) n += ((size_t)Rpad * (D + 8) + (size_t)D * (Rpad + 8)) * 2 + (size_t)Rpad * 4;
  return n;
}

__device__ __forceinline__ int att_perm_col(int r) {
  return (r & ~31) + 8 * ((r & 15) >> 2) + 4 * ((r & 31) >> 4) + (r & 3);
}

__device__ __forceinline__ int att_vslot(int j) {
  // position of key j inside a transposed V row so that a lane's 8 contraction slots are contiguous
  const int j16 = j & 15;
  return (j & ~15) + 8 * ((j16 >> 2) & 1) + 4 * (j16 >> 3) + (j16 & 3);
}

template <int D, int HPW, int RB, bool STEER, int VMODE>
__global__ __launch_bounds__(64 * HPW * RB) void attention_bf16_kernel(AttnArgs a, SteerArgs st, int Rpad) {
  constexpr int NW = HPW * RB;
  constexpr int NT = 64 * NW;
  constexpr int BQ = 32 * RB;
  constexpr int BK = ATT_BK;
  constexpr int KLD = att_kld(D);
  constexpr int VLD = VMODE == 0 ? D + 8 : BK + 8;
  constexpr int K_ELEMS = BK * KLD;
  constexpr int V_ELEMS = att_v_elems(D, VMODE);
  constexpr int KS = D / 16;          // contraction steps of S^T = K Q^T
  constexpr int DB = D / 32;          // 32-row blocks of O^T
  constexpr int CPR = D / 8;          // 16-byte chunks per tile row
  constexpr int CHUNKS = BK * CPR;
  constexpr int NCH = (CHUNKS + NT - 1) / NT;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* Kt = reinterpret_cast<uint16_t*>(smem);            // [2][BK][KLD]
  uint16_t* Vt = Kt + 2 * K_ELEMS;                             // [2][V_ELEMS]
  uint16_t* UT = Vt + 2 * V_ELEMS;                             // [Rpad][D+8]      (STEER)
  uint16_t* UN = UT + (size_t)Rpad * (D + 8);                  // [D][Rpad+8]      (STEER, columns permuted)
  float* cvec = reinterpret_cast<float*>(UN + (size_t)D * (Rpad + 8));

  const uint16_t* __restrict__ Qg = static_cast<const uint16_t*>(a.Q);
  const uint16_t* __restrict__ Kg = static_cast<const uint16_t*>(a.K);
  const uint16_t* __restrict__ Vg = static_cast<const uint16_t*>(a.V);
  uint16_t* __restrict__ Og = static_cast<uint16_t*>(a.O);

  const int S = a.S;
  const int G = a.Hq / a.Hkv;
  const int nHC = a.Hq / HPW;
  const int nQB = (S + BQ - 1) / BQ;
  const int per_qb = nHC * a.B;
  const int qb = nQB - 1 - (int)(blockIdx.x / per_qb);
  const int rem = blockIdx.x % per_qb;
  const int b = rem / nHC, hc = rem % nHC;
  const int hq0 = hc * HPW;
  const int h = hq0 / G;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hf = lane >> 5;
  const int hq = hq0 + wave / RB;
  const int qw = qb * BQ + 32 * (wave % RB);     // first query row of this wave
  const int qi = qw + l32;                       // this lane's query row

  const float gain = STEER ? st.gain[h] : 0.f;
  const bool steer_on = STEER && gain != 0.f;

  // ---- Q fragments: B operand of S^T = K Q^T, lane (col = row qi, k = 16 ks + 8 hf + e) ----
  bf16x8 qf[KS];
  {
    const bool ok = qi < S;
    const uint16_t* qp = Qg + (((size_t)b * S + (ok ? qi : 0)) * a.Hq + hq) * D + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (ok) v = *reinterpret_cast<const uint4*>(qp + 16 * ks);
      qf[ks] = __builtin_bit_cast(bf16x8, v);
    }
  }

  // ---- stage U (both orientations) and coefficients ----
  if (STEER && steer_on) {
    const int R = st.M * st.r;
    if (R != Rpad) {
      for (int i = tid; i < (Rpad - R) * (D + 8); i += NT) UT[(size_t)R * (D + 8) + i] = 0;
      for (int i = tid; i < D * (Rpad + 8); i += NT) UN[i] = 0;
      __syncthreads();
    }
    const uint16_t* Uh = static_cast<const uint16_t*>(st.U) + (size_t)h * st.M * D * st.r;
    const int r8 = st.r / 8;
    const int total = st.M * D * r8;
    for (int idx = tid; idx < total; idx += NT) {
      const int m = idx / (D * r8), rm = idx % (D * r8);
      const int d = rm / r8, v = rm % r8;
      const uint4 u = *reinterpret_cast<const uint4*>(Uh + ((size_t)m * D + d) * st.r + 8 * v);
      const int r0 = m * st.r + 8 * v;
      const uint32_t wds[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
      for (int e = 0; e < 8; ++e)
        UT[(size_t)(r0 + e) * (D + 8) + d] = (uint16_t)((wds[e >> 1] >> (16 * (e & 1))) & 0xffffu);
      *reinterpret_cast<uint2*>(UN + (size_t)d * (Rpad + 8) + att_perm_col(r0)) = make_uint2(u.x, u.y);
      *reinterpret_cast<uint2*>(UN + (size_t)d * (Rpad + 8) + att_perm_col(r0 + 4)) = make_uint2(u.z, u.w);
    }
    for (int r = tid; r < Rpad; r += NT) {
      float c = 0.f;
      if (r < R) c = gain * (st.w ? st.w[((size_t)b * a.Hkv + h) * st.M + r / st.r] : 1.f);
      cvec[r] = c;
    }
    // visibility of UT/UN/cvec is ensured by the barrier that follows the first tile write
  }

  const int last_key = min(S, qb * BQ + BQ) - 1;
  const int ntiles = last_key / BK + 1;

  uint4 kpre[NCH], vpre[NCH];
  int mpre = 0;

  auto load_tile = [&](int t) {
#pragma unroll
    for (int n = 0; n < NCH; ++n) {
      const int c = tid + NT * n;
      const int row = c / CPR, cc = c % CPR;
      const int key = t * BK + row;
      uint4 kv = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
      if ((NCH * NT == CHUNKS || c < CHUNKS) && key < S) {
        const size_t off = (((size_t)b * S + key) * a.Hkv + h) * D + 8 * cc;
        kv = *reinterpret_cast<const uint4*>(Kg + off);
        vv = *reinterpret_cast<const uint4*>(Vg + off);
      }
      kpre[n] = kv;
      vpre[n] = vv;
    }
    if (STEER && steer_on) {
      const int key = t * BK + lane;
      mpre = key < S ? st.mask[(size_t)b * S + key] : 0;
    }
  };

  auto store_tile = [&](int buf) {
    uint16_t* Kb = Kt + buf * K_ELEMS;
    uint16_t* Vb = Vt + buf * V_ELEMS;
#pragma unroll
    for (int n = 0; n < NCH; ++n) {
      const int c = tid + NT * n;
      if (NCH * NT == CHUNKS || c < CHUNKS) {
        const int row = c / CPR, cc = c % CPR;
        *reinterpret_cast<uint4*>(Kb + row * KLD + 8 * cc) = kpre[n];
        if (VMODE == 0) {
          *reinterpret_cast<uint4*>(Vb + row * VLD + 8 * cc) = vpre[n];
        } else {
          const uint32_t wds[4] = {vpre[n].x, vpre[n].y, vpre[n].z, vpre[n].w};
          const int slot = att_vslot(row);
#pragma unroll
          for (int e = 0; e < 8; ++e)
            Vb[(8 * cc + e) * VLD + slot] = (uint16_t)((wds[e >> 1] >> (16 * (e & 1))) & 0xffffu);
        }
      }
    }
  };

  // Edit the highlighted 16-key blocks of the K tile in LDS buffer `buf`.
  auto edit_tile = [&](int buf, unsigned long long bits) {
    uint16_t* Kb = Kt + buf * K_ELEMS;
    const int j = lane & 15, g = lane >> 4;
    constexpr int KS2 = D / 32;
    constexpr int MAXKR = SEKA_MAX_RANK / 32;
    const int nkr = Rpad / 32;
    for (int kblk = wave; kblk < BK / 16; kblk += NW) {
      const unsigned bits16 = (unsigned)((bits >> (16 * kblk)) & 0xffffull);
      if (bits16 == 0) continue;
      uint16_t* krow = Kb + (16 * kblk + j) * KLD + 8 * g;
      bf16x8 kreg[KS2];
#pragma unroll
      for (int s = 0; s < KS2; ++s) kreg[s] = *reinterpret_cast<const bf16x8*>(krow + 32 * s);
      const float mbit = ((bits16 >> j) & 1u) ? 1.f : 0.f;
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
              const bf16x8 ua = *reinterpret_cast<const bf16x8*>(UT + (size_t)(16 * rb + j) * (D + 8) + 32 * s + 8 * g);
              acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ua, kreg[s], acc, 0, 0, 0);
            }
            const f32x4 c4 = *reinterpret_cast<const f32x4*>(cvec + 16 * rb + 4 * g);
#pragma unroll
            for (int i = 0; i < 4; ++i) zc[4 * half + i] = acc[i] * c4[i] * mbit;
          }
          bf16x8 z;
#pragma unroll
          for (int e = 0; e < 8; ++e) z[e] = (__bf16)zc[e];
          zb[kr] = z;
        }
      }
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
              const bf16x8 ua = *reinterpret_cast<const bf16x8*>(UN + (size_t)d_row * (Rpad + 8) + 32 * kr + 8 * g);
              acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ua, zb[kr], acc, 0, 0, 0);
            }
          }
#pragma unroll
          for (int i = 0; i < 4; ++i) outv[4 * half + i] = (float)kreg[s][4 * half + i] + acc[i];
        }
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (__bf16)outv[e];
        *reinterpret_cast<bf16x8*>(krow + 32 * s) = o;
      }
    }
  };

  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float m_run = -1e30f, l_run = 0.f;
  const float c2 = a.scale * 1.4426950408889634f;   // scores are kept unscaled; exp2((s - m) * c2)

  // ---- prologue: tile 0 ----
  load_tile(0);
  store_tile(0);
  unsigned long long hl = (STEER && steer_on) ? __ballot(mpre != 0) : 0ull;
  __syncthreads();
  if (STEER && hl != 0ull) {
    edit_tile(0, hl);
    __syncthreads();
  }

  const bool wave_rows_exist = qw < S;
  for (int t = 0; t < ntiles; ++t) {
    const int buf = t & 1;
    const bool more = t + 1 < ntiles;
    if (more) load_tile(t + 1);

    const bool active = wave_rows_exist && (t * BK <= qw + 31);
    if (active) {
      const uint16_t* Kb = Kt + buf * K_ELEMS;
      const uint16_t* Vb = Vt + buf * V_ELEMS;
      f32x16 s0, s1;
#pragma unroll
      for (int r = 0; r < 16; ++r) { s0[r] = 0.f; s1[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(Kb + l32 * KLD + 16 * ks + 8 * hf);
        const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(Kb + (32 + l32) * KLD + 16 * ks + 8 * hf);
        s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qf[ks], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qf[ks], s1, 0, 0, 0);
      }
      if (t * BK + BK - 1 > qw) {   // tile reaches past this wave's first row: causal mask
        const int jbase = t * BK + 4 * hf;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int j = jbase + 8 * (r >> 2) + (r & 3);
          if (j > qi) s0[r] = -INFINITY;
          if (j + 32 > qi) s1[r] = -INFINITY;
        }
      }
      float mx = s0[0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s0[r]);
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s1[r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run, mx);
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c2);
      const float mc = m_new * c2;
      float lsum = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        s0[r] = __builtin_amdgcn_exp2f(s0[r] * c2 - mc);
        s1[r] = __builtin_amdgcn_exp2f(s1[r] * c2 - mc);
        lsum += s0[r] + s1[r];
      }
      l_run = l_run * alpha + lsum;
      m_run = m_new;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;

      bf16x8 pb[4];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        pb[0][e] = (__bf16)s0[e];
        pb[1][e] = (__bf16)s0[8 + e];
        pb[2][e] = (__bf16)s1[e];
        pb[3][e] = (__bf16)s1[8 + e];
      }
#pragma unroll
      for (int kb = 0; kb < 4; ++kb) {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          bf16x8 va;
          if (VMODE == 0) {
            const int li = lane & 15, grp = lane >> 4;
            const int col = 32 * db + 16 * (grp & 1) + 4 * (li & 3);
            const int jrow = 16 * kb + 4 * hf + (li >> 2);
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) s16x4*)(Vb + jrow * VLD + col));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) s16x4*)(Vb + (jrow + 8) * VLD + col));
            const bf16x4 lo4 = __builtin_bit_cast(bf16x4, lo), hi4 = __builtin_bit_cast(bf16x4, hi);
            va = __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
          } else {
            va = *reinterpret_cast<const bf16x8*>(Vb + (32 * db + l32) * VLD + 16 * kb + 8 * hf);
          }
          oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[kb], oacc[db], 0, 0, 0);
        }
      }
    }

    if (more) {
      store_tile(buf ^ 1);
      hl = (STEER && steer_on) ? __ballot(mpre != 0) : 0ull;
    }
    __syncthreads();
    if (STEER && more && hl != 0ull) {
      edit_tile(buf ^ 1, hl);
      __syncthreads();
    }
  }

  // ---- epilogue ----
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  if (qi < S) {
    const float inv = 1.f / l_tot;
    uint16_t* op = Og + (((size_t)b * S + qi) * a.Hq + hq) * D + 4 * hf;
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
    if (a.lse && hf == 0) a.lse[((size_t)b * a.Hq + hq) * S + qi] = m_run * a.scale + __logf(l_tot);
  }
}

}  // namespace seka
