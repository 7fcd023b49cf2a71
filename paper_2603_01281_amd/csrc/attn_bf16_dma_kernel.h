// bf16 causal GQA prefill attention for gfx950, head dimension 128, with the spectral key edit fused in
// (paper Sec. 2: logits q_i . k'_j / sqrt(d_k), k'_j = k_j + g P k_j for highlighted j; Sec. 3.3 for the
// blended P of AdaSEKA).  Flash-style: scores and edited keys never leave the CU.
//
// Same math mapping as attn_bf16_kernel.h (S^T = K Q^T with Q in registers, O^T = V^T P^T with P^T
// taken from the S^T accumulators and V^T fetched with transposing LDS reads); what differs is how
// tiles travel:
//   * K/V tiles (64 keys x 128) go from global memory straight into LDS with global_load_lds
//     (16 bytes per lane, no register staging), two tiles ahead of the math, into a ring of three
//     stages.  Completion is tracked with an explicit vmcnt wait followed by the per-tile barrier.
//   * A direct-to-LDS load writes 64 lanes x 16 bytes contiguously, so rows cannot be padded; bank
//     conflicts are avoided by choosing WHICH 16-byte chunk of a row each lane fetches (an XOR
//     swizzle of the chunk index with the row index): K chunks are swizzled by row & 15 (conflict-free
//     16-byte row reads), V chunks by 4 * (row & 3) (conflict-free transposing reads).
//   * The highlight mask is scanned once per workgroup into a per-tile 64-bit bitmap in LDS (wave
//     ballots), so the main loop has no vector-memory instruction other than the tile loads.
#pragma once
#include "common.h"

namespace seka {

constexpr int DMA_BK = 64;                       // keys per tile
constexpr int DMA_D = 128;
constexpr int DMA_TILE_BYTES = DMA_BK * DMA_D * 2;   // 16 KB
constexpr int DMA_STAGES = 3;

inline size_t attention_bf16_dma_smem_bytes(int S, bool steer, int Rpad) {
  size_t n = (size_t)2 * DMA_STAGES * DMA_TILE_BYTES;
  if (steer) {
    n += (size_t)DMA_D * (Rpad + 8) * 2 + (size_t)Rpad * 4;
    n += (size_t)((S + DMA_BK - 1) / DMA_BK) * 8;
  }
  return n;
}

typedef __attribute__((address_space(3))) s16x4* dma_lds_s16x4_ptr;
typedef __attribute__((address_space(3))) void* dma_lds_void_ptr;
typedef __attribute__((address_space(1))) const void* dma_glb_void_ptr;

__device__ __forceinline__ bf16x8 dma_read_tr_pair(const unsigned char* p0, const unsigned char* p1) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((dma_lds_s16x4_ptr)(p0));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((dma_lds_s16x4_ptr)(p1));
  const bf16x4 lo4 = __builtin_bit_cast(bf16x4, lo), hi4 = __builtin_bit_cast(bf16x4, hi);
  return __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
}

template <int N>
__device__ __forceinline__ void dma_wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Workgroup barrier that waits for this wave's LDS traffic only.  (__syncthreads() would also drain
// every outstanding vector-memory operation, i.e. the tile loads that are meant to stay in flight.)
__device__ __forceinline__ void dma_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// One direct-to-LDS load: every lane fetches 16 bytes from its own global address; the wave's 64 x 16
// bytes land contiguously at the (wave-uniform) LDS byte address lds_base.  Issued as inline assembly so
// that it stays outside the compiler's own vmcnt bookkeeping: the waits are placed by hand.
__device__ __forceinline__ void dma_load_16B(const void* gptr, uint32_t lds_base) {
  const uint32_t base = __builtin_amdgcn_readfirstlane(lds_base);   // wave-uniform by construction
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(base), "v"(gptr) : "memory", "m0");
}

// HPW heads x RBW row groups = waves per workgroup; every wave owns RPW blocks of 32 consecutive query rows.
// RPW = 2 halves the LDS traffic per flop (each K / V fragment read feeds two products) and needs the
// 512-register budget of one wave per SIMD (4 waves per workgroup).
template <int HPW, int RBW, int RPW, bool STEER>
__global__ __launch_bounds__(64 * HPW * RBW) void attention_bf16_dma_kernel(AttnArgs a, SteerArgs st, int Rpad) {
  constexpr int D = DMA_D;
  constexpr int NW = HPW * RBW;
  constexpr int NT = 64 * NW;
  constexpr int WR = 32 * RPW;          // query rows per wave
  constexpr int BQ = WR * RBW;
  constexpr int BK = DMA_BK;
  constexpr int KS = D / 16;
  constexpr int DB = D / 32;
  constexpr int SLOTS = DMA_TILE_BYTES / 1024;           // 1 KB (4 rows) per wave-wide load instruction
  constexpr int SPW = (SLOTS + NW - 1) / NW;             // load instructions per wave per tensor per tile
  constexpr int NLOAD = 2 * SPW;                         // vector-memory instructions per wave per tile

  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  unsigned char* Kst = smem;                                     // [3][16 KB] swizzled K tiles
  unsigned char* Vst = smem + DMA_STAGES * DMA_TILE_BYTES;       // [3][16 KB] swizzled V tiles
  uint16_t* UN = reinterpret_cast<uint16_t*>(smem + 2 * DMA_STAGES * DMA_TILE_BYTES);   // [D][Rpad+8] (STEER)
  const int ULD = Rpad + 8;
  float* cvec = reinterpret_cast<float*>(UN + (size_t)D * ULD);                          // [Rpad]
  unsigned long long* hlbits = reinterpret_cast<unsigned long long*>(cvec + Rpad);       // [tiles] (STEER)

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

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hf = lane >> 5;
  const int hq = hq0 + wave / RBW;
  const int qw = qb * BQ + WR * (wave % RBW);    // first query row of this wave
  const int qi0 = qw + l32;                      // this lane's query row in row block 0 (block rp: + 32 rp)

  const float gain = STEER ? st.gain[h] : 0.f;
  const bool steer_on = STEER && gain != 0.f;

  const int last_key = min(S, qb * BQ + BQ) - 1;
  const int ntiles = last_key / BK + 1;

  // ---- tile loads: global -> LDS, no registers in between ----
  // Slot s of a tile is LDS bytes [1024 s, 1024 s + 1024) = rows 4s..4s+3; lane l lands at row 4s + l/16,
  // chunk position l%16, and fetches the logical chunk that the swizzle assigns to that position.
  const int lrow = lane >> 4, lpos = lane & 15;
  const uint32_t kst_base = (uint32_t)(uintptr_t)(dma_lds_void_ptr)Kst;
  const uint32_t vst_base = (uint32_t)(uintptr_t)(dma_lds_void_ptr)Vst;
  auto issue_tile = [&](int t, int stage) {
#pragma unroll
    for (int n = 0; n < SPW; ++n) {
      const int slot = min(wave + NW * n, SLOTS - 1);          // surplus slots repeat the last one (same bytes)
      const int row = 4 * slot + lrow;
      const int key = min(t * BK + row, S - 1);                // rows past the end repeat the last key (finite data)
      const size_t goff = (((size_t)b * S + key) * a.Hkv + h) * D;
      const int ck = lpos ^ (row & 15);
      const int cv = lpos ^ (4 * (row & 3));
      dma_load_16B(Kg + goff + 8 * ck, kst_base + stage * DMA_TILE_BYTES + 1024 * slot);
      dma_load_16B(Vg + goff + 8 * cv, vst_base + stage * DMA_TILE_BYTES + 1024 * slot);
    }
  };

  issue_tile(0, 0);
  if (ntiles > 1) issue_tile(1, 1);

  // ---- Q fragments: B operand of S^T = K Q^T, lane (col = row qi, k = 16 ks + 8 hf + e) ----
  bf16x8 qf[RPW][KS];
#pragma unroll
  for (int rp = 0; rp < RPW; ++rp) {
    const int qi = qi0 + 32 * rp;
    const bool ok = qi < S;
    const uint16_t* qp = Qg + (((size_t)b * S + (ok ? qi : 0)) * a.Hq + hq) * D + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (ok) v = *reinterpret_cast<const uint4*>(qp + 16 * ks);
      qf[rp][ks] = __builtin_bit_cast(bf16x8, v);
    }
  }

  // ---- steering set-up: U_cat (row d, r contiguous), per-column coefficients, highlight bitmap ----
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
    for (int t = wave; t < ntiles; t += NW) {
      const int key = t * BK + lane;
      const int mk = key < S ? st.mask[(size_t)b * S + key] : 0;
      const unsigned long long bits = __ballot(mk != 0);
      if (lane == 0) hlbits[t] = bits;
    }
  }

  // Edit the highlighted 16-key blocks of the (swizzled) K tile at Kb; one wave per block.
  auto edit_tile = [&](unsigned char* Kb, unsigned long long bits) {
    const int j = lane & 15, g = lane >> 4;
    constexpr int KS2 = D / 32;
    constexpr int MAXKR = SEKA_MAX_RANK / 32;
    const int nkr = Rpad / 32;
    for (int kblk = wave; kblk < BK / 16; kblk += NW) {
      const unsigned bits16 = (unsigned)((bits >> (16 * kblk)) & 0xffffull);
      if (bits16 == 0) continue;
      unsigned char* krow = Kb + (16 * kblk + j) * 256;    // row & 15 == j
      bf16x8 kreg[KS2];   // K^T as B operand: lane (col = key j, k = d = 32 s + 8 g + e) = logical chunk 4 s + g
#pragma unroll
      for (int s = 0; s < KS2; ++s) kreg[s] = *reinterpret_cast<const bf16x8*>(krow + 16 * ((4 * s + g) ^ j));
      const float mbit = ((bits16 >> j) & 1u) ? 1.f : 0.f;
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
              const bf16x8 ua = dma_read_tr_pair(reinterpret_cast<const unsigned char*>(p),
                                                 reinterpret_cast<const unsigned char*>(p + 4 * ULD));
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
          for (int i = 0; i < 4; ++i) outv[4 * half + i] = (float)kreg[s][4 * half + i] + acc[i];
        }
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (__bf16)outv[e];
        *reinterpret_cast<bf16x8*>(krow + 16 * ((4 * s + g) ^ j)) = o;
      }
    }
  };

  // ---- math pieces ----
  f32x16 oacc[RPW][DB];
#pragma unroll
  for (int rp = 0; rp < RPW; ++rp)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[rp][db][r] = 0.f;
  float m_run[RPW], l_run[RPW];
#pragma unroll
  for (int rp = 0; rp < RPW; ++rp) { m_run[rp] = -1e30f; l_run[rp] = 0.f; }
  const float c2 = a.scale * 1.4426950408889634f;   // scores are kept unscaled; p = exp2((s - m) * c2)

  // K operand address of this lane inside a stage: row l32 (and l32 + 32), logical chunk 2 ks + hf,
  // physical chunk (2 ks + hf) ^ (l32 & 15)  ->  byte offset = kfix ^ (ks << 5)
  const int kfix = l32 * 256 + 16 * (hf ^ (l32 & 1)) + 32 * ((l32 & 15) >> 1);
  // S^T (64 keys x 32 RPW rows) = K tile . Q^T.  All 16 K fragments of the tile are requested before the
  // first product is issued, so the LDS latency is paid once per tile instead of once per product.
  auto qk_tile = [&](const unsigned char* Kb, f32x16 (&sc)[RPW][2]) {
    bf16x8 ka[KS][2];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const unsigned char* p = Kb + (kfix ^ (ks << 5));
      ka[ks][0] = *reinterpret_cast<const bf16x8*>(p);
      ka[ks][1] = *reinterpret_cast<const bf16x8*>(p + 32 * 256);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int rp = 0; rp < RPW; ++rp)
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int r = 0; r < 16; ++r) sc[rp][jb][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int rp = 0; rp < RPW; ++rp)
          sc[rp][jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks][jb], qf[rp][ks], sc[rp][jb], 0, 0, 0);
  };
  // causal mask of tile t for row block rp, only where the tile reaches past the block's first row
  auto causal_mask = [&](int t, int rp, f32x16 (&sc)[2]) {
    if (t * BK + BK - 1 > qw + 32 * rp) {
      const int qi = qi0 + 32 * rp;
      const int jbase = t * BK + 4 * hf;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int j = jbase + 8 * (r >> 2) + (r & 3);
        if (j > qi) sc[0][r] = -INFINITY;
        if (j + 32 > qi) sc[1][r] = -INFINITY;
      }
    }
  };
  // online softmax of one row block: scores -> packed P^T, running max / sum, rescale of O when a max moved
  auto softmax_tile = [&](int rp, f32x16 (&sc)[2], bf16x8 (&pb)[4]) {
    float mx = fmaxf(sc[0][0], sc[1][0]);
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, fmaxf(sc[0][r], sc[1][r]));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run[rp], mx);
    const float alpha = __builtin_amdgcn_exp2f((m_run[rp] - m_new) * c2);
    const float mc = m_new * c2;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      sc[0][r] = __builtin_amdgcn_exp2f(sc[0][r] * c2 - mc);
      sc[1][r] = __builtin_amdgcn_exp2f(sc[1][r] * c2 - mc);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      pb[0][e] = (__bf16)sc[0][e];
      pb[1][e] = (__bf16)sc[0][8 + e];
      pb[2][e] = (__bf16)sc[1][e];
      pb[3][e] = (__bf16)sc[1][8 + e];
    }
    // row sum of the rounded probabilities (the same values the PV product uses), two per instruction
    float lsum = 0.f;
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        const bf16x2 pp = {pb[kb][e], pb[kb][e + 1]};
        lsum = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, lsum, false);
      }
    l_run[rp] = l_run[rp] * alpha + lsum;
    m_run[rp] = m_new;
    if (__any(alpha != 1.f)) {   // rare after the first few tiles
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[rp][db][r] *= alpha;
    }
  };
  // V^T operand: lane (li, grp) supplies row 16 kb + 4 hf + (li >> 2) [+ 8], logical chunk 4 db + 2 (grp & 1) + ((li & 3) >> 1),
  // physical chunk 4 (db ^ q) + low with q = (li >> 2) & 3  ->  byte offset = vfix ^ (db << 6) (+ row immediates)
  const int li = lane & 15, grp = lane >> 4;
  const int vfix = (4 * hf + (li >> 2)) * 256 + 64 * ((li >> 2) & 3) + 16 * (2 * (grp & 1) + ((li & 3) >> 1)) + 8 * (li & 1);
  // The 16 V^T fragments are requested before the softmax so that their latency hides under it.
  auto v_fetch = [&](const unsigned char* Vb, bf16x8 (&vf)[4][DB]) {
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const unsigned char* p = Vb + (vfix ^ (db << 6)) + (16 * kb) * 256;
        vf[kb][db] = dma_read_tr_pair(p, p + 8 * 256);
      }
  };
  // O^T += V^T P^T
  auto pv_tile = [&](const bf16x8 (&vf)[4][DB], const bf16x8 (&pb)[RPW][4]) {
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int rp = 0; rp < RPW; ++rp)
          oacc[rp][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[kb][db], pb[rp][kb], oacc[rp][db], 0, 0, 0);
  };

  const bool wave_rows_exist = qw < S;
  const int tw_last = wave_rows_exist ? min(ntiles - 1, (qw + WR - 1) / BK) : -1;   // last tile this wave computes on

  // ---- prologue: tiles 0 and 1 are in flight; wait for them, edit tile 0 ----
  dma_wait_vmcnt<0>();   // also covers the Q, U and mask loads issued after the tile loads
#pragma unroll
  for (int rp = 0; rp < RPW; ++rp)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qf[rp][ks]));   // pin the compiler's own wait for Q here, not in the loop
  dma_barrier();
  if (STEER && steer_on) {
    const unsigned long long hl = hlbits[0];
    if (hl != 0ull) {
      edit_tile(Kst, hl);
      dma_barrier();
    }
  }

  int stage = 0;   // t % 3
  for (int t = 0; t < ntiles; ++t) {
    const int stage1 = stage == 2 ? 0 : stage + 1;
    const int stage2 = stage1 == 2 ? 0 : stage1 + 1;
    const bool issue = t + 2 < ntiles;
    if (issue) issue_tile(t + 2, stage2);

    if (t <= tw_last) {
      f32x16 sc[RPW][2];
      bf16x8 pb[RPW][4];
      bf16x8 vf[4][DB];
      qk_tile(Kst + stage * DMA_TILE_BYTES, sc);
      v_fetch(Vst + stage * DMA_TILE_BYTES, vf);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int rp = 0; rp < RPW; ++rp) {
        causal_mask(t, rp, sc[rp]);
        softmax_tile(rp, sc[rp], pb[rp]);
      }
      __builtin_amdgcn_sched_barrier(0);
      pv_tile(vf, pb);
    }

    if (t + 1 < ntiles) {
      if (issue) dma_wait_vmcnt<NLOAD>(); else dma_wait_vmcnt<0>();   // this wave's part of tile t+1 has landed
    }
    dma_barrier();                                                  // ... and everybody else's
    if (STEER && steer_on && t + 1 < ntiles) {
      const unsigned long long hl = hlbits[t + 1];
      if (hl != 0ull) {
        edit_tile(Kst + stage1 * DMA_TILE_BYTES, hl);
        dma_barrier();
      }
    }
    stage = stage1;
  }

  // ---- epilogue ----
#pragma unroll
  for (int rp = 0; rp < RPW; ++rp) {
    const int qi = qi0 + 32 * rp;
    const float l_tot = l_run[rp] + __shfl_xor(l_run[rp], 32);
    if (qi < S) {
      const float inv = 1.f / l_tot;
      uint16_t* op = Og + (((size_t)b * S + qi) * a.Hq + hq) * D + 4 * hf;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          bf16x4 o4;
#pragma unroll
          for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(oacc[rp][db][4 * q4 + e] * inv);
          *reinterpret_cast<uint2*>(op + 32 * db + 8 * q4) = __builtin_bit_cast(uint2, o4);
        }
      }
      if (a.lse && hf == 0) a.lse[((size_t)b * a.Hq + hq) * S + qi] = m_run[rp] * a.scale + logf(l_tot);
    }
  }
}

}  // namespace seka
