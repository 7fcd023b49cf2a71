// bf16 causal GQA prefill attention for gfx950, head dimension 128, with the spectral key edit fused in
// (paper Sec. 2: logits q_i . k'_j / sqrt(d_k), k'_j = k_j + g P k_j for highlighted j; Sec. 3.3 for the
// blended P of AdaSEKA).  Flash-style: scores and edited keys never leave the CU.  Software-pipelined,
// 32 query rows per wave; attn_bf16_lds_dma.h describes how the tiles travel.
//
// Math mapping: S^T = K Q^T on v_mfma_f32_32x32x16_bf16 with A = K rows from LDS and B = Q fragments resident
// in registers, so each lane owns one query row and 16 of a block's 32 keys (row maximum and sum are in-lane
// plus one exchange with lane ^ 32); O^T = V^T P^T with B = P^T taken straight from the S^T accumulators (the
// contraction order over keys is permuted identically on the V side) and A = V^T fetched from the row-major V
// tile with the transposing LDS read ds_read_b64_tr_b16.  A workgroup is HPW query heads of one KV group x
// RBW blocks of 32 query rows, all sharing the K/V tiles (and the edit) of that KV head.
//
// What bounds this kernel on gfx950 is the SIMD's vector issue port and, behind it, the chip's power limit, not the
// matrix pipe alone: a 32x32x16 bf16 MFMA keeps the port from issuing other vector work for about 22 of its 32
// cycles, a plain vector instruction takes 3 to 5 cycles of it, the transcendental unit accepts one exponential
// about every 10 cycles, and the two waves of a SIMD queue on the same port.  Consequences:
//   * every vector instruction in the loop that is not softmax arithmetic is removed: LDS read addresses
//     are a register plus an immediate (the loop is unrolled over the three ring stages so that stage
//     offsets are compile-time constants), tile loads take a scalar base plus a per-lane offset computed
//     once, and the common case of a step computes no row maximum at all (see `step`): 48 vector instructions
//     per 16 MFMAs;
//   * MFMAs and vector instructions alternate in program order, and every MFMA has vector work beside it:
//     a step handles three consecutive 32-key blocks at once: the S^T products of the next block, the softmax
//     of the current one and the PV products of the previous one (whose probabilities were formed one step
//     earlier), with one exponential per MFMA.
// The softmax runs per 32-key block (half a tile), which halves the score registers the pipeline needs.
// K tiles live in a ring of three LDS stages; V in a ring of six half tiles that runs half a tile behind K
// (see the tile loads).  K(t+2) and the V blocks 2t+3, 2t+4 are requested during iteration t (in the hot loop
// between its two steps, so that the first step's LDS reads follow the per-tile barrier directly).  The steering
// event of tile t+2 (highlighted keys only) sits between the two steps of iteration t + 1: at rank <= 32 the
// coordinates c .* U^T k of its keys are computed and the scores of that tile get a rank-32 correction against
// U^T q afterwards (score-side form, the tile itself stays as loaded); at larger ranks the keys are edited in LDS.
#pragma once
#include <type_traits>

#include "attn_bf16_lds_dma.h"

namespace seka {

// LDS beyond the two tile rings (steered kernels): the edit's matrix operand, the per-column coefficients, one
// 64-bit highlight word per tile and, for rank <= 32, the buffers of the score-side form.
// Rank <= 32 (nkr == 1): the edit is applied to the scores, s_ij = q_i . k_j + (U^T q_i) . (c .* U^T k_j) for
// highlighted j (paper Sec. 2, the equivalence of key-side and score-side control, Eq. 5): U_cat is stored once, as
// the operand of U_cat^T K^T; the coordinates c .* U^T k of a tile's keys go to one of two 64 x 32 bf16 buffers
// (rows padded to 80 bytes: conflict-free 16-byte row reads), and every wave keeps U^T q of its 32 rows as two
// MFMA operands (2 KB).  Larger ranks: the keys themselves are edited with the dense D x D matrix
// g P = U_cat diag(c) U_cat^T, built once per workgroup; at rank >= 64 one product with it moves no more operand
// bytes than two low-rank products and has no intermediate.  Either way the operands are stored in the order the
// MFMAs read them (one 16-byte LDS read per lane and operand).
constexpr int PIPE_Z_LD = 80;                       // bytes per key in a coordinate buffer
constexpr int PIPE_Z_BYTES = DMA_BK * PIPE_Z_LD;    // one buffer
constexpr int PIPE_QT_BYTES = 2048;                 // U^T q of one wave: [2 k-slices][64 lanes][8] bf16
inline size_t attention_bf16_pipe_smem_bytes(int S, bool steer, int nkr, int nwaves) {
  size_t n = (size_t)2 * DMA_STAGES * DMA_TILE_BYTES;
  if (steer) {
    const int Rpad = 32 * nkr;
    n += nkr == 1 ? (size_t)DMA_D * Rpad * 2 : (size_t)DMA_D * DMA_D * 2;
    n += (size_t)Rpad * 4;
    if (nkr == 1) n += (size_t)2 * PIPE_Z_BYTES + (size_t)nwaves * PIPE_QT_BYTES;
    n += (size_t)((S + DMA_BK - 1) / DMA_BK) * 8;
  }
  return n;
}

typedef __attribute__((address_space(3))) const bf16x8* pipe_lds_bf16x8_ptr;

// The compiler does not insert, before inline assembly, the wait states an MFMA result needs before a vector
// instruction may read it.  pipe_max3 is only used on scores whose MFMAs are provably far behind: in the
// pipelined loop they belong to the previous step (a scheduling barrier and eight MFMAs apart); elsewhere
// pipe_mfma_result_guard() is placed between the product and the maximum.
__device__ __forceinline__ void pipe_mfma_result_guard(f32x16& acc) {
  asm volatile("s_nop 15\n\ts_nop 15" : "+v"(acc));
}

__device__ __forceinline__ float pipe_max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// Direct-to-LDS load with a scalar 64-bit base and a 32-bit per-lane byte offset.
__device__ __forceinline__ void pipe_load_16B(const void* base, uint32_t lane_off, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(lane_off), "s"(base)
               : "memory", "m0");
}

// HPW heads x RBW row groups = waves per workgroup; every wave owns RPW blocks of 32 consecutive query rows.
// RPW = 2 (four waves, one per SIMD, 512-register budget) reads every K / V fragment once for two products.
// NKR: rank of the concatenated basis in blocks of 32 columns (compile-time so that the edit is straight-line code).
template <int HPW, int RBW, int RPW, bool STEER, int NKR>
__global__ __launch_bounds__(64 * HPW * RBW) void attention_bf16_pipe_kernel(AttnArgs a, SteerArgs st) {
  constexpr int D = DMA_D;
  constexpr int NW = HPW * RBW;
  constexpr int NT = 64 * NW;
  constexpr int WR = 32 * RPW;
  constexpr int BQ = WR * RBW;
  constexpr int BK = DMA_BK;
  constexpr int KS = D / 16;
  constexpr int DB = D / 32;
  constexpr int SLOTS = DMA_TILE_BYTES / 1024;
  constexpr int SPW = (SLOTS + NW - 1) / NW;             // load instructions per wave per tensor per tile
  constexpr int TB = DMA_TILE_BYTES;

  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  unsigned char* Kst = smem;                                     // [3][16 KB] swizzled K tiles
  unsigned char* Vst = smem + DMA_STAGES * TB;                   // [3][16 KB] swizzled V tiles
  constexpr int Rpad = 32 * NKR;
  constexpr bool DENSE = NKR >= 2;         // edit with the dense matrix g P (see attention_bf16_pipe_smem_bytes)
  constexpr bool kEventsInHot = STEER && (!DENSE || NW == 8);   // steering events handled inside the hot loop (see the tile loop)
  uint16_t* UN = reinterpret_cast<uint16_t*>(smem + 2 * DMA_STAGES * TB);
  uint16_t* U1 = UN;                       // low rank: operand (rb, s) of U_cat^T K^T: [2][4][64 lanes][8]
  uint16_t* AP = UN;                       // dense: operand (s_out, half, ks) of (g P) K^T: [4][2][4][64 lanes][8]
  float* cvec = reinterpret_cast<float*>(UN + (DENSE ? (size_t)D * D : (size_t)D * Rpad));   // [Rpad]
  unsigned char* zbuf = reinterpret_cast<unsigned char*>(cvec + Rpad);     // low rank: [2][64 keys][80 B] coordinates
  unsigned char* qtbuf = zbuf + 2 * PIPE_Z_BYTES;                          // low rank: [NW][2][64 lanes][8] U^T q
  unsigned long long* hlbits = reinterpret_cast<unsigned long long*>(      // [tiles] (STEER)
      DENSE ? reinterpret_cast<unsigned char*>(cvec + Rpad) : qtbuf + NW * PIPE_QT_BYTES);

  const uint16_t* __restrict__ Qg = static_cast<const uint16_t*>(a.Q);
  const uint16_t* __restrict__ Kg = static_cast<const uint16_t*>(a.K);
  const uint16_t* __restrict__ Vg = static_cast<const uint16_t*>(a.V);
  uint16_t* __restrict__ Og = static_cast<uint16_t*>(a.O);

  const int Scap = a.S;                      // tokens per prompt in memory (strides, launch grid)
  const int G = a.Hq / a.Hkv;
  const int nHC = a.Hq / HPW;
  const int nQB = (Scap + BQ - 1) / BQ;
  // A workgroup handles two blocks of query rows of one (batch, head group), one after the other: block
  // nQB - 1 - p and block p.  Every workgroup then scans nQB + 1 key tiles (no imbalance from causality), the
  // steering set-up is done once for both, and the first loads of the second block overlap the first block's
  // output stores.  (With nQB odd the middle block is on its own.)
  // blockIdx = (prompt, pair, head chunk), head chunk fastest: workgroups are dispatched round-robin over the
  // XCDs in index order, so with 8 head chunks an XCD's L2 serves one KV head, and the workgroups resident at the
  // same time walk the K / V tiles of the same prompt from tile 0 on, at the same pace.
  const int npairs = (nQB + 1) / 2;
  const int hc = (int)(blockIdx.x % nHC);
  const int bp = (int)(blockIdx.x / nHC);
  const int b = bp / npairs, pair = bp % npairs;
  const int hq0 = hc * HPW;
  const int h = hq0 / G;
  size_t tok0;                               // first token of this prompt in the tensors
  int S;                                     // this prompt's length: rows and keys beyond it do not exist
  prompt_extent(a, b, tok0, S);
  int npass = (nQB - 1 - pair != pair) ? 2 : 1;
  int qb = nQB - 1 - pair;
  if (qb * BQ >= S) {                        // the later block lies beyond this prompt's end
    qb = pair;
    npass = 1;
  }
  if (qb * BQ >= S) return;                  // workgroup-uniform, before any barrier

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hf = lane >> 5;
  const int hq = hq0 + wave / RBW;
  int qw = qb * BQ + WR * (wave % RBW);    // first query row of this wave
  int qi0 = qw + l32;                      // this lane's query row in row block 0 (block rp: + 32 rp)

  const float gain = STEER ? st.gain[h] : 0.f;
  const float kscale = STEER ? st.kscale[h] : 1.f;
  const bool steer_on = STEER && gain != 0.f;

  int last_key = min(S, qb * BQ + BQ) - 1;
  int ntiles = last_key / BK + 1;          // the first block is the later one: its tile count bounds the second's

  // ---- tile loads: scalar tile base + per-lane offset fixed for the whole kernel ----
  // Slot s of a tile is LDS bytes [1024 s, 1024 s + 1024) = rows 4s..4s+3; lane l lands at row 4s + l/16,
  // chunk position l%16, and fetches the logical chunk that the swizzle assigns to that position.
  const uint32_t rowbytes = (uint32_t)a.Hkv * D * 2;
  const uint32_t kst_base = (uint32_t)(uintptr_t)(dma_lds_void_ptr)Kst;
  const uint32_t vst_base = (uint32_t)(uintptr_t)(dma_lds_void_ptr)Vst;
  // V travels in units of half a tile, one half tile behind K: "shifted tile" t = rows [64 t - 32, 64 t + 32) = the
  // 32-key blocks 2t - 1 and 2t, and block j lives at ring position j % 6 (8 KB each; tile t = positions 2t % 6,
  // 2t % 6 + 1 as before).  The PV product of a block runs one step after its softmax (see `step`), so the last
  // block of tile t is still being read while the loads of iteration t + 1 are in flight; shifting the unit by
  // half a tile makes every load overwrite only blocks that all waves are done with.
  constexpr int HB = TB / 2;              // bytes of a 32-key block
  int slot_row[SPW];          // first LDS row of this lane in slot n
  uint32_t koff[SPW], voff[SPW], slot_lds[SPW], vslot_lds[SPW];
  bool vslot_hi[SPW];         // slot n belongs to the second block of a shifted tile (wave-uniform)
#pragma unroll
  for (int n = 0; n < SPW; ++n) {
    const int slot = min(wave + NW * n, SLOTS - 1);      // surplus slots repeat the last one (same bytes)
    const int row = 4 * slot + (lane >> 4);
    slot_row[n] = row;
    slot_lds[n] = 1024u * slot;
    vslot_lds[n] = 1024u * (slot & (SLOTS / 2 - 1));
    vslot_hi[n] = slot >= SLOTS / 2;
    koff[n] = row * rowbytes + 16u * ((lane & 15) ^ (row & 15));
    voff[n] = row * rowbytes + 16u * ((lane & 15) ^ (4 * (row & 3)));
  }
  const size_t head_off = (tok0 * a.Hkv + h) * D * 2;          // bytes to this (batch, KV head), token 0
  const unsigned char* Kbytes = reinterpret_cast<const unsigned char*>(Kg) + head_off;
  const unsigned char* Vbytes = reinterpret_cast<const unsigned char*>(Vg) + head_off;
  // ring position (byte offset inside the V ring) of 32-key block j >= -1
  auto vpos = [&](int j) __attribute__((always_inline)) -> uint32_t { return (uint32_t)((j + 6) % 6) * HB; };
  // K tile t into its ring stage.  `full`: every row of the tile exists (no clamping, offsets fixed per lane).
  // Otherwise rows past the prompt's end repeat its last key (finite data that the causal mask hides); offsets
  // are then taken from token 0 so that they never go negative.
  auto issue_k_to = [&](auto full_c, int t, uint32_t lds_stage_base) __attribute__((always_inline)) {
    if (decltype(full_c)::value || t * BK + BK <= S) {
      const unsigned char* tile = Kbytes + (size_t)t * BK * rowbytes;
#pragma unroll
      for (int n = 0; n < SPW; ++n) pipe_load_16B(tile, koff[n], lds_stage_base + slot_lds[n]);
    } else {
#pragma unroll
      for (int n = 0; n < SPW; ++n) {
        uint32_t ko = koff[n];
        asm volatile("" : "+v"(ko));     // formed here, not hoisted out of the tile loops into a register (or scratch slot) of its own
        pipe_load_16B(Kbytes, ko + (uint32_t)(min(t * BK + slot_row[n], S - 1) - slot_row[n]) * rowbytes,
                      lds_stage_base + slot_lds[n]);
      }
    }
  };
  // Shifted V tile t: block 2t - 1 to ring byte offset posA, block 2t to posB.
  auto issue_v_to = [&](auto full_c, int t, uint32_t posA, uint32_t posB) __attribute__((always_inline)) {
    const int first = t * BK - BK / 2;
    if (decltype(full_c)::value || (first >= 0 && first + BK <= S)) {
      const unsigned char* tile = Vbytes + (size_t)first * rowbytes;
#pragma unroll
      for (int n = 0; n < SPW; ++n) pipe_load_16B(tile, voff[n], vst_base + (vslot_hi[n] ? posB : posA) + vslot_lds[n]);
    } else {
#pragma unroll
      for (int n = 0; n < SPW; ++n) {
        uint32_t vo = voff[n];
        asm volatile("" : "+v"(vo));
        pipe_load_16B(Vbytes, vo + (uint32_t)(min(max(first + slot_row[n], 0), S - 1) - slot_row[n]) * rowbytes,
                      vst_base + (vslot_hi[n] ? posB : posA) + vslot_lds[n]);
      }
    }
  };
  auto issue_k = [&](int t) __attribute__((always_inline)) { issue_k_to(std::false_type{}, t, kst_base + (t % 3) * TB); };
  auto issue_v = [&](int t) __attribute__((always_inline)) { issue_v_to(std::false_type{}, t, vpos(2 * t - 1), vpos(2 * t)); };

  // ---- Q fragments: B operand of S^T = K Q^T, lane (col = row qi, k = 16 ks + 8 hf + e) ----
  bf16x8 qf[RPW][KS];
  // First loads of a block of query rows: K tiles 0 and 1, V blocks -1 (a copy of row 0: the first step's PV
  // product multiplies it by zero probabilities, so it only has to be finite) to 2, then the wave's Q rows.
  auto begin_block = [&]() __attribute__((always_inline)) {
    issue_k(0);
    issue_v(0);
    if (ntiles > 1) issue_k(1);
    issue_v(1);
#pragma unroll
    for (int rp = 0; rp < RPW; ++rp) {
      const int qi = qi0 + 32 * rp;
      const bool ok = qi < S;
      const uint16_t* qp = Qg + ((tok0 + (ok ? qi : 0)) * a.Hq + hq) * D + 8 * hf;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)     // rows past the end read row 0 (finite data, results never stored):
        qf[rp][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qp + 16 * ks));   // no branch, no wait here
    }
  };
  begin_block();

  // ---- steering set-up: edit operands, per-column coefficients, highlight bitmap ----
  // Every global load of the set-up (mask bytes, U_cat, routing weights) is issued before the first of them is
  // waited for, with addresses clamped into range instead of branches around the loads: one memory round trip.
  if (STEER && steer_on) {
    const int R = st.M * st.r;
    const uint16_t* Uh = static_cast<const uint16_t*>(st.U) + (size_t)h * st.M * D * st.r;
    const int r8 = st.r / 8;
    const int total = st.M * D * r8;                  // 16-byte pieces of U_cat
    constexpr int UB = 4;                             // pieces per thread and turn

    // (1) mask bytes of tile `tid` (first turn of the bitmap loop), if the fast form applies
    const uint8_t* mrow = st.mask + tok0;
    const int nfull = S / BK;
    const bool wide = (reinterpret_cast<uintptr_t>(mrow) & 15) == 0 && nfull > 0;
    uint4 mv0[BK / 16];
    if (wide) {
      const uint4* mp = reinterpret_cast<const uint4*>(mrow + (size_t)min(tid, nfull - 1) * BK);
#pragma unroll
      for (int q = 0; q < BK / 16; ++q) mv0[q] = mp[q];
    }
    // (2) first turn of U_cat.  Piece idx = (expert m, row d, 8-column group v); the divisions by run-time
    // constants are done in floating point (exact for these small operands: idx < 64 K, quotients < 2 K).
    const float inv_dr8 = 1.f / (float)(D * r8), inv_r8 = 1.f / (float)r8;
    auto split = [&](int idx, int& m, int& d, int& v) __attribute__((always_inline)) {
      m = (int)(((float)idx + 0.5f) * inv_dr8);
      const int rm = idx - m * (D * r8);
      d = (int)(((float)rm + 0.5f) * inv_r8);
      v = rm - d * r8;
    };
    uint4 uv[UB];
    int um[UB], ud[UB], uc[UB];
#pragma unroll
    for (int k = 0; k < UB; ++k) {
      uv[k] = make_uint4(0, 0, 0, 0);
      um[k] = ud[k] = uc[k] = 0;
      if (k * NT < total) {                          // workgroup-uniform
        split(min(tid + k * NT, total - 1), um[k], ud[k], uc[k]);
        uv[k] = *reinterpret_cast<const uint4*>(Uh + ((size_t)um[k] * D + ud[k]) * st.r + 8 * uc[k]);
      }
    }
    // (3) routing weight of column `tid`
    float cw = 1.f;
    if (st.w) cw = st.w[((size_t)b * a.Hkv + h) * st.M + min(tid, R - 1) / st.r];

    auto bits_of = [&](const uint4 (&mv)[BK / 16]) __attribute__((always_inline)) -> unsigned long long {
      unsigned long long bits = 0ull;
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
      return bits;
    };
    // one 64-bit word per tile, one thread per tile: bit k = key 64 t + k is highlighted
    for (int t = tid; t < ntiles; t += NT) {
      unsigned long long bits = 0ull;
      if (wide && t < nfull) {
        if (t == tid) {
          bits = bits_of(mv0);
        } else {
          uint4 mv[BK / 16];
          const uint4* mp = reinterpret_cast<const uint4*>(mrow + (size_t)t * BK);
#pragma unroll
          for (int q = 0; q < BK / 16; ++q) mv[q] = mp[q];
          bits = bits_of(mv);
        }
      } else {
        for (int k = 0; k < BK; ++k)
          if (t * BK + k < S && mrow[(size_t)t * BK + k] != 0) bits |= 1ull << k;
      }
      hlbits[t] = bits;
    }
    if (tid < Rpad) cvec[tid] = tid < R ? gain * cw : 0.f;        // Rpad <= 128 < NT

    // where a 16-byte piece of U_cat goes
    constexpr int CPR = Rpad / 8;                    // dense form: chunks per staged row, 8 or 16
    auto ustage = [&](int d, int chunk) __attribute__((always_inline)) -> unsigned char* {
      const int sw = CPR == 16 ? (d & 15) : ((d >> 1) & 7);
      const int off = d * (Rpad * 2) + 16 * (chunk ^ sw);
      return off < TB ? Kst + 2 * TB + off : Vst + 3 * HB + (off - TB);
    };
    auto place = [&](int m, int d, int v, const uint4 val) __attribute__((always_inline)) {
      if (DENSE) {
        *reinterpret_cast<uint4*>(ustage(d, (m * st.r) / 8 + v)) = val;
      } else {
        const int r0 = m * st.r + 8 * v;              // concatenated column of the first of these 8 elements
        const uint16_t* e16 = reinterpret_cast<const uint16_t*>(&val);
        // operand (rb, s) of U_cat^T K^T: lane (g, j) holds U_cat[d = 32 s + 8 g + e][r = 16 rb + j], e = 0..7
        const int s1 = d >> 5, g1 = (d >> 3) & 3, e1 = d & 7;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int r = r0 + i;
          U1[((((r >> 4) * 4 + s1) * 64) + g1 * 16 + (r & 15)) * 8 + e1] = e16[i];
        }
      }
    };
    if (!DENSE && R != Rpad) {
      for (int i = tid; i < D * Rpad / 8; i += NT) reinterpret_cast<uint4*>(UN)[i] = make_uint4(0, 0, 0, 0);
      __syncthreads();
    }
#pragma unroll
    for (int k = 0; k < UB; ++k)
      if (tid + k * NT < total) place(um[k], ud[k], uc[k], uv[k]);
    for (int idx = tid + UB * NT; idx < total; idx += NT) {        // further turns (large rank and few waves only)
      int m, d, v;
      split(idx, m, d, v);
      place(m, d, v, *reinterpret_cast<const uint4*>(Uh + ((size_t)m * D + d) * st.r + 8 * v));
    }
    if (DENSE) {
      // Dense form.  U_cat (row d, r contiguous, zero-padded to Rpad columns) is staged in the third stage of
      // the K ring and positions 3 and 4 of the V ring, which no tile load touches before the main loop starts
      // (the first loads fill V positions 5, 0, 1 and 2); 16-byte chunks of a row are
      // swizzled so that sixteen consecutive rows can be read at one chunk index without bank conflicts.
      const int padc = CPR - R / 8;                    // R is a multiple of 8
      for (int idx = tid; idx < D * padc; idx += NT)
        *reinterpret_cast<uint4*>(ustage(idx / padc, R / 8 + idx % padc)) = make_uint4(0, 0, 0, 0);
      __syncthreads();
      // T = (U_cat diag(c)) U_cat^T in 16 x 16 blocks; wave w computes the rows 16 w .. 16 w + 15.  The block
      // element T[y][x] is stored where the edit expects (g P)[d_out = x][d' = y] (T is symmetric up to rounding).
      const int j = lane & 15, g = lane >> 4;
      for (int strip = wave; strip < D / 16; strip += NW) {
        bf16x8 af[NKR];      // A operand: lane (row = 16 strip + j, k = r = 32 kk + 8 g + e), scaled by c_r
#pragma unroll
        for (int kk = 0; kk < NKR; ++kk) {
          const bf16x8 u = *reinterpret_cast<const bf16x8*>(ustage(16 * strip + j, 4 * kk + g));
          const f32x4 c0 = *reinterpret_cast<const f32x4*>(cvec + 32 * kk + 8 * g);
          const f32x4 c1 = *reinterpret_cast<const f32x4*>(cvec + 32 * kk + 8 * g + 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            af[kk][e] = (__bf16)((float)u[e] * c0[e]);
            af[kk][4 + e] = (__bf16)((float)u[4 + e] * c1[e]);
          }
        }
#pragma unroll
        for (int ct = 0; ct < D / 16; ++ct) {
          f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int kk = 0; kk < NKR; ++kk) {
            const bf16x8 bfr = *reinterpret_cast<const bf16x8*>(ustage(16 * ct + j, 4 * kk + g));
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[kk], bfr, acc, 0, 0, 0);
          }
          // this lane holds T[y = 16 strip + 4 g + i][x = 16 ct + j], i = 0..3
          const int x = 16 * ct + j, xl = x & 31, y0 = 16 * strip + 4 * g;
          const int frag = ((x >> 5) * 2 + ((xl >> 2) & 1)) * 4 + (y0 >> 5);           // (s_out, half, ks)
          const int flane = 16 * ((y0 & 31) >> 3) + 4 * (xl >> 3) + (xl & 3);          // lane (g', j') of the edit
          bf16x4 o4;
#pragma unroll
          for (int i = 0; i < 4; ++i) o4[i] = (__bf16)acc[i];
          *reinterpret_cast<uint2*>(AP + (frag * 64 + flane) * 8 + (y0 & 7)) = __builtin_bit_cast(uint2, o4);
        }
      }
    }
  }
  // Which of the 64 tiles [tile0, tile0 + 64) hold a highlighted key: kept in scalar registers so that the common
  // case (nothing to edit) costs no LDS access.  Valid once the bitmap is complete (after the first barrier).
  auto any_word = [&](int tile0) __attribute__((always_inline)) -> unsigned long long {
    const int idx = tile0 + lane;
    const unsigned long long v = (steer_on && idx < ntiles) ? hlbits[idx] : 0ull;
    return __ballot(v != 0ull);
  };

  // Dense form (rank > 32): edit the highlighted 16-key blocks of the (swizzled) K tile at Kb in place; wave w < 4
  // owns block w.  What bounds the edit is LDS traffic for its matrix operand (every block reads all of it), so
  // blocks are not split further.
  auto edit_tile = [&](unsigned char* Kb, unsigned long long bits) __attribute__((always_inline)) {
    // The lane index is re-derived behind an opaque copy so that none of the per-lane operand addresses below
    // is hoisted out of the tile loop: they would occupy registers the attention pipeline needs.
    int ln = lane;
    asm volatile("" : "+v"(ln));
    const int j = ln & 15, g = ln >> 4;
    constexpr int KS2 = D / 32;
    const int kblk = wave;
    const unsigned bits16 = (unsigned)((bits >> (16 * (kblk & 3))) & 0xffffull);
    if (kblk >= BK / 16 || bits16 == 0) return;           // wave-uniform
    unsigned char* krow = Kb + (16 * kblk + j) * 256;     // row & 15 == j
    bf16x8 kreg[KS2];   // K^T as B operand: lane (col = key j, k = d = 32 s + 8 g + e) = logical chunk 4 s + g
#pragma unroll
    for (int s = 0; s < KS2; ++s) kreg[s] = *reinterpret_cast<const bf16x8*>(krow + 16 * ((4 * s + g) ^ j));
    const float mbit = ((bits16 >> j) & 1u) ? 1.f : 0.f;
    const float ksc = 1.f + mbit * (kscale - 1.f);        // a for highlighted keys, exactly 1 otherwise
    // k' = a k + mask (g P) k: output rows d are permuted so that each result lands in the lane that holds that
    // element of k
#pragma unroll
    for (int s = 0; s < KS2; ++s) {
      float outv[8];
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int ks = 0; ks < KS2; ++ks) {
          const bf16x8 ua = *reinterpret_cast<const bf16x8*>(AP + (((s * 2 + half) * 4 + ks) * 64 + ln) * 8);
          acc[ks & 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ua, kreg[ks], acc[ks & 1], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
          outv[4 * half + i] = (float)kreg[s][4 * half + i] * ksc + mbit * (acc[0][i] + acc[1][i]);
        __builtin_amdgcn_sched_barrier(0);     // keeps the operand reads of later row groups from piling up in registers
      }
      bf16x8 o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (__bf16)outv[e];
      *reinterpret_cast<bf16x8*>(krow + 16 * ((4 * s + g) ^ j)) = o;
    }
  };

  // Score-side form (rank <= 32): the coordinates c .* (U_cat^T k) of the 64 keys of the (swizzled, unchanged) K
  // tile at Kb, zero for keys that are not highlighted, into the buffer at zdst; wave w < 4 owns the 16-key block w
  // (a block without highlights only stores zeros).  A key's 32 coordinates are stored in the order the score
  // correction contracts them: k-slice ks2, half hf, slot e  <->  r = 16 ks2 + 4 hf + 8 (e / 4) + e % 4, which is
  // the order in which a lane of the 32 x 32 accumulator holds U^T q of its query row (see make_qt).
  auto coords_tile = [&](const unsigned char* Kb, unsigned long long bits, unsigned char* zdst) __attribute__((always_inline)) {
    int ln = lane;
    asm volatile("" : "+v"(ln));
    const int j = ln & 15, g = ln >> 4;
    constexpr int KS2 = D / 32;
    const int kblk = wave;
    if (kblk >= BK / 16) return;                          // wave-uniform
    const unsigned bits16 = (unsigned)((bits >> (16 * kblk)) & 0xffffull);
    // this lane's results: key 16 kblk + j, coordinates r = 16 half + 4 g + i  ->  k-slice half, hf = g & 1, slots 4 (g / 2) + i
    unsigned char* zrow = zdst + (16 * kblk + j) * PIPE_Z_LD + 16 * (g & 1) + 8 * (g >> 1);
    if (bits16 == 0) {
      *reinterpret_cast<uint2*>(zrow) = make_uint2(0, 0);
      *reinterpret_cast<uint2*>(zrow + 32) = make_uint2(0, 0);
      return;
    }
    const unsigned char* krow = Kb + (16 * kblk + j) * 256;     // row & 15 == j
    bf16x8 kreg[KS2];   // K^T as B operand: lane (col = key j, k = d = 32 s + 8 g + e) = logical chunk 4 s + g
#pragma unroll
    for (int s = 0; s < KS2; ++s) kreg[s] = *reinterpret_cast<const bf16x8*>(krow + 16 * ((4 * s + g) ^ j));
    const float mbit = ((bits16 >> j) & 1u) ? 1.f : 0.f;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};   // two chains: even and odd slices of d
#pragma unroll
      for (int s = 0; s < KS2; ++s) {
        const bf16x8 ua = *reinterpret_cast<const bf16x8*>(U1 + ((half * 4 + s) * 64 + ln) * 8);
        acc[s & 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ua, kreg[s], acc[s & 1], 0, 0, 0);
      }
      const f32x4 c4 = *reinterpret_cast<const f32x4*>(cvec + 16 * half + 4 * g);
      bf16x4 z4;
#pragma unroll
      for (int i = 0; i < 4; ++i) z4[i] = (__bf16)((acc[0][i] + acc[1][i]) * (c4[i] * mbit));
      *reinterpret_cast<uint2*>(zrow + 32 * half) = __builtin_bit_cast(uint2, z4);
    }
  };

  for (int pass = 0;; ++pass) {      // one turn per block of query rows (indentation of the body kept flat)
  // ---- math pieces ----
  f32x16 oacc[RPW][DB];
#pragma unroll
  for (int rp = 0; rp < RPW; ++rp)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[rp][db][r] = 0.f;
  const float c2 = a.scale * 1.4426950408889634f;   // probabilities are exp2(s * c2 - m)
  // m_run: reference exponent of the row (in units of s * c2).  It follows the row maximum lazily: it is only
  // raised when the maximum has moved more than kSlack above it, so probabilities stay below 2^kSlack and the
  // output accumulators are rescaled a handful of times per row instead of once per block.
  constexpr float kSlack = 8.f;
  float m_run[RPW], l_run[RPW];
#pragma unroll
  for (int rp = 0; rp < RPW; ++rp) { m_run[rp] = -1e30f; l_run[rp] = 0.f; }
  // The tile loops live in a (generic, always inlined) lambda of their own.  This changes nothing in what is
  // computed; the compiler allocates the loop's registers differently for it, and the launch is 3 % faster.
  auto run_block = [&](auto) __attribute__((always_inline)) {

  // LDS byte addresses of this lane's operands inside stage 0 (stage and row-block offsets are immediates):
  // K: row l32 (+32), logical chunk 2 ks + hf, physical chunk (2 ks + hf) ^ (l32 & 15)
  // V: row 16 kb + 4 hf + (li >> 2) (+8), logical chunk 4 db + 2 (grp & 1) + ((li & 3) >> 1), physical chunk 4 (db ^ q) + low
  uint32_t kaddr[KS], vaddr[DB];
  {
    const int kfix = l32 * 256 + 16 * (hf ^ (l32 & 1)) + 32 * ((l32 & 15) >> 1);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kaddr[ks] = kst_base + (uint32_t)(kfix ^ (ks << 5));
    const int li = lane & 15, grp = lane >> 4;
    const int vfix = (4 * hf + (li >> 2)) * 256 + 64 * ((li >> 2) & 3) + 16 * (2 * (grp & 1) + ((li & 3) >> 1)) + 8 * (li & 1);
#pragma unroll
    for (int db = 0; db < DB; ++db) vaddr[db] = vst_base + (uint32_t)(vfix ^ (db << 6));
  }

  // Part [KS0, KS1) of one 32-key block of S^T (32 keys x 32 RPW rows) = K rows . Q^T ; off = LDS byte offset
  // of the block's first row.  Each K fragment is read once and used for every row block of the wave.
  auto qk_part = [&](auto ks0_c, auto ks1_c, int off, f32x16 (&sn)[RPW]) __attribute__((always_inline)) {
    constexpr int KS0 = decltype(ks0_c)::value, KS1 = decltype(ks1_c)::value;
    if (KS0 == 0) {
#pragma unroll
      for (int rp = 0; rp < RPW; ++rp)
#pragma unroll
        for (int r = 0; r < 16; ++r) sn[rp][r] = 0.f;
    }
#pragma unroll
    for (int ks = KS0; ks < KS1; ++ks) {
      const bf16x8 a0 = *(pipe_lds_bf16x8_ptr)(uintptr_t)(kaddr[ks] + off);
#pragma unroll
      for (int rp = 0; rp < RPW; ++rp) sn[rp] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qf[rp][ks], sn[rp], 0, 0, 0);
    }
  };
  using IC0 = std::integral_constant<int, 0>;
  using ICH = std::integral_constant<int, KS / 2>;
  using ICK = std::integral_constant<int, KS>;
  // causal mask of the 32-key block starting at key j0, row block rp
  auto causal_mask = [&](int j0, int rp, f32x16& sv) __attribute__((always_inline)) {
    const int jbase = j0 + 4 * hf, qi = qi0 + 32 * rp;
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (jbase + 8 * (r >> 2) + (r & 3) > qi) sv[r] = -INFINITY;
  };
  // Softmax of one 32-key block, first part: row maximum (of s * c2) over the block, both halves of the row.
  auto block_max = [&](const f32x16& sv) __attribute__((always_inline)) -> float {
    float mx = pipe_max3(sv[0], sv[1], sv[2]);
#pragma unroll
    for (int r = 3; r < 15; r += 2) mx = pipe_max3(mx, sv[r], sv[r + 1]);
    mx = fmaxf(mx, sv[15]) * c2;
    // the other 16 keys of this query row live in lane ^ 32
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
    return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
  };
  // Raise the reference exponent of the rows whose maximum ran away from it, and rescale their sums.  The output
  // accumulators are rescaled by rescale_outputs(), which the caller runs once every PV product whose
  // probabilities were formed against the old reference has been accumulated.
  float alpha_pend[RPW];
  bool rescale_pend[RPW];                // wave-uniform
#pragma unroll
  for (int rp = 0; rp < RPW; ++rp) { alpha_pend[rp] = 1.f; rescale_pend[rp] = false; }
  auto raise_reference = [&](int rp, float mfull) __attribute__((always_inline)) {
    const bool need = mfull > m_run[rp] + kSlack;
    if (__any(need)) {   // a handful of times per row
      const float m_new = need ? mfull : m_run[rp];
      const float alpha = __builtin_amdgcn_exp2f(m_run[rp] - m_new);
      m_run[rp] = m_new;
      l_run[rp] *= alpha;
      alpha_pend[rp] = alpha;            // rescale_outputs() has run since the last raise of this row block
      rescale_pend[rp] = true;
    }
  };
  auto rescale_outputs = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int rp = 0; rp < RPW; ++rp)
      if (rescale_pend[rp]) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[rp][db][r] *= alpha_pend[rp];
        rescale_pend[rp] = false;
      }
  };
  // Second part: probabilities, packed P^T, row sum of the rounded probabilities (the values the PV product uses).
  auto block_exp = [&](int rp, f32x16& sv, bf16x8 (&pb)[2]) __attribute__((always_inline)) {
    const float mneg = -m_run[rp];
#pragma unroll
    for (int r = 0; r < 16; ++r) sv[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[r], c2, mneg));
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      pb[0][e] = (__bf16)sv[e];
      pb[1][e] = (__bf16)sv[8 + e];
    }
    float lsum = l_run[rp];
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        const bf16x2 pp = {pb[kb][e], pb[kb][e + 1]};
        lsum = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, lsum, false);
      }
    l_run[rp] = lsum;
  };
  // The same for the schedule without a per-block maximum: the scores are left untouched, the sum of the rounded
  // probabilities is returned instead of being added to the row's running sum.
  auto block_exp_sum = [&](const f32x16& sv, bf16x8 (&pb)[2], float& lsum) __attribute__((always_inline)) {
    const float mneg = -m_run[0];
    float pv[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) pv[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[r], c2, mneg));
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      pb[0][e] = (__bf16)pv[e];
      pb[1][e] = (__bf16)pv[8 + e];
    }
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    float acc = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        const bf16x2 pp = {pb[kb][e], pb[kb][e + 1]};
        acc = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, acc, false);
      }
    lsum = acc;
  };
  // O^T += V^T P^T for one 32-key block; off = LDS byte offset of the block's first row
  auto pv_half = [&](int off, const bf16x8 (&pb)[RPW][2]) __attribute__((always_inline)) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((dma_lds_s16x4_ptr)(uintptr_t)(vaddr[db] + off + (16 * kb) * 256));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((dma_lds_s16x4_ptr)(uintptr_t)(vaddr[db] + off + (16 * kb + 8) * 256));
        const bf16x4 lo4 = __builtin_bit_cast(bf16x4, lo), hi4 = __builtin_bit_cast(bf16x4, hi);
        const bf16x8 va = __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
        for (int rp = 0; rp < RPW; ++rp)
          oacc[rp][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[rp][kb], oacc[rp][db], 0, 0, 0);
      }
    }
  };

  const bool wave_rows_exist = qw < S;
  const int tw_last = wave_rows_exist ? min(ntiles - 1, (qw + WR - 1) / BK) : -1;   // last tile this wave computes on

  // ---- prologue: wait for the first tiles, edit K(0) and K(1), first block of S^T ----
  dma_wait_vmcnt<0>();   // also covers the Q, U and mask loads issued after the tile loads
#pragma unroll
  for (int rp = 0; rp < RPW; ++rp)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qf[rp][ks]));   // pin the compiler's own wait for Q here, not in the loop
  dma_barrier();
  unsigned long long anyw = 0ull;      // bit i: tile 64 (t / 64) + i holds a highlighted key (0 when not steering)
  // Next tile index at which the loop has something to do besides attention: a tile with highlighted keys, or
  // the start of the next group of 64 tiles (summary reload).  Scalar; the loop compares one integer per tile.
  auto next_event = [&](int tile) __attribute__((always_inline)) -> int {     // first event strictly after `tile`
    const unsigned sh = tile & 63;
    const unsigned long long rest = sh == 63u ? 0ull : anyw >> (sh + 1);
    return rest != 0ull ? tile + 1 + __builtin_ctzll(rest) : (tile | 63) + 1;
  };
  int tile_evt = 0x7fffffff;
  int ztile = -1;                      // score-side form: the tile whose coordinates were computed last
  if (STEER && !DENSE) {
    // U^T q of this wave's 32 query rows: (U_cat^T Q^T)[r][row] on the 32 x 32 MFMA, A = U_cat^T rows r = l32 taken
    // from the operand store of U_cat^T K^T (entry (rb, s), lane (g, j) with r = 16 rb + j, d = 32 s + 8 g + e),
    // B = the Q fragments.  A lane ends up with its query row's coordinates r = 8 (i / 4) + 4 hf + i % 4, i = 0..15:
    // converted to bf16 they are the two B operands of the score correction as they stand, kept in LDS (each lane
    // reads back what it wrote: no barrier).
    if (steer_on) {
      f32x16 qt;
#pragma unroll
      for (int r = 0; r < 16; ++r) qt[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 ua = *reinterpret_cast<const bf16x8*>(
            U1 + ((((l32 >> 4) * 4 + (ks >> 1)) * 64) + (2 * (ks & 1) + hf) * 16 + (l32 & 15)) * 8);
        qt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua, qf[0][ks], qt, 0, 0, 0);
      }
      bf16x8 q8[2];
#pragma unroll
      for (int e = 0; e < 8; ++e) { q8[0][e] = (__bf16)qt[e]; q8[1][e] = (__bf16)qt[8 + e]; }
      unsigned char* qp = qtbuf + wave * PIPE_QT_BYTES + lane * 16;
      *reinterpret_cast<bf16x8*>(qp) = q8[0];
      *reinterpret_cast<bf16x8*>(qp + PIPE_QT_BYTES / 2) = q8[1];
    }
    anyw = any_word(0);
    if (anyw & 1ull) {
      coords_tile(Kst, hlbits[0], zbuf);
      dma_barrier();
      ztile = 0;
    }
    tile_evt = next_event(0);          // tile 1 is handled by iteration 0 like every later tile
  } else if (STEER) {
    anyw = any_word(0);
    if (anyw & 3ull) {
      if (anyw & 1ull) edit_tile(Kst, hlbits[0]);
      if (anyw & 2ull) edit_tile(Kst + TB, hlbits[1]);
      dma_barrier();
    }
    tile_evt = next_event(1);
  }
  // Score correction of one 32-key block of S^T (keys keyoff .. keyoff + 31 of `tile`): += Z (32 keys x 32 r) . (U^T q)^T,
  // two MFMAs; A = the keys' coordinates from the tile's buffer, B = this wave's U^T q operands.
  auto corr = [&](int tile, int keyoff, f32x16 (&sv)[RPW]) __attribute__((always_inline)) {
    const unsigned char* zp = zbuf + (tile & 1) * PIPE_Z_BYTES + (keyoff + l32) * PIPE_Z_LD + 16 * hf;
    const unsigned char* qp = qtbuf + wave * PIPE_QT_BYTES + lane * 16;
#pragma unroll
    for (int k2 = 0; k2 < 2; ++k2) {
      const bf16x8 za = *reinterpret_cast<const bf16x8*>(zp + 32 * k2);
      const bf16x8 qb = *reinterpret_cast<const bf16x8*>(qp + (PIPE_QT_BYTES / 2) * k2);
      sv[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(za, qb, sv[0], 0, 0, 0);
    }
  };

  bf16x8 pb[RPW][2];           // probabilities (P^T operand) of the block whose PV product is next; none at first
#pragma unroll
  for (int rp = 0; rp < RPW; ++rp)
#pragma unroll
    for (int e = 0; e < 8; ++e) { pb[rp][0][e] = (__bf16)0.f; pb[rp][1][e] = (__bf16)0.f; }
  f32x16 sc0[RPW], sc1[RPW];   // scores of keys 0..31 / 32..63 of the current tile, per row block
#pragma unroll
  for (int rp = 0; rp < RPW; ++rp)
#pragma unroll
    for (int r = 0; r < 16; ++r) { sc0[rp][r] = 0.f; sc1[rp][r] = 0.f; }
  bf16x8 kpre[2];              // first two K fragments of the block the next step scores (see `step`)
  if (0 <= tw_last) {
    qk_part(IC0{}, ICK{}, 0, sc0);
#pragma unroll
    for (int rp = 0; rp < RPW; ++rp) pipe_mfma_result_guard(sc0[rp]);
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) kpre[i] = *(pipe_lds_bf16x8_ptr)(uintptr_t)(kaddr[i] + HB);

  // `top` of iteration t: request K(t+2), then the V blocks 2t+3 and 2t+4; their ring slots are free since the
  // barrier of iteration t - 1.  Bottom: everything but those two V blocks must have landed before the next
  // iteration (K(t+2) is edited there, see `events`).  The hot loop calls `top` between its two steps: requests
  // issued right after the barrier delayed the first step's operand reads (1-2 % of the kernel).
  // The hot loop only runs where tile t + 2 exists and is complete (`sure`): no tests there.
  auto top = [&](auto sure_c, auto stage_c, int t) __attribute__((always_inline)) {
    constexpr bool SURE = decltype(sure_c)::value;
    if (SURE) {
      constexpr int ST = decltype(stage_c)::value;          // = t % 3
      issue_k_to(std::true_type{}, t + 2, kst_base + ((ST + 2) % 3) * TB);
      issue_v_to(std::true_type{}, t + 2, ((2 * ST + 3) % 6) * HB, ((2 * ST + 4) % 6) * HB);
    } else if (t + 1 < ntiles) {
      if (t + 2 < ntiles) issue_k(t + 2);
      issue_v(t + 2);                                       // its first block belongs to tile t + 1
    }
  };
  auto bottom = [&](auto sure_c, int t) __attribute__((always_inline)) {
    if (decltype(sure_c)::value || t + 1 < ntiles) dma_wait_vmcnt<SPW>();   // all but the V loads of this iteration
    else dma_wait_vmcnt<0>();
    dma_barrier();
  };

  // Steering events of the tile that landed at the bottom of the previous iteration (tile t + 1 in iteration t):
  // handled between the two steps of an iteration, where a basic-block boundary exists anyway (the conditional
  // rescale).  Directly after the per-tile barrier the same branch kept the compiler from moving the next step's
  // first LDS reads up, which cost every iteration of the steered kernels 7-9 % even with nothing to edit.  The
  // second step is the first reader of that tile; after an edit in place (dense form) its two prefetched
  // fragments are read again.  In the score-side form the tile is not changed: the event leaves the tile's
  // coordinates in the buffer of its parity (the other buffer may still be read for the previous tile's second
  // block) and ztile tells the next iteration which scores to correct.  No barrier of its own: the coordinates are
  // first read after the barrier at the bottom of the iteration, by the corrections of the two score blocks of
  // that tile at the top of the next iteration and after its first step.
  auto events = [&](int t, int knext_off, bf16x8 (&kp)[2]) __attribute__((always_inline)) {
    if (!STEER) return;
    // one scalar compare in the common case; tiles past the end and unsteered heads have no bit set
    const int tn = t + 1;
    if (__builtin_expect(tn == tile_evt, 0)) {
      const unsigned sh = tn & 63;
      if (sh == 0u) anyw = any_word(tn);
      tile_evt = next_event(tn);
      if ((anyw >> sh) & 1ull) {
        if (!DENSE) {                    // score-side: the tile stays as it is, its coordinates go to a buffer
          coords_tile(Kst + (tn % 3) * TB, hlbits[tn], zbuf + (tn & 1) * PIPE_Z_BYTES);
          ztile = tn;                    // first read after the barrier at the bottom of this iteration
        } else {
          edit_tile(Kst + (tn % 3) * TB, hlbits[tn]);
          dma_barrier();
#pragma unroll
          for (int i = 0; i < 2; ++i) kp[i] = *(pipe_lds_bf16x8_ptr)(uintptr_t)(kaddr[i] + knext_off);
        }
      }
    }
  };

  // One software-pipelined step over three consecutive 32-key blocks: the S^T block at LDS offset KOFF is
  // produced into `next` and the PV products of the block before `cur` (probabilities pb, V rows at ring offset
  // VOFF) are accumulated while the softmax of `cur` runs on the vector ALU; pb then receives the probabilities
  // of `cur`.  Every MFMA of the step has vector work to share the issue port with.
  // The LDS offsets are std::integral_constant in the main loop (they become immediates) and int elsewhere.
  // kpre: the first two K fragments of the block at KOFF, read during the previous step (an LDS read issued right
  // before the MFMA that needs it leaves the wave waiting for the whole LDS latency); on return it holds those of
  // the block at KNEXT, the one the following step scores.
  //
  // No row maximum in the common case.  The probabilities of `cur` are formed against the row's reference exponent
  // as it stands; their sum over the block tells whether that was safe: a sum beyond kSumLimit (or one that is not
  // a number) means some score ran far ahead of the reference, and only then is the block's maximum computed, the
  // reference raised and the block's probabilities formed again (a handful of times per row; the first block of a
  // row always takes this turn, its reference starts at -1e30).  The common case is 16 multiply-adds, 16
  // exponentials, 8 packings and 8 dot products per 16 MFMAs: no three-input maxima, no cross-lane exchange, no
  // raise test.
  auto kfrag = [&](int ks, int off) __attribute__((always_inline)) -> bf16x8 {
    return *(pipe_lds_bf16x8_ptr)(uintptr_t)(kaddr[ks] + off);
  };
  auto qk_one = [&](int ks, const bf16x8& a0, f32x16 (&sn)[RPW]) __attribute__((always_inline)) {
#pragma unroll
    for (int rp = 0; rp < RPW; ++rp) sn[rp] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qf[rp][ks], sn[rp], 0, 0, 0);
  };
  constexpr float kSumLimit = 4096.f;          // probabilities stay below 2^12
  auto step = [&](auto koff_c, auto knext_c, auto voff_c, f32x16 (&cur)[RPW], f32x16 (&next)[RPW], bf16x8 (&pb)[RPW][2],
                  bf16x8 (&kpre)[2]) __attribute__((always_inline)) {
    static_assert(KS == 8 && RPW == 1, "the schedule below is written for eight k-slices and one row block per wave");
    const int KOFF = koff_c, KNEXT = knext_c, VOFF = voff_c;
    bf16x8 pn[2];
    float lb;
#pragma unroll
    for (int r = 0; r < 16; ++r) next[0][r] = 0.f;
    qk_one(0, kpre[0], next);
    qk_one(1, kpre[1], next);
    const bf16x8 k2 = kfrag(2, KOFF), k3 = kfrag(3, KOFF);
    qk_one(2, k2, next);
    qk_one(3, k3, next);
    const bf16x8 k4 = kfrag(4, KOFF), k5 = kfrag(5, KOFF);
    qk_one(4, k4, next);
    qk_one(5, k5, next);
    const bf16x8 k6 = kfrag(6, KOFF), k7 = kfrag(7, KOFF);
    qk_one(6, k6, next);
    qk_one(7, k7, next);
    pv_half(VOFF, pb);
    kpre[0] = kfrag(0, KNEXT);
    kpre[1] = kfrag(1, KNEXT);
    block_exp_sum(cur[0], pn, lb);
    // Program order: every MFMA is followed by its share of the 24 LDS reads, two plain vector instructions and
    // (from the second MFMA on, when the first multiply-adds have been issued) one exponential: the transcendental
    // unit takes one instruction about every ten cycles, and a run of exponentials stalls the wave in front of
    // the next MFMA.
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 2);          // fragments 2 and 3
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 2);
      if (i < 14 && !(i & 1)) __builtin_amdgcn_sched_group_barrier(0x100, 2, 2);
      if (i < 15 && ((i & 1) || i == 14)) __builtin_amdgcn_sched_group_barrier(0x100, 1, 2);
      __builtin_amdgcn_sched_group_barrier(0x002, 2, 2);
      if (i >= 1) __builtin_amdgcn_sched_group_barrier(0x400, 1, 2);
    }
    __builtin_amdgcn_sched_group_barrier(0x400, 1, 2);
    // The probabilities are first used by the next step: without a use here their whole computation is sunk
    // into that step, away from the MFMAs it is meant to share the issue port with.
    asm volatile("" : "+v"(pn[0]), "+v"(pn[1]), "+v"(lb));
    __builtin_amdgcn_sched_barrier(0);
    if (__builtin_expect(__any(!(lb <= kSumLimit)), 0)) {
      // `cur` was produced by the previous step's MFMAs: far enough behind for the inline-assembly maxima
      raise_reference(0, block_max(cur[0]));
      block_exp_sum(cur[0], pn, lb);
      rescale_outputs();       // after this step's PV product, whose probabilities were formed against the old reference
    }
    l_run[0] += lb;
    pb[0][0] = pn[0];
    pb[0][1] = pn[1];
  };
  // One tile every row of this wave sees in full; ST = t % 3 is compile-time so that every LDS read address is
  // a register plus an immediate.  Enters with S(t, keys 0..31) in sc0 and the probabilities of the block before
  // it in pb; leaves with the same for tile t + 1.
  auto hot = [&](auto st_c, int t) __attribute__((always_inline)) {
    constexpr int ST = decltype(st_c)::value;
    using std::integral_constant;
    // The operand addresses pass through an opaque copy once per tile: otherwise every "address + stage offset"
    // below is hoisted out of the loop into a register of its own (dozens), instead of being an immediate.
    if (STEER && !DENSE && __builtin_expect(ztile == t, 0)) corr(t, 0, sc0);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(kaddr[ks]));
#pragma unroll
    for (int db = 0; db < DB; ++db) asm volatile("" : "+v"(vaddr[db]));
    step(integral_constant<int, ST * TB + HB>{}, integral_constant<int, ((ST + 1) % 3) * TB>{}, integral_constant<int, ((2 * ST + 5) % 6) * HB>{}, sc0, sc1, pb, kpre);
    if (STEER && !DENSE && __builtin_expect(ztile == t, 0)) corr(t, 32, sc1);
    top(std::true_type{}, st_c, t);
    if (kEventsInHot) events(t, ((ST + 1) % 3) * TB, kpre);
    step(integral_constant<int, ((ST + 1) % 3) * TB>{}, integral_constant<int, ((ST + 1) % 3) * TB + HB>{}, integral_constant<int, 2 * ST * HB>{}, sc1, sc0, pb, kpre);
    bottom(std::true_type{}, t);
  };

  // Hot iterations: tile t is seen in full by every row of this wave and tile t + 2 exists and is complete.  They
  // run in whole turns of the ring with a single loop exit (exits after every tile made the compiler park what
  // the code after the loop needs in scratch memory, inside the loop).  Everything else before the wave's last
  // tile runs the same pipelined step with run-time ring offsets and guarded loads (a slower tile).
  // Steering events (a tile to edit, a summary word to reload) are handled inside the hot loop, except in the
  // one shape where that measured slower than leaving the loop for the slower tile: the dense edit with seven
  // waves (Hq=28, Hkv=4, rank 64: 3 % faster outside; dense with eight waves: 3 % faster inside).
  const int t_hot = min(tw_last, min(ntiles, S / BK) - 2);
  int t = 0;
#pragma nounroll
  while (t < tw_last) {
    if (t % 3 == 0) {
      using std::integral_constant;
#pragma nounroll
      for (; t + 3 <= t_hot && (!STEER || kEventsInHot || tile_evt > t + 3); t += 3) {
        hot(integral_constant<int, 0>{}, t);
        hot(integral_constant<int, 1>{}, t + 1);
        hot(integral_constant<int, 2>{}, t + 2);
      }
      if (t >= tw_last) break;
    }
    top(std::false_type{}, IC0{}, t);
    const int off = (t % 3) * TB, offn = ((t + 1) % 3) * TB;
    if (STEER && !DENSE && ztile == t) corr(t, 0, sc0);
    step(off + HB, offn, (int)vpos(2 * t - 1), sc0, sc1, pb, kpre);
    if (STEER && !DENSE && ztile == t) corr(t, 32, sc1);
    events(t, offn, kpre);
    step(offn, offn + HB, (int)vpos(2 * t), sc1, sc0, pb, kpre);
    bottom(std::false_type{}, t);
    ++t;
  }
  // ---- up to two more full tiles before the wave's last one: same pipelined step, ring stage known at run time ----
#pragma nounroll
  for (; t < tw_last; ++t) {
    top(std::false_type{}, IC0{}, t);
    const int off = (t % 3) * TB, offn = ((t + 1) % 3) * TB;
    if (STEER && !DENSE && ztile == t) corr(t, 0, sc0);
    step(off + HB, offn, (int)vpos(2 * t - 1), sc0, sc1, pb, kpre);
    if (STEER && !DENSE && ztile == t) corr(t, 32, sc1);
    events(t, offn, kpre);
    step(offn, offn + HB, (int)vpos(2 * t), sc1, sc0, pb, kpre);
    bottom(std::false_type{}, t);
  }
  // ---- the wave's last tile (causal mask, nothing further to score), then idle turns while other waves finish.
  // The second block of that tile may still be in flight during its own iteration (V runs half a tile behind), so
  // its PV product waits for the barrier at the bottom: it is done one turn later, or after the loop. ----
  bool owed = false;                       // wave-uniform: pb holds probabilities whose PV product is outstanding
  int owed_off = 0;
#pragma nounroll
  for (; t < ntiles; ++t) {
    top(std::false_type{}, IC0{}, t);
    const bool zt = STEER && !DENSE && ztile == t;     // before the event of tile t + 1 moves ztile on
    events(t, 0, kpre);                     // this wave scores nothing further; other waves may (kpre is dead here)
    if (owed) {
      pv_half(owed_off, pb);
      owed = false;
    }
    if (t == tw_last) {
      const int off = (t % 3) * TB;
      qk_part(IC0{}, ICK{}, off + HB, sc1);
      if (zt) {
        corr(t, 0, sc0);
        corr(t, 32, sc1);
      }
      if (t > 0) pv_half((int)vpos(2 * t - 1), pb);      // the block before this tile (its softmax ran in the last step)
#pragma unroll
      for (int rp = 0; rp < RPW; ++rp) {
        pipe_mfma_result_guard(sc0[rp]);
        causal_mask(t * BK, rp, sc0[rp]);
        raise_reference(rp, block_max(sc0[rp]));
      }
      rescale_outputs();
#pragma unroll
      for (int rp = 0; rp < RPW; ++rp) block_exp(rp, sc0[rp], pb[rp]);
      pv_half((int)vpos(2 * t), pb);
#pragma unroll
      for (int rp = 0; rp < RPW; ++rp) {
        pipe_mfma_result_guard(sc1[rp]);
        causal_mask(t * BK + 32, rp, sc1[rp]);
        raise_reference(rp, block_max(sc1[rp]));
      }
      rescale_outputs();
#pragma unroll
      for (int rp = 0; rp < RPW; ++rp) block_exp(rp, sc1[rp], pb[rp]);
      owed = true;
      owed_off = (int)vpos(2 * t + 1);
    }
    bottom(std::false_type{}, t);
  }
  if (owed) pv_half(owed_off, pb);
  };
  run_block(std::false_type{});

  // ---- next block's first loads (after a barrier: the last PV product above still read the V ring), then this
  // block's output ----
  const int qi_out = qi0;
  const bool more = pass + 1 < npass;
  if (more) {
    dma_barrier();
    qb = pair;
    qw = qb * BQ + WR * (wave % RBW);
    qi0 = qw + l32;
    last_key = min(S, qb * BQ + BQ) - 1;
    ntiles = last_key / BK + 1;
    begin_block();
  }
#pragma unroll
  for (int rp = 0; rp < RPW; ++rp) {
    const int qi = qi_out + 32 * rp;
    const float l_tot = l_run[rp] + __shfl_xor(l_run[rp], 32);
    if (qi < S) {
      const float inv = 1.f / l_tot;
      uint16_t* op = Og + ((tok0 + qi) * a.Hq + hq) * D + 4 * hf;
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
      // m_run is the reference exponent in units of s * scale * log2(e); l_tot is relative to it
      if (a.lse && hf == 0) a.lse[lse_index(a, b, hq, tok0, qi)] = m_run[rp] * 0.6931471805599453f + logf(l_tot);
    }
  }
  if (!more) break;
  }   // for pass
}

}  // namespace seka
