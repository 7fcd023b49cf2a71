// seka_edit_keys: standalone key-editing hook (paper Algorithm 1/2, inference part):
//   k' = k + g * sum_m w_m U_m (U_m^T k)   on highlighted tokens of selected heads.
//
// HBM-bound (read K once, write K' once).  bf16 path: one tile = 64 tokens of one KV head,
// one wave = 16 tokens.  A wave keeps its 16 x D key tile in registers in exactly the layout the
// 16x16x32 bf16 MFMA wants for its B operand, so the two small GEMMs
//   Z^T = U_cat^T K^T   (R x 16, contraction over D)      and
//   C^T = U_cat (c .* Z^T)   (D x 16, contraction over R)
// run on the matrix cores without moving the keys again, and the correction lands in the same
// lanes that hold the matching key elements (the row order of U fed to the second GEMM is
// permuted to make that so).  Tiles without highlighted tokens are a plain 16-byte copy (or are
// skipped entirely when editing in place).  U is staged in LDS only by workgroups that need it; at large
// ranks a tile is 128 tokens, a wave owns two groups of 16, and U is staged once instead of twice.
#include "common.h"

namespace seka {

namespace {

typedef __attribute__((address_space(3))) s16x4* edit_lds_s16x4_ptr;
constexpr int kEditThreads = 256;
constexpr int kEditTokens = 64;   // tokens per workgroup (bf16 path)

__device__ __forceinline__ int perm_col(int r) {
  // position of U's column r inside its group of 32 so that one 16-byte LDS read yields the
  // 8 contraction slots an MFMA lane owns: slot order follows the 16x16 accumulator layout
  // (4 consecutive rows per lane per 16-row block).
  return (r & ~31) + 8 * ((r & 15) >> 2) + 4 * ((r & 31) >> 4) + (r & 3);
}

// First token row and length of prompt b: rows b*S .. b*S+S-1 of a padded batch, or rows cu[b] .. cu[b+1]-1 of a
// packed one (offsets clamped into the tensor, lengths to [0, S]).
__device__ __forceinline__ void edit_prompt_extent(const int* __restrict__ cu, int total, int b, int S, size_t& tok0, int& len) {
  tok0 = (size_t)b * S;
  len = S;
  if (cu != nullptr) {
    const int start = min(max(cu[b], 0), total);
    len = min(max(min(cu[b + 1] - start, total - start), 0), S);
    tok0 = (size_t)start;
  }
}

template <int D, int TG>
__global__ __launch_bounds__(kEditThreads) void edit_keys_bf16_kernel(const uint16_t* __restrict__ K_in,
                                                                      uint16_t* __restrict__ K_out, int S, int Hkv,
                                                                      SteerArgs st, int inplace, int Rpad,
                                                                      const int* __restrict__ cu, int total) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int TOK = kEditTokens * TG;        // tokens per tile: a wave owns TG groups of 16 consecutive tokens
  // Small ranks (TG = 1): U twice in LDS, each copy in the order one product reads it with 16-byte reads (U^T
  // [Rpad][D], and U [D][Rpad] with permuted columns).  Large ranks (TG = 2, WIDE): U once, as stored ([D][Rpad],
  // columns in order): the first product fetches its operand with transposing reads, the second with two 8-byte
  // reads; half the LDS (35 KB instead of 70 KB at rank 128: four workgroups per CU instead of two) and a staging
  // pass of plain 16-byte copies.
  constexpr bool WIDE = TG == 2;
  constexpr int UT_LD = D + 8;                 // row stride of U^T [Rpad][D] in elements
  const int UN_LD = Rpad + 8;                  // row stride of U [D][Rpad]
  uint16_t* UT = reinterpret_cast<uint16_t*>(smem);
  uint16_t* UN = WIDE ? UT : UT + (size_t)Rpad * UT_LD;
  float* cvec = reinterpret_cast<float*>(UN + (size_t)D * UN_LD);

  const int b = blockIdx.z, h = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = lane & 15, g = lane >> 4;
  size_t tok0;
  int len;
  edit_prompt_extent(cu, total, b, S, tok0, len);
  const float gain = st.gain[h];
  const float kscale = st.kscale[h];
  // One tile per workgroup.  At large ranks (35 KB of LDS: four workgroups per CU where small ranks have eight) a
  // wave owns two token groups (TG = 2): twice the bytes in flight per wave, and every U fragment read from LDS
  // serves both groups.
  const int tile = blockIdx.x;
  if (tile * TOK >= len) return;                         // workgroup-uniform, before any barrier
  constexpr int KS = D / 32;
  int mk[TG];
  bool valid[TG];
  size_t row_off[TG];
  bf16x8 kreg[TG][KS];
#pragma unroll
  for (int tg = 0; tg < TG; ++tg) {
    const int t = tile * TOK + (wave * TG + tg) * 16 + j;
    valid[tg] = t < len;
    row_off[tg] = ((tok0 + (valid[tg] ? t : 0)) * Hkv + h) * D;
#pragma unroll
    for (int s = 0; s < KS; ++s) kreg[tg][s] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
  }
  auto load_keys = [&](int tg) __attribute__((always_inline)) {
#pragma unroll
    for (int s = 0; s < KS; ++s)
      kreg[tg][s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(K_in + row_off[tg] + 32 * s + 8 * g));
  };
  // Out of place every key is needed whatever the mask says: the keys are requested first and the mask bytes
  // travel with them.  In place a group whose 16 tokens are not highlighted is neither edited nor copied, so the
  // mask decides which keys are read at all.
  if (!inplace) {
#pragma unroll
    for (int tg = 0; tg < TG; ++tg)
      if (valid[tg]) load_keys(tg);
  }
#pragma unroll
  for (int tg = 0; tg < TG; ++tg) mk[tg] = valid[tg] ? st.mask[tok0 + tile * TOK + (wave * TG + tg) * 16 + j] : 0;
  if (inplace) {
#pragma unroll
    for (int tg = 0; tg < TG; ++tg)
      if (valid[tg] && __ballot(mk[tg] != 0) != 0ull) load_keys(tg);
  }
  bool any_mk = false;
#pragma unroll
  for (int tg = 0; tg < TG; ++tg) any_mk = any_mk || mk[tg] != 0;
  const bool wave_hl = __ballot(any_mk) != 0ull;
  const bool block_hl = __syncthreads_or(any_mk) != 0;
  const bool steered = block_hl && gain != 0.f;
  auto copy_out = [&]() __attribute__((always_inline)) {
    if (inplace) return;
#pragma unroll
    for (int tg = 0; tg < TG; ++tg)
      if (valid[tg]) {
#pragma unroll
        for (int s = 0; s < KS; ++s)
          *reinterpret_cast<uint4*>(K_out + row_off[tg] + 32 * s + 8 * g) = __builtin_bit_cast(uint4, kreg[tg][s]);
      }
  };

  if (!steered) {
    copy_out();
    return;
  }

  // ---- stage U and the per-column coefficients in LDS ----
  const int R = st.M * st.r;
  if (R != Rpad) {
    if (!WIDE)
      for (int i = threadIdx.x; i < (Rpad - R) * UT_LD; i += kEditThreads) UT[(size_t)R * UT_LD + i] = 0;
    for (int i = threadIdx.x; i < D * UN_LD; i += kEditThreads) UN[i] = 0;
    __syncthreads();
  }
  if (WIDE) {
    const uint16_t* Uh = reinterpret_cast<const uint16_t*>(st.U) + (size_t)h * st.M * D * st.r;
    const int r8 = st.r / 8;
    const int total_chunks = st.M * D * r8;
    for (int idx = threadIdx.x; idx < total_chunks; idx += kEditThreads) {
      const int m = idx / (D * r8), rm = idx % (D * r8);
      const int d = rm / r8, v = rm % r8;
      *reinterpret_cast<uint4*>(UN + (size_t)d * UN_LD + m * st.r + 8 * v) =
          *reinterpret_cast<const uint4*>(Uh + ((size_t)m * D + d) * st.r + 8 * v);
    }
    for (int r = threadIdx.x; r < Rpad; r += kEditThreads) {
      float c = 0.f;
      if (r < R) c = gain * (st.w ? st.w[((size_t)b * Hkv + h) * st.M + r / st.r] : 1.f);
      cvec[r] = c;
    }
  } else {
    const uint16_t* Uh = reinterpret_cast<const uint16_t*>(st.U) + (size_t)h * st.M * D * st.r;
    // A thread takes the same 8 columns of four consecutive rows d (four 16-byte pieces of U), so that the
    // transposed copy is written 8 bytes at a time instead of 2.
    const int r8 = st.r / 8;
    const int quads = st.M * (D / 4) * r8;
    for (int idx = threadIdx.x; idx < quads; idx += kEditThreads) {
      const int m = idx / ((D / 4) * r8), rem = idx % ((D / 4) * r8);
      const int d0 = 4 * (rem / r8), v = rem % r8;
      const int r0 = m * st.r + 8 * v;
      uint32_t wds[4][4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint4 u = *reinterpret_cast<const uint4*>(Uh + ((size_t)m * D + d0 + q) * st.r + 8 * v);
        wds[q][0] = u.x; wds[q][1] = u.y; wds[q][2] = u.z; wds[q][3] = u.w;
        *reinterpret_cast<uint2*>(UN + (size_t)(d0 + q) * UN_LD + perm_col(r0)) = make_uint2(u.x, u.y);
        *reinterpret_cast<uint2*>(UN + (size_t)(d0 + q) * UN_LD + perm_col(r0 + 4)) = make_uint2(u.z, u.w);
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int sh = 16 * (e & 1);
        const uint32_t lo = ((wds[0][e >> 1] >> sh) & 0xffffu) | (((wds[1][e >> 1] >> sh) & 0xffffu) << 16);
        const uint32_t hi = ((wds[2][e >> 1] >> sh) & 0xffffu) | (((wds[3][e >> 1] >> sh) & 0xffffu) << 16);
        *reinterpret_cast<uint2*>(UT + (size_t)(r0 + e) * UT_LD + d0) = make_uint2(lo, hi);
      }
    }
    for (int r = threadIdx.x; r < Rpad; r += kEditThreads) {
      float c = 0.f;
      if (r < R) c = gain * (st.w ? st.w[((size_t)b * Hkv + h) * st.M + r / st.r] : 1.f);
      cvec[r] = c;
    }
  }
  __syncthreads();

  if (!wave_hl) {
    copy_out();
    return;
  }

  // ---- Z^T = U^T K^T, scaled by c_r and by the token's mask bit; packed as the next B operand ----
  // (a group without a highlighted token rides along: its mask bits are zero, its correction is exactly zero
  // and its keys come out bit for bit as they went in)
  float mbit[TG];
#pragma unroll
  for (int tg = 0; tg < TG; ++tg) mbit[tg] = mk[tg] != 0 ? 1.f : 0.f;
  constexpr int MAXKS2 = SEKA_MAX_RANK / 32;
  bf16x8 zb[TG][MAXKS2];
  const int nks2 = Rpad / 32;
#pragma unroll
  for (int ks2 = 0; ks2 < MAXKS2; ++ks2) {
    if (ks2 < nks2) {
      float zc[TG][8];
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int rb = 2 * ks2 + half;
        f32x4 acc[TG];
#pragma unroll
        for (int tg = 0; tg < TG; ++tg) acc[tg] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          bf16x8 a;
          if (WIDE) {
            // U^T fragment (row r = 16 rb + j, k = d = 32 s + 8 g + e) out of the row-d layout: a group of 16 lanes
            // reads 4 rows x 16 columns (lane: row d0 + j / 4, columns 16 rb + 4 (j % 4) ..) and receives them transposed
            const uint16_t* up = UN + (size_t)(32 * s + 8 * g + (j >> 2)) * UN_LD + 16 * rb + 4 * (j & 3);
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((edit_lds_s16x4_ptr)(up));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((edit_lds_s16x4_ptr)(up + 4 * UN_LD));
            a = __builtin_shufflevector(__builtin_bit_cast(bf16x4, lo), __builtin_bit_cast(bf16x4, hi), 0, 1, 2, 3, 4, 5, 6, 7);
          } else {
            a = *reinterpret_cast<const bf16x8*>(UT + (size_t)(16 * rb + j) * UT_LD + 32 * s + 8 * g);
          }
#pragma unroll
          for (int tg = 0; tg < TG; ++tg) acc[tg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, kreg[tg][s], acc[tg], 0, 0, 0);
        }
        const f32x4 c4 = *reinterpret_cast<const f32x4*>(cvec + 16 * rb + 4 * g);
#pragma unroll
        for (int tg = 0; tg < TG; ++tg)
#pragma unroll
          for (int i = 0; i < 4; ++i) zc[tg][4 * half + i] = acc[tg][i] * c4[i] * mbit[tg];
      }
#pragma unroll
      for (int tg = 0; tg < TG; ++tg) {
        bf16x8 z;
#pragma unroll
        for (int e = 0; e < 8; ++e) z[e] = (__bf16)zc[tg][e];
        zb[tg][ks2] = z;
      }
    }
  }

  // ---- C^T = U (c .* Z^T); rows of U are visited in the order that puts d = 32 s + 8 g + e in lane (j, g) ----
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    float outv[TG][8];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int d_row = 32 * s + 8 * (j >> 2) + 4 * half + (j & 3);
      f32x4 acc[TG];
#pragma unroll
      for (int tg = 0; tg < TG; ++tg) acc[tg] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks2 = 0; ks2 < MAXKS2; ++ks2) {
        if (ks2 < nks2) {
          bf16x8 a;
          if (WIDE) {
            // slot e of lane (j, g) is column r = 32 ks2 + 16 (e / 4) + 4 g + e % 4: two 8-byte pieces of row d_row
            const uint16_t* up = UN + (size_t)d_row * UN_LD + 32 * ks2 + 4 * g;
            a = __builtin_shufflevector(*reinterpret_cast<const bf16x4*>(up), *reinterpret_cast<const bf16x4*>(up + 16), 0, 1, 2, 3, 4, 5, 6, 7);
          } else {
            a = *reinterpret_cast<const bf16x8*>(UN + (size_t)d_row * UN_LD + 32 * ks2 + 8 * g);
          }
#pragma unroll
          for (int tg = 0; tg < TG; ++tg) acc[tg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, zb[tg][ks2], acc[tg], 0, 0, 0);
        }
      }
#pragma unroll
      for (int tg = 0; tg < TG; ++tg)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          outv[tg][4 * half + i] = (float)kreg[tg][s][4 * half + i] * (1.f + mbit[tg] * (kscale - 1.f)) + acc[tg][i];
    }
#pragma unroll
    for (int tg = 0; tg < TG; ++tg) {
      bf16x8 o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (__bf16)outv[tg][e];
      if (valid[tg] && (!inplace || mk[tg] != 0))
        *reinterpret_cast<uint4*>(K_out + row_off[tg] + 32 * s + 8 * g) = __builtin_bit_cast(uint4, o);
    }
  }
}

// fp32 path (small problems, exactness over speed): one workgroup = 16 tokens of one KV head.
template <int D>
__global__ __launch_bounds__(kEditThreads) void edit_keys_f32_kernel(const float* __restrict__ K_in,
                                                                     float* __restrict__ K_out, int S, int Hkv,
                                                                     SteerArgs st, int inplace,
                                                                     const int* __restrict__ cu, int total) {
  constexpr int TT = 16;
  __shared__ float ktile[TT][D];
  __shared__ float z[TT][SEKA_MAX_RANK];
  __shared__ int mtile[TT];
  const int b = blockIdx.z, h = blockIdx.y;
  const int t0 = blockIdx.x * TT;
  const float gain = st.gain[h];
  const float kscale = st.kscale[h];
  const int R = st.M * st.r;
  size_t tok0;
  int len;
  edit_prompt_extent(cu, total, b, S, tok0, len);
  int any = 0;
  if (threadIdx.x < TT) {
    const int t = t0 + threadIdx.x;
    const int mk = (t < len) ? st.mask[tok0 + t] : 0;
    mtile[threadIdx.x] = mk;
    any = mk != 0;
  }
  const bool steered = __syncthreads_or(any) != 0 && gain != 0.f;
  for (int i = threadIdx.x; i < TT * D; i += kEditThreads) {
    const int tt = i / D, d = i % D, t = t0 + tt;
    ktile[tt][d] = (t < len) ? K_in[((tok0 + t) * Hkv + h) * D + d] : 0.f;
  }
  __syncthreads();
  if (steered) {
    const float* Uh = static_cast<const float*>(st.U) + (size_t)h * st.M * D * st.r;
    for (int i = threadIdx.x; i < TT * R; i += kEditThreads) {
      const int tt = i / R, r = i % R, m = r / st.r, rr = r % st.r;
      float acc = 0.f;
      if (mtile[tt]) {
        const float* u = Uh + (size_t)m * D * st.r + rr;
        for (int d = 0; d < D; ++d) acc = fmaf(u[(size_t)d * st.r], ktile[tt][d], acc);
        acc *= gain * (st.w ? st.w[((size_t)b * Hkv + h) * st.M + m] : 1.f);
      }
      z[tt][r] = acc;
    }
    __syncthreads();
  }
  for (int i = threadIdx.x; i < TT * D; i += kEditThreads) {
    const int tt = i / D, d = i % D, t = t0 + tt;
    if (t >= len) continue;
    float v = ktile[tt][d];
    const bool edited = steered && mtile[tt];
    if (edited) {
      const float* Uh = static_cast<const float*>(st.U) + (size_t)h * st.M * D * st.r;
      float acc = 0.f;
      for (int r = 0; r < R; ++r) {
        const int m = r / st.r, rr = r % st.r;
        acc = fmaf(Uh[((size_t)m * D + d) * st.r + rr], z[tt][r], acc);
      }
      v = fmaf(kscale, v, acc);
    }
    if (!inplace || edited) K_out[((tok0 + t) * Hkv + h) * D + d] = v;
  }
}

}  // namespace

hipError_t launch_edit_keys(const void* K_in, void* K_out, int B, int S, int Hkv, int D, int dtype,
                            const SteerArgs& steer, hipStream_t s, const int* cu, int total) {
  const int inplace = (K_in == K_out) ? 1 : 0;
  if (dtype == SEKA_BF16) {
    const int R = steer.M * steer.r;
    const int Rpad = (R + 31) / 32 * 32;
    const bool wide = Rpad > 64;          // see the kernel (at smaller ranks the two-copy form measured the same or faster): one staged copy of U, 128-token tiles
    const size_t smem = ((wide ? 0 : (size_t)Rpad * (D + 8)) + (size_t)D * (Rpad + 8)) * 2 + (size_t)Rpad * 4;
    const int tok = wide ? 2 * kEditTokens : kEditTokens;
    const dim3 grid((S + tok - 1) / tok, Hkv, B);
    auto launch = [&](auto kernel) -> hipError_t {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      if (e != hipSuccess) return e;
      hipLaunchKernelGGL(kernel, grid, dim3(kEditThreads), smem, s, static_cast<const uint16_t*>(K_in),
                         static_cast<uint16_t*>(K_out), S, Hkv, steer, inplace, Rpad, cu, total);
      return hipGetLastError();
    };
    if (wide) return D == 128 ? launch(edit_keys_bf16_kernel<128, 2>) : launch(edit_keys_bf16_kernel<64, 2>);
    return D == 128 ? launch(edit_keys_bf16_kernel<128, 1>) : launch(edit_keys_bf16_kernel<64, 1>);
  }
  const dim3 grid((S + 15) / 16, Hkv, B);
  if (D == 128)
    hipLaunchKernelGGL(edit_keys_f32_kernel<128>, grid, dim3(kEditThreads), 0, s, static_cast<const float*>(K_in),
                       static_cast<float*>(K_out), S, Hkv, steer, inplace, cu, total);
  else
    hipLaunchKernelGGL(edit_keys_f32_kernel<64>, grid, dim3(kEditThreads), 0, s, static_cast<const float*>(K_in),
                       static_cast<float*>(K_out), S, Hkv, steer, inplace, cu, total);
  return hipGetLastError();
}

}  // namespace seka
