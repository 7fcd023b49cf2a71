// Tile transport shared by the direct-to-LDS bf16 attention kernels (gfx950, head dimension 128):
//   * K/V tiles (64 keys x 128) go from global memory straight into LDS with global_load_lds
//     (16 bytes per lane, no register staging), two tiles ahead of the math, into rings of three
//     stages.  Completion is tracked with an explicit vmcnt wait followed by the per-tile barrier.
//   * A direct-to-LDS load writes 64 lanes x 16 bytes contiguously, so rows cannot be padded; bank
//     conflicts are avoided by choosing WHICH 16-byte chunk of a row each lane fetches (an XOR
//     swizzle of the chunk index with the row index): K chunks are swizzled by row & 15 (conflict-free
//     16-byte row reads), V chunks by 4 * (row & 3) (conflict-free transposing reads).
#pragma once
#include "common.h"

namespace seka {

constexpr int DMA_BK = 64;                       // keys per tile
constexpr int DMA_D = 128;
constexpr int DMA_TILE_BYTES = DMA_BK * DMA_D * 2;   // 16 KB
constexpr int DMA_STAGES = 3;

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

}  // namespace seka
