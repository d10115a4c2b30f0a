// LDS tile layouts, global->LDS DMA and MFMA operand reads shared by the attention kernels (gfx950).
//
// Every MFMA operand is fetched with one 16-byte LDS read per lane (8 bf16 along the contraction index).
// Tiles are stored as rows of 16-byte chunks; the chunk position inside a row is permuted per row
// ("swizzle") so that the 16 lanes served together by a ds_read_b128 -- 16 consecutive rows, same logical
// chunk -- fall on 16 distinct bank groups.  Tiles are filled by global_load_lds (the data never passes
// through registers): lane x of a wave-wide load writes LDS bytes [16 x, 16 x + 16) past a wave-uniform
// base, so each lane simply fetches the global chunk that belongs at its LDS position.
#pragma once
#include <type_traits>

#include "device_common.hpp"

namespace chunk_attn {

// physical chunk position of logical chunk c in row `row` of a tile with CHUNKS 16-byte chunks per row
template <int CHUNKS>
__device__ __forceinline__ int swz(int row, int c) {
  if constexpr (CHUNKS == 32) {
    // 512-byte rows: every row starts on the same bank, so the chunk is rotated by the row index; 16 consecutive rows then
    // fall on 16 distinct bank groups
    return (c + row) & 31;
  } else if constexpr (CHUNKS == 16) {
    // 256-byte rows: rotate by a 4x4 bit-transposed row index; conflict-free for 16 consecutive rows
    const int f = ((row & 3) << 2) | ((row >> 2) & 3);
    return (c + f) & 15;
  } else if constexpr (CHUNKS == 8) {
    // 128-byte rows: two rows share a 256-byte bank line, so the permutation changes every other row
    return c ^ ((row >> 1) & 7);
  } else {
    static_assert(CHUNKS == 4, "tiles have 4, 8, 16 or 32 chunks per row");
    // 64-byte rows: four rows share a bank line
    return c ^ ((row >> 2) & 3);
  }
}
// logical chunk stored at physical position pc (inverse of swz)
template <int CHUNKS>
__device__ __forceinline__ int unswz(int row, int pc) {
  if constexpr (CHUNKS == 32) {
    return (pc - row) & 31;
  } else if constexpr (CHUNKS == 16) {
    const int f = ((row & 3) << 2) | ((row >> 2) & 3);
    return (pc - f) & 15;
  } else if constexpr (CHUNKS == 8) {
    return pc ^ ((row >> 1) & 7);
  } else {
    return pc ^ ((row >> 2) & 3);
  }
}
// element offset of (row, logical chunk c) in a swizzled tile
template <int CHUNKS>
__device__ __forceinline__ int tile_elem(int row, int c) {
  return (row * CHUNKS + swz<CHUNKS>(row, c)) * 8;
}

__device__ __forceinline__ void dma4(const void* gsrc, void* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 4, 0, 0);
}
__device__ __forceinline__ void dma16(const void* gsrc, void* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}

// Explicit LDS address-space pointers: accesses through them are always ds_* instructions, whatever the
// compiler can or cannot prove about a generic pointer.
typedef __attribute__((address_space(3))) __bf16 lds_bf16;
typedef __attribute__((address_space(3))) float lds_f32;
__device__ __forceinline__ bf16x8 lds_load8(const lds_bf16* p) {
  return *(const __attribute__((address_space(3))) bf16x8*)p;
}
__device__ __forceinline__ void lds_store8(lds_bf16* p, bf16x8 v) { *(__attribute__((address_space(3))) bf16x8*)p = v; }
__device__ __forceinline__ f32x4 lds_load4f(const lds_f32* p) {
  return *(const __attribute__((address_space(3))) f32x4*)p;
}
// LDS transpose read (ds_read_b64_tr_b16), see device_common.hpp
__device__ __forceinline__ s16x4 lds_read_tr(const lds_bf16* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
}
__device__ __forceinline__ void dma4(const void* gsrc, lds_f32* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 4, 0, 0);
}
__device__ __forceinline__ void dma16(const void* gsrc, lds_bf16* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}

// DMA a row-major tile of ROWS x (8 CHUNKS) bf16 from global rows `src + min(r, last_row) * row_stride`
// into a swizzled LDS tile.  Called by all 256 threads of the workgroup.
template <int ROWS, int CHUNKS>
__device__ __forceinline__ void dma_rows_tile(const __bf16* src, int64_t row_stride, int last_row, __bf16* lds_tile,
                                              int wave, int lane) {
  constexpr int N = ROWS * CHUNKS / 256;  // instructions per thread
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const int x0 = (i * 4 + wave) * 64;   // wave-uniform first chunk of this instruction
    const int x = x0 + lane;
    const int row = x / CHUNKS, pc = x % CHUNKS;
    const int c = unswz<CHUNKS>(row, pc);
    dma16(src + (int64_t)min(row, last_row) * row_stride + c * 8, lds_tile + x0 * 8);
  }
}

// DMA a contiguous image of BYTES bytes (already in LDS order) into LDS.
template <int BYTES>
__device__ __forceinline__ void dma_image(const __bf16* src, __bf16* lds_tile, int wave, int lane) {
  constexpr int N = BYTES / 16 / 256;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const int x0 = (i * 4 + wave) * 64;
    dma16(src + (int64_t)(x0 + lane) * 8, lds_tile + x0 * 8);
  }
}

// Workgroup barrier without the memory fence of __syncthreads(): the fence would wait for every outstanding
// global->LDS copy, including the ones prefetching later stages.  Callers wait (s_waitcnt vmcnt) for exactly
// the copies the next stage needs before calling this; LDS reads of the finished stage have completed
// because their values were consumed.
__device__ __forceinline__ void wg_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Two waves that share a SIMD and run the same MFMA-phase / VALU-phase loop tend to fall into lockstep:
// both want the matrix pipe at the same time, then both want the vector ALU, and the two pipes never
// overlap.  Giving the waves of one SIMD different issue priorities (by the parity of their hardware
// wave slot) breaks the symmetry: the favoured wave runs its phases back to back and the other one
// fills the gaps, so matrix and vector work of different waves overlap.
__device__ __forceinline__ void stagger_wave_priority() {
  // HW_REG_HW_ID (register 4), bits [3:0] = wave slot on the SIMD
  const unsigned slot = __builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 4);
  if (slot & 1) __builtin_amdgcn_s_setprio(3);
  else __builtin_amdgcn_s_setprio(0);
}

// 8 bf16 of (row, logical chunk c)
template <int CHUNKS>
__device__ __forceinline__ bf16x8 lds_chunk(const __bf16* tile, int row, int c) {
  return *reinterpret_cast<const bf16x8*>(tile + tile_elem<CHUNKS>(row, c));
}

// Position p (0..63) of a 64-wide transposed tile row holds contraction index cperm(p): the order in which
// an accumulator tile presents its rows when it is reused as a B operand (device_common.hpp, "C-order").
__host__ __device__ __forceinline__ int cperm(int p) {
  return (p & ~15) | ((p & 4) << 1) | ((p & 8) >> 1) | (p & 3);
}

// Chunk-major tile of 32 rows (rows of Q, dO, K or V: D / 8 chunks of 16 bytes each): chunk c of row r sits at slot
// c * 32 + (r ^ 4 (c & 3)).  Such a tile serves both as rows (16-byte reads: operand X[row][k]) and transposed
// (ds_read_b64_tr_b16: operand X^T[column][row]), both kinds of read bank-conflict free and their addresses one
// per-lane base plus constants.  cm_elem: element offset of (row r, chunk c).
__device__ __forceinline__ int cm_elem(int r, int c) { return (c * 32 + (r ^ ((c & 3) << 2))) * 8; }

// LDS accesses as opaque instructions, for the software-pipelined kernels.  The compiler makes a wave wait for ALL of its
// outstanding global->LDS copies before an LDS read it cannot tell apart from their destinations (the
// transpose read in particular), which would serialise the copies of later stages with the reads of the
// current one.  Issued like this, the reads are invisible to that logic; the kernels order them themselves with
// explicit s_waitcnt lgkmcnt(n) (LDS operations of a wave complete in order).  `addr` is a byte address.
template <int OFF>
__device__ __forceinline__ bf16x8 lds_asm_read16(unsigned addr) {
  bf16x8 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
}
template <int OFF>
__device__ __forceinline__ f32x4 lds_asm_read16f(unsigned addr) {
  f32x4 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
}
template <int OFF>
__device__ __forceinline__ s16x4 lds_asm_read_tr(unsigned addr) {
  s16x4 v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
}
template <int OFF>
__device__ __forceinline__ void lds_asm_write16(unsigned addr, bf16x8 v) {
  asm volatile("ds_write_b128 %0, %1 offset:%2" : : "v"(addr), "v"(v), "n"(OFF) : "memory");
}
__device__ __forceinline__ unsigned lds_addr(const lds_bf16* p) { return (unsigned)(uintptr_t)p; }
__device__ __forceinline__ unsigned lds_addr(const lds_f32* p) { return (unsigned)(uintptr_t)p; }

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

}  // namespace chunk_attn
