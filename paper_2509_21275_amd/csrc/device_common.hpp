// Device-side building blocks shared by the chunk-attention kernels (gfx950 only).
//
// MFMA v_mfma_f32_32x32x16_bf16 operand layout (wave of 64 lanes, l32 = lane % 32, hh = lane / 32):
//   A (32 x 16): lane holds A[row = l32][k = 8 hh .. 8 hh + 7]
//   B (16 x 32): lane holds B[k = 8 hh .. 8 hh + 7][col = l32]
//   C (32 x 32): lane holds C[row = 8 g + 4 hh + r][col = l32] in acc[4 g + r], g, r = 0..3
// The k slots of A and B only have to agree with each other, which lets an accumulator
// tile be fed straight back as a B operand: slot e of half hh in k-step s then stands for
// contraction index 16 s + 8 (e / 4) + 4 hh + (e % 4)   ("C-order"), and the matching A
// operand is gathered in that order with the LDS transpose read below.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace chunk_attn {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Idles long enough for the last MFMA's results to be written back (for code that reads results of MFMAs the
// compiler does not know about).
__device__ __forceinline__ void mfma_settle() { asm volatile("s_nop 15\n\ts_nop 7" ::: "memory"); }

// value of the lane 32 away
__device__ __forceinline__ float other_half(float x) {
  u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  // lanes < 32 hold {own, partner} in {r0, r1}; lanes >= 32 hold {partner, own}
  return (threadIdx.x & 32) ? __uint_as_float(r[0]) : __uint_as_float(r[1]);
}
__device__ __forceinline__ float max_halves(float x) {
  u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_halves(float x) {
  u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Pack 8 floats to bf16 (round to nearest even, hardware conversion).
__device__ __forceinline__ bf16x8 pack8(float a0, float a1, float a2, float a3, float a4, float a5, float a6,
                                        float a7) {
  bf16x8 r;
  r[0] = (__bf16)a0; r[1] = (__bf16)a1; r[2] = (__bf16)a2; r[3] = (__bf16)a3;
  r[4] = (__bf16)a4; r[5] = (__bf16)a5; r[6] = (__bf16)a6; r[7] = (__bf16)a7;
  return r;
}
__device__ __forceinline__ bf16x4 pack4(float a0, float a1, float a2, float a3) {
  bf16x4 r;
  r[0] = (__bf16)a0; r[1] = (__bf16)a1; r[2] = (__bf16)a2; r[3] = (__bf16)a3;
  return r;
}

// LDS transpose read (ds_read_b64_tr_b16).  Inside each group of 16 lanes, lane i receives,
// for e = 0..3, 16-bit element (i % 4) of the 8 bytes addressed by lane (i / 4 + 4 e) of the group.
__device__ __forceinline__ s16x4 lds_read_tr(const __bf16* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, p));
}

// ---- clock log of a persistent workgroup (measurement only) ----
// When the caller of the library has asked for it, the first lane of every persistent workgroup records two counters
// when it starts (`end` = 0) and when it has run out of blocks (`end` = 1): the constant 100 MHz counter and the
// shader-clock counter.  The ratio of the two differences is the clock the kernel ran at.  Entry of workgroup b:
// {100 MHz start, 100 MHz end, shader clock start, shader clock end}.  Grids beyond kClockLogWorkgroups are not logged.
constexpr int kClockLogWorkgroups = 1024;
__device__ __forceinline__ void clock_log_stamp(unsigned long long* log, int end) {
  if (log != nullptr && threadIdx.x == 0 && blockIdx.x < kClockLogWorkgroups) {
    unsigned long long* e = log + 4 * blockIdx.x + end;
    e[0] = __builtin_amdgcn_s_memrealtime();
    e[2] = __builtin_amdgcn_s_memtime();
  }
}

// ---- dynamic assignment of a launch's blocks to persistent workgroups ----
// A launch has `total` blocks of work (what used to be one workgroup each).  They are dealt to eight queues by index
// modulo 8: a grid's workgroup b normally runs on XCD b % 8, so the host's block order already puts blocks that share data
// (the same key/value head) on one XCD, whose L2 then serves the stream they share.  One workgroup per CU is launched;
// it takes blocks from the queue of the XCD it runs on, front to back (the host puts long sequences first and ends every sequence with its short blocks), and once
// that queue is empty from the queue with the most blocks left.  The XCDs of a chip do not run at the same speed (their
// finishing times differed by 4 - 7 % with a fixed share each); this way the fast ones take over what the slow ones
// have not started, and only the blocks taken over lose their L2 neighbourhood.  `taken` (device, 8 counters, zero when
// the kernel starts) counts the claims per queue; an index past the end of a queue means it is empty.  No workgroup
// ever waits for another one.
__device__ __forceinline__ int xcd_of_this_wave() { return __builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 20) & 7; }
__device__ __forceinline__ int block_queue_len(int total, int x) { return total > x ? (total - x + 7) >> 3 : 0; }
// Claim of the next block of queue x, issued by lane 0 without waiting for the answer (the caller reads `idx` later).
__device__ __forceinline__ int block_claim_issue(int32_t* taken, int x) {
  int idx = 0;
  if ((threadIdx.x & 63) == 0) idx = __hip_atomic_fetch_add(taken + x, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return idx;
}
// Turns the answer of block_claim_issue into a block index, or finds a block in another queue; -1: nothing is left.
// Called by one whole wave; the result is wave-uniform.
__device__ __forceinline__ int block_claim_finish(int32_t* taken, int total, int x, int idx) {
  idx = __builtin_amdgcn_readfirstlane(idx);
  if (idx < block_queue_len(total, x)) return x + 8 * idx;
  const int lane = threadIdx.x & 63;
  // a failed claim proves its queue empty for good (the counters only grow), so eight rounds see every queue empty
  for (int round = 0; round < 8; ++round) {
    int left = 0;
    if (lane < 8)
      left = block_queue_len(total, lane) - __hip_atomic_load(taken + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int best = 0, y = -1;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int l = __builtin_amdgcn_readlane(left, i);
      if (l > best) {
        best = l;
        y = i;
      }
    }
    if (y < 0) return -1;
    idx = __builtin_amdgcn_readfirstlane(block_claim_issue(taken, y));
    if (idx < block_queue_len(total, y)) return y + 8 * idx;
  }
  return -1;
}
// Hands a wave-uniform value of wave 0 to the whole workgroup through `slot` (LDS).  Contains a workgroup barrier
// without a memory fence: outstanding global stores are not waited for.
// Blocks that read the same rows side by side (one queue = one key/value head's blocks, `width` of them at a time): a
// block marked for it starts only when `ended[queue]`, the number of the queue's blocks that have ended, has reached the
// first index of its group of `width`.  Called by one wave for block `blk` (>= 0); the wait is bounded (the blocks
// waited for were claimed earlier and are running, so it ends by itself; the bound only keeps a surprise from turning
// into a hang) and nothing but timing depends on it.
__device__ __forceinline__ void wait_for_earlier_groups(const int32_t* ended, int blk, int width) {
  const int need = (blk / 8) / width * width;
  if (need == 0) return;
  for (int spins = 0; spins < 256; ++spins) {
    const int seen = __hip_atomic_load(ended + (blk & 7), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (__builtin_amdgcn_readfirstlane(seen) >= need) break;
    __builtin_amdgcn_s_sleep(32);
  }
}
__device__ __forceinline__ int broadcast_from_wave0(int* slot, int value) {
  if (threadIdx.x == 0) *(volatile int*)slot = value;
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  return __builtin_amdgcn_readfirstlane(*(volatile int*)slot);
}

}  // namespace chunk_attn
