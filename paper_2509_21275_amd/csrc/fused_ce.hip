// Fused in-place cross-entropy (include/fused_ce.h; paper section 4, "Fused In-Place Cross-Entropy").
//
// HBM-bound by construction: one workgroup of 512 threads owns one row of logits at a time, loads it once into
// registers (16 bytes per lane and load, consecutive lanes consecutive chunks: fully coalesced), reduces the
// maximum and the sum of exponentials across the workgroup (wave reductions, then 8 partial results through LDS),
// and stores the gradient over the logits.  Algorithmic traffic: 4 bytes per logit.  The exponential of an element
// is evaluated twice (for the sum and for the gradient) rather than kept: the vector work of a row is several times
// shorter than the time HBM needs to deliver it.  Workgroups walk the rows with a grid stride, the grid sized to a
// few workgroups per compute unit, so that loads of the next row are in flight while a row drains.
#include <hip/hip_runtime.h>

#include "../../include/fused_ce.h"
#include "device_common.hpp"

namespace chunk_attn {
namespace {

constexpr int kThreads = 512;
constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

// NCH: 16-byte chunks per thread (a row has at most 512 * 8 * NCH logits; 32 chunks = 128 registers is what fits)
template <int NCH>
__global__ __launch_bounds__(kThreads) void fused_ce_kernel(__bf16* __restrict__ logits, const int32_t* __restrict__ targets,
                                                            float* __restrict__ loss, int64_t rows, int vocab,
                                                            int64_t row_stride, float grad_scale) {
  __shared__ float red[2][kThreads / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_chunks = vocab / 8;
  for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {
    __bf16* const z = logits + row * row_stride;
    const int y = targets[row];
    const bool ignored = y < 0 || y >= vocab;
    const float zy = ignored ? 0.f : (float)z[y];  // read before the row is overwritten (every thread: one cached load)
    bf16x8 v[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int ch = c * kThreads + tid;
      if (ch < n_chunks) v[c] = *reinterpret_cast<const bf16x8*>(z + (int64_t)ch * 8);
    }
    // Between the three passes the row is kept as it was loaded (packed bf16): the opaque statements stop the compiler
    // from keeping a widened fp32 copy of the whole row alive, which would not fit the register file.
    float mx = -INFINITY;
#pragma unroll
    for (int c = 0; c < NCH; ++c)
      if (c * kThreads + tid < n_chunks) {
#pragma unroll
        for (int e = 0; e < 8; ++e) mx = fmaxf(mx, (float)v[c][e]);
      }
    mx = wave_max(mx);
    if (lane == 0) red[0][wave] = mx;
    __syncthreads();
    mx = red[0][0];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) mx = fmaxf(mx, red[0][w]);
    const float m2 = mx * kLog2e;
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) asm volatile("" : "+v"(v[c]));
#pragma unroll
    for (int c = 0; c < NCH; ++c)
      if (c * kThreads + tid < n_chunks) {
#pragma unroll
        for (int e = 0; e < 8; ++e) sum += __builtin_amdgcn_exp2f((float)v[c][e] * kLog2e - m2);
      }
    sum = wave_sum(sum);
    if (lane == 0) red[1][wave] = sum;
    __syncthreads();
    sum = 0.f;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) sum += red[1][w];
    const float lse2 = m2 + __builtin_amdgcn_logf(sum);  // log2 of the sum of exponentials
    if (tid == 0) loss[row] = ignored ? 0.f : lse2 * kLn2 - zy;
    const float scale = ignored ? 0.f : grad_scale;
#pragma unroll
    for (int c = 0; c < NCH; ++c) asm volatile("" : "+v"(v[c]));
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int ch = c * kThreads + tid;
      if (ch < n_chunks) {
        const int d = y - ch * 8;  // position of the target inside this chunk, if it is there
        bf16x8 g;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float pe = __builtin_amdgcn_exp2f((float)v[c][e] * kLog2e - lse2);
          if (d == e) pe -= 1.0f;
          g[e] = (__bf16)(pe * scale);
        }
        *reinterpret_cast<bf16x8*>(z + (int64_t)ch * 8) = g;
      }
    }
    __syncthreads();  // red[] is reused by the next row
  }
}

// Rows too long for the registers of one workgroup: the same three passes, each reading the row from memory
// (8 bytes per logit).
__global__ __launch_bounds__(kThreads) void fused_ce_stream_kernel(__bf16* __restrict__ logits, const int32_t* __restrict__ targets,
                                                                   float* __restrict__ loss, int64_t rows, int vocab,
                                                                   int64_t row_stride, float grad_scale) {
  __shared__ float red[2][kThreads / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_chunks = vocab / 8;
  for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {
    __bf16* const z = logits + row * row_stride;
    const int y = targets[row];
    const bool ignored = y < 0 || y >= vocab;
    const float zy = ignored ? 0.f : (float)z[y];
    float mx = -INFINITY;
    for (int ch = tid; ch < n_chunks; ch += kThreads) {
      const bf16x8 v = *reinterpret_cast<const bf16x8*>(z + (int64_t)ch * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) mx = fmaxf(mx, (float)v[e]);
    }
    mx = wave_max(mx);
    if (lane == 0) red[0][wave] = mx;
    __syncthreads();
    mx = red[0][0];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) mx = fmaxf(mx, red[0][w]);
    const float m2 = mx * kLog2e;
    float sum = 0.f;
    for (int ch = tid; ch < n_chunks; ch += kThreads) {
      const bf16x8 v = *reinterpret_cast<const bf16x8*>(z + (int64_t)ch * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) sum += __builtin_amdgcn_exp2f((float)v[e] * kLog2e - m2);
    }
    sum = wave_sum(sum);
    if (lane == 0) red[1][wave] = sum;
    __syncthreads();
    sum = 0.f;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) sum += red[1][w];
    const float lse2 = m2 + __builtin_amdgcn_logf(sum);
    if (tid == 0) loss[row] = ignored ? 0.f : lse2 * kLn2 - zy;
    const float scale = ignored ? 0.f : grad_scale;
    for (int ch = tid; ch < n_chunks; ch += kThreads) {
      const bf16x8 v = *reinterpret_cast<const bf16x8*>(z + (int64_t)ch * 8);
      const int d = y - ch * 8;
      bf16x8 g;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float pe = __builtin_amdgcn_exp2f((float)v[e] * kLog2e - lse2);
        if (d == e) pe -= 1.0f;
        g[e] = (__bf16)(pe * scale);
      }
      *reinterpret_cast<bf16x8*>(z + (int64_t)ch * 8) = g;
    }
    __syncthreads();
  }
}

template <int NCH>
hipError_t launch(void* logits, const int32_t* targets, float* loss, int64_t rows, int vocab, int64_t row_stride,
                  float grad_scale, hipStream_t stream) {
  // two workgroups per compute unit when the registers allow it, rows dealt round robin
  const int64_t grid = rows < 512 ? rows : 512;
  hipLaunchKernelGGL((fused_ce_kernel<NCH>), dim3((unsigned)grid), dim3(kThreads), 0, stream, (__bf16*)logits, targets, loss,
                     rows, vocab, row_stride, grad_scale);
  return hipGetLastError();
}

}  // namespace
}  // namespace chunk_attn

extern "C" int fused_ce_inplace(void* logits, const int32_t* targets, float* loss, int64_t rows, int32_t vocab,
                                int64_t row_stride, float grad_scale, void* hip_stream) {
  using namespace chunk_attn;
  if (rows < 0 || vocab < 8 || row_stride < vocab) return CHUNK_ATTN_INVALID_ARG;
  if (vocab % 8 != 0 || row_stride % 8 != 0 || vocab > FUSED_CE_MAX_VOCAB) return CHUNK_ATTN_UNSUPPORTED;
  if (rows == 0) return CHUNK_ATTN_OK;  // nothing to do (the pointers of empty buffers may be null)
  if (!logits || !targets || !loss || ((uintptr_t)logits & 15) != 0) return CHUNK_ATTN_INVALID_ARG;
  hipStream_t s = (hipStream_t)hip_stream;
  const int per_thread = (vocab / 8 + kThreads - 1) / kThreads;
  hipError_t e;
  if (per_thread <= 8) e = launch<8>(logits, targets, loss, rows, vocab, row_stride, grad_scale, s);
  else if (per_thread <= 16) e = launch<16>(logits, targets, loss, rows, vocab, row_stride, grad_scale, s);
  else if (per_thread <= 32) e = launch<32>(logits, targets, loss, rows, vocab, row_stride, grad_scale, s);
  else {  // more than 131072 logits per row
    const int64_t grid = rows < 512 ? rows : 512;
    hipLaunchKernelGGL(fused_ce_stream_kernel, dim3((unsigned)grid), dim3(kThreads), 0, s, (__bf16*)logits, targets, loss, rows,
                       vocab, row_stride, grad_scale);
    e = hipGetLastError();
  }
  return e == hipSuccess ? CHUNK_ATTN_OK : CHUNK_ATTN_HIP_ERROR;
}
