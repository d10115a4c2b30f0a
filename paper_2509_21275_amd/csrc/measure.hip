// Measurement hook: the rate at which this GPU sustains nothing but bf16 matrix instructions.
//
// The published bf16 peak of the MI355X (2516.6 TFLOP/s) is 256 CUs x 4096 flop per clock x the 2.4 GHz peak engine
// clock.  Under sustained matrix load the chip runs at a lower clock, so no kernel reaches that figure; what the clock
// allows is measured here by a kernel that issues only independent v_mfma_f32_32x32x16_bf16 on random operands (the
// operand values matter: the power drawn, and with it the clock, depends on the bits that toggle), one workgroup of
// four waves per CU, for a given wall time.  bench.py reports the attention kernels against both figures.
#include <hip/hip_runtime.h>

#include "../../include/chunk_attn.h"
#include "device_common.hpp"

namespace chunk_attn {
namespace {

__global__ __launch_bounds__(256, 1) void mfma_rate_kernel(const unsigned short* __restrict__ src, float* __restrict__ out,
                                                           int iters) {
  const int lane = threadIdx.x & 63;
  const bf16x8 a = *reinterpret_cast<const bf16x8*>(src + lane * 8);
  const bf16x8 b = *reinterpret_cast<const bf16x8*>(src + 512 + lane * 8);
  f32x16 c[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) c[j][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int h = 0; h < 8; ++h) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c[h & 3]) : "v"(a), "v"(b));
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += c[j][i];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void fill_operands_kernel(unsigned short* dst, int n) {
  // bf16 values of either sign with magnitudes in [1/16, 4) and pseudo-random mantissas (a multiplicative hash of the
  // index): like the attention operands, most bits of an operand differ from its neighbour's
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) {
    const unsigned h = (unsigned)i * 2654435761u;
    const unsigned sign = (h >> 31) & 1u, expo = 0x7bu + ((h >> 27) % 6u), mant = (h >> 12) & 0x7fu;
    dst[i] = (unsigned short)((sign << 15) | (expo << 7) | mant);
  }
}

}  // namespace
}  // namespace chunk_attn

namespace {
int measure_mfma_rate(int milliseconds, int workgroups, void* scratch, size_t scratch_bytes, void* stream_v, double* tflops);
}

extern "C" int chunk_attn_measure_mfma_rate(int milliseconds, void* scratch, size_t scratch_bytes, void* stream_v,
                                            double* tflops) {
  return measure_mfma_rate(milliseconds, 0, scratch, scratch_bytes, stream_v, tflops);
}

extern "C" int chunk_attn_measure_mfma_rate_on(int milliseconds, int workgroups, void* scratch, size_t scratch_bytes,
                                               void* stream_v, double* tflops) {
  if (workgroups < 1) return CHUNK_ATTN_INVALID_ARG;
  return measure_mfma_rate(milliseconds, workgroups, scratch, scratch_bytes, stream_v, tflops);
}

namespace {
// workgroups == 0: one per CU
int measure_mfma_rate(int milliseconds, int workgroups, void* scratch, size_t scratch_bytes, void* stream_v, double* tflops) {
  using namespace chunk_attn;
  constexpr size_t kNeed = 4096 + 1024 * 256 * sizeof(float);   // operands, then one float per thread of up to 1024 workgroups
  if (!scratch || !tflops || milliseconds < 1 || milliseconds > 10000) return CHUNK_ATTN_INVALID_ARG;
  if (scratch_bytes < kNeed || (reinterpret_cast<uintptr_t>(scratch) & 255) != 0) return CHUNK_ATTN_WORKSPACE_TOO_SMALL;
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    return CHUNK_ATTN_HIP_ERROR;
  if (cus < 1 || cus > 1024) return CHUNK_ATTN_HIP_ERROR;
  if (workgroups > cus) return CHUNK_ATTN_INVALID_ARG;
  if (workgroups > 0) cus = workgroups;  // from here on: the number of workgroups launched
  unsigned short* src = static_cast<unsigned short*>(scratch);
  float* out = reinterpret_cast<float*>(static_cast<char*>(scratch) + 4096);
  hipLaunchKernelGGL(fill_operands_kernel, dim3(8), dim3(256), 0, stream, src, 2048);
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return CHUNK_ATTN_HIP_ERROR;
  // A short launch sets the iteration count for about a tenth of the requested time per launch; then launches are repeated
  // until the time is used up, and the last one is the one that counts (the clock has settled by then).
  int iters = 2000;
  float ms = 0.f;
  double best = 0.0;
  float used = 0.f;
  int rc = CHUNK_ATTN_OK;
  for (int round = 0; round < 64 && used < (float)milliseconds; ++round) {
    if (hipEventRecord(e0, stream) != hipSuccess) { rc = CHUNK_ATTN_HIP_ERROR; break; }
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(cus), dim3(256), 0, stream, src, out, iters);
    if (hipEventRecord(e1, stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
        hipEventElapsedTime(&ms, e0, e1) != hipSuccess || hipGetLastError() != hipSuccess) { rc = CHUNK_ATTN_HIP_ERROR; break; }
    used += ms;
    // flops: workgroups x 4 waves x iterations x 8 MFMAs x (32 x 32 x 16 multiply-adds x 2)
    best = (double)cus * 4.0 * iters * 8.0 * 32768.0 / (ms * 1e-3) / 1e12;
    const double want_ms = milliseconds / 10.0;
    if (ms < want_ms) iters = (int)(iters * (want_ms / (ms > 0.01f ? ms : 0.01f))) + 1;
    if (iters > (1 << 24)) iters = 1 << 24;
  }
  if (hipEventDestroy(e0) != hipSuccess || hipEventDestroy(e1) != hipSuccess) rc = CHUNK_ATTN_HIP_ERROR;
  if (rc == CHUNK_ATTN_OK) *tflops = best;
  return rc;
}
}  // namespace
