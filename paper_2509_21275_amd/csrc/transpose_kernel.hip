// Pre-pass that prepares transposed operand tiles.
//
// For X[rows][H][D] (bf16) and a list of W-row tiles (W = 64 or 32), writes for every (head, tile) an "image"
// T[D][W] with T[c][p] = X[row0 + cperm(p)][head][c] (zero past the tile's valid rows), already in
// the swizzled chunk order in which the attention kernels keep it in LDS.  The attention kernels then
// fetch an image with a linear global->LDS copy and read MFMA operands whose contraction index runs
// along X's row index (V^T for O += P V, K^T for dQ += dS K, Q^T and dO^T for dK, dV) with plain
// 16-byte LDS reads.  Cost: one read and one write of X, negligible next to the attention itself.
#include "kernels.hpp"
#include "tiles.hpp"

namespace chunk_attn {

template <int D, int W>
__global__ __launch_bounds__(256) void transpose_tiles_kernel(const __bf16* __restrict__ x, int num_heads,
                                                              const TileJob* __restrict__ jobs, int64_t total_tiles,
                                                              __bf16* __restrict__ out, const int32_t* __restrict__ gate) {
  if (gate && *gate == 0) return;
  constexpr int P = D + 2;  // LDS pitch (elements) of the staging tile
  __shared__ __bf16 stage[W * P];
  const int tid = threadIdx.x;
  const int h = blockIdx.x % num_heads;
  const TileJob job = jobs[blockIdx.x / num_heads];
  const int64_t stride = (int64_t)num_heads * D;
  for (int idx = tid; idx < W * (D / 8); idx += 256) {
    const int row = idx / (D / 8), c = idx % (D / 8);
    bf16x8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (__bf16)0.0f;
    if (row < job.valid_rows) v = *reinterpret_cast<const bf16x8*>(x + ((int64_t)job.src_row0 + row) * stride + (int64_t)h * D + c * 8);
#pragma unroll
    for (int i = 0; i < 8; ++i) stage[row * P + c * 8 + i] = v[i];
  }
  __syncthreads();
  __bf16* img = out + ((int64_t)h * total_tiles + job.image) * (D * W);
  constexpr int WC = W / 8;
  for (int idx = tid; idx < D * WC; idx += 256) {
    const int d = idx / WC, pc = idx % WC;
    const int c = unswz<WC>(d, pc);
    bf16x8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = stage[cperm(8 * c + i) * P + d];
    *reinterpret_cast<bf16x8*>(img + (int64_t)idx * 8) = v;
  }
}

template <int D, int W>
static void launch_t(const __bf16* x, int num_heads, const TileJob* jobs, int64_t blocks, int64_t total_tiles,
                     __bf16* out, hipStream_t stream, const int32_t* gate) {
  hipLaunchKernelGGL((transpose_tiles_kernel<D, W>), dim3((unsigned)blocks), dim3(256), 0, stream, x, num_heads, jobs,
                     total_tiles, out, gate);
}

hipError_t launch_transpose(const __bf16* x, int num_heads, int head_dim, int width, const TileJob* jobs, int num_jobs,
                            int64_t total_tiles, __bf16* out, hipStream_t stream, const int32_t* gate) {
  if (num_jobs == 0) return hipSuccess;
  const int64_t blocks = (int64_t)num_jobs * num_heads;
  if (blocks > 0x7fffffff) return hipErrorInvalidValue;
  if (head_dim == 128 && width == 64) launch_t<128, 64>(x, num_heads, jobs, blocks, total_tiles, out, stream, gate);
  else if (head_dim == 128 && width == 32) launch_t<128, 32>(x, num_heads, jobs, blocks, total_tiles, out, stream, gate);
  else if (head_dim == 64 && width == 64) launch_t<64, 64>(x, num_heads, jobs, blocks, total_tiles, out, stream, gate);
  else if (head_dim == 64 && width == 32) launch_t<64, 32>(x, num_heads, jobs, blocks, total_tiles, out, stream, gate);
  else if (head_dim == 256 && width == 64) launch_t<256, 64>(x, num_heads, jobs, blocks, total_tiles, out, stream, gate);
  else if (head_dim == 256 && width == 32) launch_t<256, 32>(x, num_heads, jobs, blocks, total_tiles, out, stream, gate);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace chunk_attn
