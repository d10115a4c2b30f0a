// Chunk attention backward for gfx950 (gradients of L = sum(O .* dO) under the chunk mask of the
// paper's section 3.1; key/value gradients include the context rows, section 2.1 / 3.2.2).
//
// Three kernels:
//   bwd_pre   D_i = <dO_i, O_i> per (head, row), and zero the float32 dQ accumulator;
//   bwd_main  one workgroup per tile of 128 key rows of one key/value head.  It keeps that K/V tile
//             resident (K in LDS and registers, V in registers) and walks over the query heads of the
//             group and over the 64-row query tiles that see the key tile, recomputing
//             P = exp(S - LSE) from the saved log-sum-exp.  dK and dV accumulate in registers over
//             all queries and all heads of the group; dQ contributions are added with float32
//             atomics into the workspace;
//   bwd_post  dQ = bf16(scale * accumulator); zero the key rows no segment covers.
//
// Orientation: S = Q K^T is computed with the key index along lanes, so P and dS come out of the MFMA
// already in B-operand form for dV^T += dO^T P and dK^T += Q^T dS ("C-order", device_common.hpp);
// only dS has to cross lanes (through LDS) for dQ += dS K.
#include "kernels.hpp"

#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

namespace chunk_attn {

namespace {

constexpr int BN = 128;  // key rows per workgroup
constexpr int BM = 64;   // query rows per iteration
constexpr int DSP = 96;  // pitch (elements) of the dS^T tile [BN][BM]

// Element offset inside a row-major bf16 LDS tile with D columns.  D = 128: 256-byte rows whose sixteen
// 16-byte groups are rotated by a per-row amount chosen so that both 16 consecutive rows at one column
// group (row reads of 16 bytes) and 4 consecutive rows x 4 consecutive groups (transpose reads) fall on
// distinct groups.  D = 64: padded rows.
template <int D>
__device__ __forceinline__ int tile_off(int row, int col) {
  if constexpr (D == 128) {
    const int f = ((row & 3) << 2) | ((row >> 2) & 3);
    return row * 128 + ((((col >> 3) + f) & 15) << 3) + (col & 7);
  } else {
    return row * (D + 8) + col;
  }
}
template <int D>
constexpr int tile_elems(int rows) { return D == 128 ? rows * 128 : rows * (D + 8); }

// A operand in C-order gathered from a tile T[k][m] laid out with tile_off<D>.
template <int D>
__device__ __forceinline__ bf16x8 a_tr(const __bf16* tile, int k0, int m0, int lane) {
  const int row = k0 + 4 * (lane >> 5) + ((lane & 15) >> 2);
  const int col = m0 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  s16x4 lo = lds_read_tr(tile + tile_off<D>(row, col));
  s16x4 hi = lds_read_tr(tile + tile_off<D>(row + 8, col));
  s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

template <int D>
__global__ __launch_bounds__(256) void bwd_pre_kernel(const __bf16* __restrict__ o, const __bf16* __restrict__ d_o,
                                                      float* __restrict__ dsum, float* __restrict__ dq_acc,
                                                      int total_q, int num_q_heads) {
  constexpr int LPR = D / 8;  // lanes per (row, head)
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t pair = gid / LPR;  // row * Hq + head
  const int part = (int)(gid % LPR);
  const int64_t n_pairs = (int64_t)total_q * num_q_heads;
  float acc = 0.f;
  if (pair < n_pairs) {
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(o + pair * D + part * 8);
    const bf16x8 b = *reinterpret_cast<const bf16x8*>(d_o + pair * D + part * 8);
#pragma unroll
    for (int i = 0; i < 8; ++i) acc += (float)a[i] * (float)b[i];
    f32x4 z = {0.f, 0.f, 0.f, 0.f};
    *reinterpret_cast<f32x4*>(dq_acc + pair * D + part * 8) = z;
    *reinterpret_cast<f32x4*>(dq_acc + pair * D + part * 8 + 4) = z;
  }
#pragma unroll
  for (int s = LPR / 2; s >= 1; s >>= 1) acc += __shfl_xor(acc, s);
  if (pair < n_pairs && part == 0) {
    const int64_t row = pair / num_q_heads, head = pair % num_q_heads;
    dsum[head * total_q + row] = acc;
  }
}

template <int D>
__global__ __launch_bounds__(256) void bwd_post_kernel(const float* __restrict__ dq_acc, __bf16* __restrict__ dq,
                                                       int64_t n_elems8, float scale) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n_elems8) {
    const f32x4 a = *reinterpret_cast<const f32x4*>(dq_acc + i * 8);
    const f32x4 b = *reinterpret_cast<const f32x4*>(dq_acc + i * 8 + 4);
    *reinterpret_cast<bf16x8*>(dq + i * 8) =
        pack8(a[0] * scale, a[1] * scale, a[2] * scale, a[3] * scale, b[0] * scale, b[1] * scale, b[2] * scale,
              b[3] * scale);
  }
}

// zero `n16` 16-byte units starting at p
__global__ __launch_bounds__(256) void zero_fill_kernel(u32x4* __restrict__ p, int64_t n16) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n16) p[i] = u32x4{0u, 0u, 0u, 0u};
}

template <int D>
__global__ __launch_bounds__(256) void bwd_main_kernel(BwdParams p) {
  constexpr int DK = D / 16;  // k-steps over the head dimension
  constexpr int DB = D / 32;  // 32-row blocks along the head dimension
  constexpr int QCH = BM * D / 8 / 256;  // 16-byte chunks per thread per Q (or dO) tile
  constexpr int KCH = BN * D / 8 / 256;

  extern __shared__ __attribute__((aligned(16))) char smem[];
  __bf16* Kt = reinterpret_cast<__bf16*>(smem);          // [BN][D]
  __bf16* Qt = Kt + tile_elems<D>(BN);                    // [2][BM][D]
  __bf16* Gt = Qt + 2 * tile_elems<D>(BM);                // [2][BM][D]   (dO)
  __bf16* dSt = Gt + 2 * tile_elems<D>(BM);               // [BN][DSP]    (dS^T)
  float* lse_s = reinterpret_cast<float*>(dSt + BN * DSP);  // [2][BM]
  float* dsum_s = lse_s + 2 * BM;                           // [2][BM]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hh = lane >> 5;

  const int kvh = blockIdx.x % p.num_kv_heads;
  const BwdItem it = p.items[blockIdx.x / p.num_kv_heads];
  const int G = p.group;
  const int64_t q_stride = (int64_t)p.num_q_heads * D, kv_stride = (int64_t)p.num_kv_heads * D;
  const float c = p.scale_log2;

  // ---- resident K tile (LDS) and this wave's K / V fragments (registers) ----
  {
    const __bf16* Kg = p.k + (int64_t)it.kv_row0 * kv_stride + (int64_t)kvh * D;
#pragma unroll
    for (int ci = 0; ci < KCH; ++ci) {
      const int idx = tid + 256 * ci;
      const int row = idx / (D / 8), col = (idx % (D / 8)) * 8;
      const int64_t grow = min(row, it.kv_rows - 1);
      *reinterpret_cast<u32x4*>(Kt + tile_off<D>(row, col)) = *reinterpret_cast<const u32x4*>(Kg + grow * kv_stride + col);
    }
  }
  bf16x8 kf[DK], vf[DK];  // B operands: lane holds K[key = 32 wave + l32][16 ks + 8 hh ..+7]
  {
    const int64_t grow = it.kv_row0 + min(32 * wave + l32, it.kv_rows - 1);
    const __bf16* kp = p.k + grow * kv_stride + (int64_t)kvh * D + 8 * hh;
    const __bf16* vp = p.v + grow * kv_stride + (int64_t)kvh * D + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) {
      kf[ks] = *reinterpret_cast<const bf16x8*>(kp + 16 * ks);
      vf[ks] = *reinterpret_cast<const bf16x8*>(vp + 16 * ks);
    }
  }

  f32x16 dkacc[DB], dvacc[DB];  // dK^T, dV^T: [D] x [32 keys of this wave]
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) { dkacc[db][i] = 0.f; dvacc[db][i] = 0.f; }

  const int nqt = (it.q_rows + BM - 1) / BM;
  const int n_iter = nqt * G;

  // ---- Q / dO tile staging ----
  u32x4 qreg[QCH], greg[QCH];
  float lse_reg = 0.f, dsum_reg = 0.f;
  auto load_tiles = [&](int iter) {
    const int hg = iter / nqt, qt = iter % nqt;
    const int head = kvh * G + hg;
    const int rows_left = it.q_rows - qt * BM;  // >= 1
    const int64_t base_row = (int64_t)it.q_row0 + qt * BM;
#pragma unroll
    for (int ci = 0; ci < QCH; ++ci) {
      const int idx = tid + 256 * ci;
      const int row = idx / (D / 8), col = (idx % (D / 8)) * 8;
      const int64_t grow = base_row + min(row, rows_left - 1);
      qreg[ci] = *reinterpret_cast<const u32x4*>(p.q + grow * q_stride + (int64_t)head * D + col);
      greg[ci] = *reinterpret_cast<const u32x4*>(p.d_o + grow * q_stride + (int64_t)head * D + col);
    }
    if (tid < BM) {
      if (tid < rows_left) {
        lse_reg = p.lse[(int64_t)head * p.total_q + base_row + tid] * 1.4426950408889634f;
        dsum_reg = p.dsum[(int64_t)head * p.total_q + base_row + tid];
      } else {
        lse_reg = INFINITY;  // rows past the segment end: P = exp2(S - inf) = 0
        dsum_reg = 0.f;
      }
    }
  };
  auto store_tiles = [&](int buf) {
#pragma unroll
    for (int ci = 0; ci < QCH; ++ci) {
      const int idx = tid + 256 * ci;
      const int row = idx / (D / 8), col = (idx % (D / 8)) * 8;
      *reinterpret_cast<u32x4*>(Qt + buf * tile_elems<D>(BM) + tile_off<D>(row, col)) = qreg[ci];
      *reinterpret_cast<u32x4*>(Gt + buf * tile_elems<D>(BM) + tile_off<D>(row, col)) = greg[ci];
    }
    if (tid < BM) {
      lse_s[buf * BM + tid] = lse_reg;
      dsum_s[buf * BM + tid] = dsum_reg;
    }
  };

  load_tiles(0);
  store_tiles(0);
  __syncthreads();

  for (int iter = 0; iter < n_iter; ++iter) {
    const int buf = iter & 1;
    const int hg = iter / nqt, qt = iter % nqt;
    if (iter + 1 < n_iter) load_tiles(iter + 1);

    const __bf16* Qb = Qt + buf * tile_elems<D>(BM);
    const __bf16* Gb = Gt + buf * tile_elems<D>(BM);

    // ---- S = Q K^T and dP = dO V^T : [64 queries] x [32 keys of this wave] ----
    f32x16 sacc[2], pacc[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int i = 0; i < 16; ++i) { sacc[qb][i] = 0.f; pacc[qb][i] = 0.f; }
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int ks = 0; ks < DK; ++ks) {
        const bf16x8 aq = *reinterpret_cast<const bf16x8*>(Qb + tile_off<D>(32 * qb + l32, 16 * ks + 8 * hh));
        const bf16x8 ag = *reinterpret_cast<const bf16x8*>(Gb + tile_off<D>(32 * qb + l32, 16 * ks + 8 * hh));
        sacc[qb] = mfma32(aq, kf[ks], sacc[qb]);
        pacc[qb] = mfma32(ag, vf[ks], pacc[qb]);
      }

    // ---- P = exp2(S c - LSE), dS = P (dP - D); masked entries give P = dS = 0 ----
    // key index inside the segment of this lane's column, and the first query row of the tile:
    // query row rr (counted from it.q_row0) sees key j iff j < it.n0 + rr.
    const int jkey = it.j0 + 32 * wave + l32;
    const int rr0 = qt * BM;
    bf16x8 pfrag[4], dsfrag[4];  // B operands per k-step of 16 queries
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const bool need_mask = (it.j0 + 32 * wave + 31) >= (it.n0 + rr0 + 32 * qb);
      float pv[16], dsv[16];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 l4 = *reinterpret_cast<const f32x4*>(lse_s + buf * BM + 32 * qb + 8 * g + 4 * hh);
        const f32x4 d4 = *reinterpret_cast<const f32x4*>(dsum_s + buf * BM + 32 * qb + 8 * g + 4 * hh);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int i = 4 * g + r;
          float s = sacc[qb][i] * c - l4[r];
          if (need_mask) {
            const int rr = rr0 + 32 * qb + 8 * g + 4 * hh + r;
            if (jkey >= it.n0 + rr) s = -INFINITY;
          }
          const float pe = __builtin_amdgcn_exp2f(s);
          pv[i] = pe;
          dsv[i] = pe * (pacc[qb][i] - d4[r]);
        }
      }
      pfrag[2 * qb] = pack8(pv[0], pv[1], pv[2], pv[3], pv[4], pv[5], pv[6], pv[7]);
      pfrag[2 * qb + 1] = pack8(pv[8], pv[9], pv[10], pv[11], pv[12], pv[13], pv[14], pv[15]);
      dsfrag[2 * qb] = pack8(dsv[0], dsv[1], dsv[2], dsv[3], dsv[4], dsv[5], dsv[6], dsv[7]);
      dsfrag[2 * qb + 1] = pack8(dsv[8], dsv[9], dsv[10], dsv[11], dsv[12], dsv[13], dsv[14], dsv[15]);
      // dS^T tile: row = key (32 wave + l32), columns = 4 consecutive queries per store
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const bf16x4 w = pack4(dsv[4 * g], dsv[4 * g + 1], dsv[4 * g + 2], dsv[4 * g + 3]);
        *reinterpret_cast<bf16x4*>(dSt + (32 * wave + l32) * DSP + 32 * qb + 8 * g + 4 * hh) = w;
      }
    }

    // ---- dV^T += dO^T P, dK^T += Q^T dS : [D] x [32 keys], contraction over the 64 queries ----
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const bf16x8 ag = a_tr<D>(Gb, 16 * ks, 32 * db, lane);
        const bf16x8 aq = a_tr<D>(Qb, 16 * ks, 32 * db, lane);
        dvacc[db] = mfma32(ag, pfrag[ks], dvacc[db]);
        dkacc[db] = mfma32(aq, dsfrag[ks], dkacc[db]);
      }

    __syncthreads();  // dS^T of all four waves is in LDS

    // ---- dQ += dS K : [64 queries] x [D], contraction over the 128 keys; the 2 DB output blocks of
    //      32 x 32 are dealt out to the four waves (block b: query block b % 2, column block b / 2) ----
    {
      constexpr int NB = 2 * DB / 4;
      f32x16 dq[NB];
#pragma unroll
      for (int n = 0; n < NB; ++n)
#pragma unroll
        for (int i = 0; i < 16; ++i) dq[n][i] = 0.f;
#pragma unroll
      for (int ks = 0; ks < BN / 16; ++ks) {
#pragma unroll
        for (int n = 0; n < NB; ++n) {
          const int b = wave * NB + n, qb = b & 1, db = b >> 1;
          // B operand: K[key in C-order][column 32 db + l32], gathered with transpose reads
          const bf16x8 bk = a_tr<D>(Kt, 16 * ks, 32 * db, lane);
          // A operand: dS[query 32 qb + l32][key in C-order] from the dS^T tile
          const int row = 16 * ks + 4 * hh + ((lane & 15) >> 2);
          const int col = 32 * qb + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
          s16x4 lo = lds_read_tr(dSt + row * DSP + col);
          s16x4 hi = lds_read_tr(dSt + (row + 8) * DSP + col);
          s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          dq[n] = mfma32(__builtin_bit_cast(bf16x8, v), bk, dq[n]);
        }
      }
      const int head = kvh * G + hg;
      const int rows_left = it.q_rows - qt * BM;
#pragma unroll
      for (int n = 0; n < NB; ++n) {
        const int b = wave * NB + n, qb = b & 1, db = b >> 1;
        float* dqp = p.dq_acc + ((int64_t)it.q_row0 + qt * BM) * q_stride + (int64_t)head * D + 32 * db + l32;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int r = 32 * qb + 8 * (i >> 2) + 4 * hh + (i & 3);
          if (r < rows_left) unsafeAtomicAdd(dqp + (int64_t)r * q_stride, dq[n][i]);
        }
      }
    }

    if (iter + 1 < n_iter) store_tiles(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: dK = scale * dK^T, dV = dV^T, written (or added) as bf16 ----
  {
    const int kr = 32 * wave + l32;
    if (kr < it.kv_rows) {
      const int64_t off = ((int64_t)it.kv_row0 + kr) * kv_stride + (int64_t)kvh * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int col = 32 * db + 8 * g + 4 * hh;
          float k0 = dkacc[db][4 * g] * p.scale, k1 = dkacc[db][4 * g + 1] * p.scale,
                k2 = dkacc[db][4 * g + 2] * p.scale, k3 = dkacc[db][4 * g + 3] * p.scale;
          float v0 = dvacc[db][4 * g], v1 = dvacc[db][4 * g + 1], v2 = dvacc[db][4 * g + 2], v3 = dvacc[db][4 * g + 3];
          bf16x4* dkp = reinterpret_cast<bf16x4*>(p.dk + off + col);
          bf16x4* dvp = reinterpret_cast<bf16x4*>(p.dv + off + col);
          if (p.accumulate) {
            const bf16x4 ok = *dkp, ov = *dvp;
            k0 += (float)ok[0]; k1 += (float)ok[1]; k2 += (float)ok[2]; k3 += (float)ok[3];
            v0 += (float)ov[0]; v1 += (float)ov[1]; v2 += (float)ov[2]; v3 += (float)ov[3];
          }
          *dkp = pack4(k0, k1, k2, k3);
          *dvp = pack4(v0, v1, v2, v3);
        }
    }
  }
}

template <int D>
size_t bwd_smem_bytes_t() {
  return (size_t)(tile_elems<D>(BN) + 4 * tile_elems<D>(BM) + BN * DSP) * 2 + 4 * BM * sizeof(float);
}

struct BwdLayout {
  size_t dq_off, dsum_off, items_off, total;
};
BwdLayout bwd_layout(const chunk_attn_desc* d) {
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  BwdLayout L;
  L.dq_off = 0;
  const size_t dq_bytes = (size_t)d->total_q * d->num_q_heads * d->head_dim * sizeof(float);
  L.dsum_off = up(dq_bytes);
  const size_t dsum_bytes = (size_t)d->total_q * d->num_q_heads * sizeof(float);
  L.items_off = L.dsum_off + up(dsum_bytes);
  size_t n_items = 0;
  for (int t = 0; t < d->num_segments; ++t) n_items += (d->segments[t].kv_len + BN - 1) / BN;
  L.total = L.items_off + up(n_items * sizeof(BwdItem));
  return L;
}

template <int D>
hipError_t launch_bwd_t(const chunk_attn_desc* d, const BwdArgs& a, const std::vector<BwdItem>& items,
                        hipStream_t stream) {
  const BwdLayout L = bwd_layout(d);
  float* dq_acc = reinterpret_cast<float*>(a.workspace + L.dq_off);
  float* dsum = reinterpret_cast<float*>(a.workspace + L.dsum_off);
  const int64_t n_pairs = (int64_t)d->total_q * d->num_q_heads;

  {  // D = <dO, O>, dQ accumulator = 0
    const int64_t threads = n_pairs * (D / 8);
    hipLaunchKernelGGL((bwd_pre_kernel<D>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream, a.o, a.d_o,
                       dsum, dq_acc, d->total_q, d->num_q_heads);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (!a.accumulate) {  // rows no segment covers receive no gradient
    for (const auto& gap : uncovered_kv_ranges(d)) {
      const int64_t elems = (int64_t)(gap.second - gap.first) * d->num_kv_heads * D;
      const int64_t n16 = elems / 8;
      for (__bf16* base : {a.dk, a.dv}) {
        u32x4* ptr = reinterpret_cast<u32x4*>(base + (int64_t)gap.first * d->num_kv_heads * D);
        hipLaunchKernelGGL(zero_fill_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, stream, ptr, n16);
      }
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
  }
  {
    BwdParams p;
    p.q = a.q; p.k = a.k; p.v = a.v; p.d_o = a.d_o; p.lse = a.lse; p.dsum = dsum;
    p.dq_acc = dq_acc; p.dk = a.dk; p.dv = a.dv;
    p.items = reinterpret_cast<const BwdItem*>(a.workspace + L.items_off);
    p.num_q_heads = d->num_q_heads; p.num_kv_heads = d->num_kv_heads; p.group = d->num_q_heads / d->num_kv_heads;
    p.total_q = d->total_q;
    p.scale = d->softmax_scale;
    p.scale_log2 = d->softmax_scale * 1.4426950408889634f;
    p.accumulate = a.accumulate ? 1 : 0;
    const size_t smem = bwd_smem_bytes_t<D>();
    static bool attr_set = false;
    if (!attr_set) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_main_kernel<D>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      if (e != hipSuccess) return e;
      attr_set = true;
    }
    const int64_t blocks = (int64_t)items.size() * d->num_kv_heads;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    ProfileEvents pe = profile_events();
    profile_events() = ProfileEvents{};
    hipError_t e;
    if (pe.start && (e = hipEventRecord(pe.start, stream)) != hipSuccess) return e;
    hipLaunchKernelGGL((bwd_main_kernel<D>), dim3((unsigned)blocks), dim3(256), smem, stream, p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (pe.stop && (e = hipEventRecord(pe.stop, stream)) != hipSuccess) return e;
  }
  {
    const int64_t n8 = n_pairs * (D / 8);
    hipLaunchKernelGGL((bwd_post_kernel<D>), dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, stream, dq_acc, a.dq, n8,
                       d->softmax_scale);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace

size_t bwd_workspace_bytes(const chunk_attn_desc* d) { return bwd_layout(d).total; }

void bwd_prepare(const chunk_attn_desc* d, std::vector<BwdItem>& items, size_t* items_off) {
  items = plan_bwd(d, BN);
  *items_off = bwd_layout(d).items_off;
}

hipError_t launch_bwd(const chunk_attn_desc* d, const BwdArgs& a, const std::vector<BwdItem>& items,
                      hipStream_t stream) {
  return d->head_dim == 128 ? launch_bwd_t<128>(d, a, items, stream) : launch_bwd_t<64>(d, a, items, stream);
}

}  // namespace chunk_attn
