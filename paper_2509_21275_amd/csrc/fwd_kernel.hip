// Chunk attention forward for gfx950: O = softmax(scale Q K^T + mask) V and LSE, where the mask is the
// chunk mask of the paper's section 3.1 (each segment's queries see their own context and the causal
// part of their own slice; packed sequences see nothing of each other).
//
// One workgroup (4 waves) takes one forward work item -- a tile of query rows of one segment -- for up
// to four query heads that share one key/value head, and streams that segment's visible K/V rows
// through LDS in tiles of 64 rows.  Each wave owns NQ blocks of 32 query rows of one head and keeps
// their Q fragments in registers.  Scores are computed transposed, S^T = K Q^T, so that after the
// MFMA every lane holds one query column: the row maximum and row sum are a loop over the lane's own
// registers plus one exchange with the lane 32 away, and the bf16 probabilities are already laid out
// as the B operand of O^T += V^T P^T (device_common.hpp, "C-order").
#include "kernels.hpp"

namespace chunk_attn {

template <int D, int NQ>
__global__ __launch_bounds__(256, NQ == 1 ? 2 : 1) void fwd_kernel(FwdParams p) {
  constexpr int BN = 64;            // key rows per LDS tile
  constexpr int KS = D + 8;         // K tile pitch (elements): 16-byte row skew for ds_read_b128
  constexpr int VS = D + 32;        // V tile pitch: 64-byte row skew for the transpose reads
  constexpr int DK = D / 16;        // k-steps of S^T = K Q^T
  constexpr int DB = D / 32;        // 32-row blocks of O^T
  constexpr int CH = BN * D / 8 / 256;  // 16-byte chunks per thread per tile

  extern __shared__ __attribute__((aligned(16))) char smem[];
  __bf16* Ks = reinterpret_cast<__bf16*>(smem);                 // [2][BN][KS]
  __bf16* Vs = Ks + 2 * BN * KS;                                // [2][BN][VS]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hh = lane >> 5;

  const int inner_n = p.num_kv_heads * p.head_splits;
  const int inner = blockIdx.x % inner_n;
  const FwdItem it = p.items[blockIdx.x / inner_n];
  const int kvh = inner % p.num_kv_heads, hs = inner / p.num_kv_heads;
  const int head = kvh * p.group + hs * p.heads_per_wg + wave % p.heads_per_wg;
  const int wave_row0 = (wave / p.heads_per_wg) * (32 * NQ);  // first tile-local row of this wave

  const int n_wg = it.n0 + it.q_rows - 1;                     // keys visible to the last valid row
  const int nt_wg = (n_wg + BN - 1) / BN;
  int nt_w = 0;
  if (wave_row0 < it.q_rows) {
    const int last = min(wave_row0 + 32 * NQ, it.q_rows) - 1;
    nt_w = (it.n0 + last + BN - 1) / BN;
  }

  const int64_t q_stride = (int64_t)p.num_q_heads * D, kv_stride = (int64_t)p.num_kv_heads * D;
  const __bf16* __restrict__ Kg = p.k + (int64_t)it.kv_row0 * kv_stride + (int64_t)kvh * D;
  const __bf16* __restrict__ Vg = p.v + (int64_t)it.kv_row0 * kv_stride + (int64_t)kvh * D;

  // Q fragments: B operand of S^T = K Q^T; lane holds Q[row = l32][16 ks + 8 hh ..+7]
  bf16x8 qf[NQ][DK];
#pragma unroll
  for (int qb = 0; qb < NQ; ++qb) {
    const int r = min(wave_row0 + 32 * qb + l32, it.q_rows - 1);  // clamp: rows past the tile repeat the last one
    const __bf16* qp = p.q + (int64_t)(it.q_row0 + r) * q_stride + (int64_t)head * D + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) qf[qb][ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
  }

  f32x16 oacc[DB][NQ];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[db][qb][i] = 0.f;
  float m_run[NQ], l_run[NQ];
#pragma unroll
  for (int qb = 0; qb < NQ; ++qb) { m_run[qb] = -INFINITY; l_run[qb] = 0.f; }

  const float c = p.scale_log2;

  // ---- K/V tile staging: global -> registers -> LDS ----
  u32x4 kreg[CH], vreg[CH];
  auto load_tile = [&](int t) {
#pragma unroll
    for (int ci = 0; ci < CH; ++ci) {
      const int idx = tid + 256 * ci;
      const int row = idx / (D / 8), col = (idx % (D / 8)) * 8;
      const int64_t grow = min(BN * t + row, n_wg - 1);  // clamp inside the visible range
      kreg[ci] = *reinterpret_cast<const u32x4*>(Kg + grow * kv_stride + col);
      vreg[ci] = *reinterpret_cast<const u32x4*>(Vg + grow * kv_stride + col);
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int ci = 0; ci < CH; ++ci) {
      const int idx = tid + 256 * ci;
      const int row = idx / (D / 8), col = (idx % (D / 8)) * 8;
      *reinterpret_cast<u32x4*>(Ks + (buf * BN + row) * KS + col) = kreg[ci];
      *reinterpret_cast<u32x4*>(Vs + (buf * BN + row) * VS + col) = vreg[ci];
    }
  };

  load_tile(0);
  store_tile(0);
  __syncthreads();

  for (int t = 0; t < nt_wg; ++t) {
    const int buf = t & 1;
    if (t + 1 < nt_wg) load_tile(t + 1);

    if (t < nt_w) {
      const __bf16* Kt = Ks + buf * BN * KS;
      const __bf16* Vt = Vs + buf * BN * VS;
      // ---- S^T = K Q^T : [64 keys] x [32 NQ queries] ----
      f32x16 sacc[2][NQ];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int qb = 0; qb < NQ; ++qb)
#pragma unroll
          for (int i = 0; i < 16; ++i) sacc[kb][qb][i] = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int ks = 0; ks < DK; ++ks) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(Kt + (32 * kb + l32) * KS + 16 * ks + 8 * hh);
#pragma unroll
          for (int qb = 0; qb < NQ; ++qb) sacc[kb][qb] = mfma32(a, qf[qb][ks], sacc[kb][qb]);
        }
      }
      // ---- mask, running max / sum, probabilities ----
      bf16x8 pf[NQ][4];
#pragma unroll
      for (int qb = 0; qb < NQ; ++qb) {
        const int row_min = wave_row0 + 32 * qb;
        // key j (tile-local index 64 t + ...) is visible to tile row r iff j < n0 + r
        if (BN * t + BN > it.n0 + row_min) {
          const int lim = it.n0 + row_min + l32 - BN * t;  // visible iff local key index < lim
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int j = 32 * kb + 8 * (i >> 2) + 4 * hh + (i & 3);
              if (j >= lim) sacc[kb][qb][i] = -INFINITY;
            }
        }
        float mx = sacc[0][qb][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[kb][qb][i]);
        mx = max_halves(mx);
        const float m_new = fmaxf(m_run[qb], mx);
        if (__any(m_new != m_run[qb])) {
          const float alpha = __builtin_amdgcn_exp2f((m_run[qb] - m_new) * c);
          l_run[qb] *= alpha;
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[db][qb][i] *= alpha;
          m_run[qb] = m_new;
        }
        const float mc = m_new * c;
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          float e[16];
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            e[i] = __builtin_amdgcn_exp2f(sacc[kb][qb][i] * c - mc);
            psum += e[i];
          }
          pf[qb][2 * kb] = pack8(e[0], e[1], e[2], e[3], e[4], e[5], e[6], e[7]);
          pf[qb][2 * kb + 1] = pack8(e[8], e[9], e[10], e[11], e[12], e[13], e[14], e[15]);
        }
        l_run[qb] += psum;
      }
      // ---- O^T += V^T P^T : [D] x [32 NQ queries], contraction over the 64 keys ----
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const bf16x8 a = lds_a_operand_transposed(Vt, VS, 16 * ks, 32 * db, lane);
#pragma unroll
          for (int qb = 0; qb < NQ; ++qb) oacc[db][qb] = mfma32(a, pf[qb][ks], oacc[db][qb]);
        }
      }
    }

    if (t + 1 < nt_wg) store_tile(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: O = O^T / l, LSE = ln(l) + m scale ----
#pragma unroll
  for (int qb = 0; qb < NQ; ++qb) {
    const int r = wave_row0 + 32 * qb + l32;
    const float l_tot = sum_halves(l_run[qb]);
    if (r < it.q_rows) {
      const float inv = 1.0f / l_tot;
      __bf16* op = p.o + (int64_t)(it.q_row0 + r) * q_stride + (int64_t)head * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const bf16x4 v = pack4(oacc[db][qb][4 * g] * inv, oacc[db][qb][4 * g + 1] * inv,
                                 oacc[db][qb][4 * g + 2] * inv, oacc[db][qb][4 * g + 3] * inv);
          *reinterpret_cast<bf16x4*>(op + 32 * db + 8 * g + 4 * hh) = v;
        }
      if (hh == 0)
        p.lse[(int64_t)head * p.total_q + it.q_row0 + r] = (m_run[qb] * c + log2f(l_tot)) * 0.6931471805599453f;
    }
  }
}

size_t fwd_smem_bytes(int head_dim) { return (size_t)2 * 64 * ((head_dim + 8) + (head_dim + 32)) * 2; }

template <int D, int NQ>
static hipError_t launch_fwd_t(const FwdParams& p, int num_blocks, hipStream_t stream) {
  const size_t smem = fwd_smem_bytes(D);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&fwd_kernel<D, NQ>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((fwd_kernel<D, NQ>), dim3(num_blocks), dim3(256), smem, stream, p);
  return hipGetLastError();
}

hipError_t launch_fwd(const FwdParams& p, int head_dim, int nq, int num_blocks, hipStream_t stream) {
  if (head_dim == 128) return nq == 2 ? launch_fwd_t<128, 2>(p, num_blocks, stream) : launch_fwd_t<128, 1>(p, num_blocks, stream);
  return nq == 2 ? launch_fwd_t<64, 2>(p, num_blocks, stream) : launch_fwd_t<64, 1>(p, num_blocks, stream);
}

}  // namespace chunk_attn
