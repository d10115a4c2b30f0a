// Chunk attention forward for gfx950: O = softmax(scale Q K^T + mask) V and LSE, where the mask is the
// chunk mask of the paper's section 3.1 (each segment's queries see their own context and the causal
// part of their own slice; packed sequences see nothing of each other).
//
// One workgroup (4 waves) takes one forward work item -- a tile of query rows of one segment -- for up
// to four query heads that share one key/value head, and streams that segment's visible keys/values
// through LDS in tiles of 64 rows: K row-major, V as the pre-transposed image (transpose_kernel.hip),
// both copied global->LDS without passing through registers and double-buffered.  Each wave owns 32
// query rows of one head and keeps their Q fragments in registers.  Scores are computed transposed,
// S^T = K Q^T, so that after the MFMA every lane holds one query column: the row maximum and row sum
// are a loop over the lane's own registers plus one exchange with the lane 32 away, and the bf16
// probabilities are already laid out as the B operand of O^T += V^T P^T (device_common.hpp, "C-order").
// Two workgroups share a compute unit, so one wave's softmax arithmetic overlaps another's MFMAs.
#include <type_traits>

#include "kernels.hpp"
#include "tiles.hpp"

namespace chunk_attn {

template <int D>
__global__ __launch_bounds__(256, 2) void fwd_kernel(FwdParams p) {
  constexpr int BN = 64;       // key rows per LDS tile
  constexpr int KC = D / 8;    // 16-byte chunks per K row
  constexpr int DK = D / 16;   // k-steps of S^T = K Q^T
  constexpr int DB = D / 32;   // 32-row blocks of O^T
  constexpr int KT = BN * D;   // elements per K tile and per V^T image

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  __bf16* Ks = reinterpret_cast<__bf16*>(smem);  // [2][BN][D]  swizzled rows
  __bf16* Vs = Ks + 2 * KT;                      // [2][D][BN]  transposed image

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, kept in a scalar register
  const int l32 = lane & 31, hh = lane >> 5;
  stagger_wave_priority();

  const int inner_n = p.num_kv_heads * p.head_splits;
  const int inner = blockIdx.x % inner_n;
  const FwdItem it = p.items[blockIdx.x / inner_n];
  const int kvh = inner % p.num_kv_heads, hs = inner / p.num_kv_heads;
  const int head = kvh * p.group + hs * p.heads_per_wg + wave % p.heads_per_wg;
  const int wave_row0 = (wave / p.heads_per_wg) * 32;  // first tile-local row of this wave

  const int n_wg = it.n0 + it.q_rows - 1;              // keys visible to the last valid row
  const int nt_wg = (n_wg + BN - 1) / BN;
  int nt_w = 0;
  if (wave_row0 < it.q_rows) {
    const int last = min(wave_row0 + 32, it.q_rows) - 1;
    nt_w = (it.n0 + last + BN - 1) / BN;
  }

  const int64_t q_stride = (int64_t)p.num_q_heads * D, kv_stride = (int64_t)p.num_kv_heads * D;
  const __bf16* __restrict__ Kg = p.k + (int64_t)it.kv_row0 * kv_stride + (int64_t)kvh * D;
  const __bf16* __restrict__ Vimg = p.vt + ((int64_t)kvh * p.total_kv_tiles + it.kv_tile0) * KT;

  // Per-lane source offsets of the global->LDS copies (elements).  A K tile is 64 rows x KC chunks; copy
  // instruction i of wave w fills LDS chunks [(4 i + w) 64, +64), so the lane fetches the chunk that the
  // swizzle puts there.  The V^T image is copied linearly.
  constexpr int NK = BN * KC / 256, NV = KT / 8 / 256;
  unsigned k_src[NK];
  int k_row[NK];
#pragma unroll
  for (int i = 0; i < NK; ++i) {
    const int x = (i * 4 + wave) * 64 + lane;
    k_row[i] = x / KC;
    k_src[i] = (unsigned)(k_row[i] * (int)kv_stride + unswz<KC>(k_row[i], x % KC) * 8);
  }
  auto dma_tile = [&](int t, int buf) {
    const __bf16* ksrc = Kg + (int64_t)(BN * t) * kv_stride;  // wave-uniform
    const int last_row = n_wg - 1 - BN * t;                   // rows past it are clamped (last tile only)
    __bf16* kdst = Ks + buf * KT;
    if (last_row >= BN - 1) {
#pragma unroll
      for (int i = 0; i < NK; ++i) dma16(ksrc + k_src[i], kdst + (i * 4 + wave) * 512);
    } else {
#pragma unroll
      for (int i = 0; i < NK; ++i) {
        const unsigned off = k_src[i] - (unsigned)((k_row[i] - min(k_row[i], last_row)) * (int)kv_stride);
        dma16(ksrc + off, kdst + (i * 4 + wave) * 512);
      }
    }
    const __bf16* vsrc = Vimg + (int64_t)t * KT;              // wave-uniform
    __bf16* vdst = Vs + buf * KT;
#pragma unroll
    for (int i = 0; i < NV; ++i) dma16(vsrc + (unsigned)(((i * 4 + wave) * 64 + lane) * 8), vdst + (i * 4 + wave) * 512);
  };

  dma_tile(0, 0);

  // Q fragments: B operand of S^T = K Q^T; lane holds Q[row = l32][16 ks + 8 hh ..+7]
  bf16x8 qf[DK];
  {
    const int r = min(wave_row0 + l32, it.q_rows - 1);  // rows past the tile repeat the last one (never stored)
    const __bf16* qp = p.q + (int64_t)(it.q_row0 + r) * q_stride + (int64_t)head * D + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
  }

  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c = p.scale_log2;

  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  // LDS operand addresses (elements).  Row l32 and row 32 + l32 share their swizzle, so the second block of
  // each tile is a constant offset away; the buffer index is a compile-time constant of the unrolled loop.
  int k_off[DK], v_off[4];
#pragma unroll
  for (int ks = 0; ks < DK; ++ks) k_off[ks] = tile_elem<KC>(l32, 2 * ks + hh);
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) v_off[ks] = tile_elem<8>(l32, 2 * ks + hh);

  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  bf16x2 ones;
  ones[0] = (__bf16)1.0f; ones[1] = (__bf16)1.0f;

  auto tile_step = [&](int t, auto buf_c) {
    constexpr int buf = decltype(buf_c)::value;
    if (t + 1 < nt_wg) dma_tile(t + 1, buf ^ 1);

    if (t < nt_w) {
      const __bf16* Kt = Ks + buf * KT;
      const __bf16* Vt = Vs + buf * KT;
      // ---- S^T = K Q^T : [64 keys] x [32 queries] ----
      f32x16 s0, s1;
#pragma unroll
      for (int ks = 0; ks < DK; ++ks) {
        const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(Kt + k_off[ks]);
        const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(Kt + k_off[ks] + 32 * D);
        s0 = mfma32(a0, qf[ks], ks == 0 ? zero16 : s0);
        s1 = mfma32(a1, qf[ks], ks == 0 ? zero16 : s1);
      }
      // ---- mask: key j of the tile (j = 64 t + local) is visible to tile row r iff j < n0 + r ----
      if (BN * t + BN > it.n0 + wave_row0) {
        const int lim = it.n0 + wave_row0 + l32 - BN * t;  // visible iff local key index < lim
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int j = 8 * (i >> 2) + 4 * hh + (i & 3);
          if (j >= lim) s0[i] = -INFINITY;
          if (j + 32 >= lim) s1[i] = -INFINITY;
        }
      }
      // ---- running max (refreshed lazily), probabilities, running sum ----
      float mx0 = fmaxf(fmaxf(s0[0], s0[1]), s0[2]), mx1 = fmaxf(fmaxf(s1[0], s1[1]), s1[2]);
#pragma unroll
      for (int i = 3; i < 15; i += 2) {
        mx0 = fmaxf(fmaxf(mx0, s0[i]), s0[i + 1]);
        mx1 = fmaxf(fmaxf(mx1, s1[i]), s1[i + 1]);
      }
      float mx = fmaxf(fmaxf(mx0, mx1), fmaxf(s0[15], s1[15]));
      mx = max_halves(mx);
      // The reference maximum only has to keep exp2 in range: it is moved when the tile maximum exceeds it
      // by more than 2^8 (first tile: from -inf), which spares the O^T rescale on almost every tile.
      if (__any((mx - m_run) * c > 8.0f)) {
        const float m_new = fmaxf(m_run, mx);
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
        m_run = m_new;
      }
      const float mc = m_run * c;
      bf16x8 pf[4];
      {
        float e[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) e[i] = __builtin_amdgcn_exp2f(s0[i] * c - mc);
        pf[0] = pack8(e[0], e[1], e[2], e[3], e[4], e[5], e[6], e[7]);
        pf[1] = pack8(e[8], e[9], e[10], e[11], e[12], e[13], e[14], e[15]);
#pragma unroll
        for (int i = 0; i < 16; ++i) e[i] = __builtin_amdgcn_exp2f(s1[i] * c - mc);
        pf[2] = pack8(e[0], e[1], e[2], e[3], e[4], e[5], e[6], e[7]);
        pf[3] = pack8(e[8], e[9], e[10], e[11], e[12], e[13], e[14], e[15]);
      }
      // row sum of the rounded probabilities (the same values the PV product uses), two per instruction
      float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        ps0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pf[j], pf[j], 0, 1), ones, ps0, false);
        ps1 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pf[j], pf[j], 2, 3), ones, ps1, false);
        ps0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pf[j], pf[j], 4, 5), ones, ps0, false);
        ps1 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pf[j], pf[j], 6, 7), ones, ps1, false);
      }
      l_run += ps0 + ps1;
      // ---- O^T += V^T P^T : [D] x [32 queries], contraction over the 64 keys ----
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(Vt + v_off[ks] + db * 32 * 64);
          oacc[db] = mfma32(a, pf[ks], oacc[db]);
        }
      }
    }

    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  };

  for (int t = 0; t < nt_wg; t += 2) {
    tile_step(t, std::integral_constant<int, 0>{});
    if (t + 1 < nt_wg) tile_step(t + 1, std::integral_constant<int, 1>{});
  }

  // ---- epilogue: O = O^T / l, LSE = ln(l) + m scale ----
  {
    const int r = wave_row0 + l32;
    const float l_tot = sum_halves(l_run);
    if (r < it.q_rows) {
      const float inv = 1.0f / l_tot;
      __bf16* op = p.o + (int64_t)(it.q_row0 + r) * q_stride + (int64_t)head * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const bf16x4 v = pack4(oacc[db][4 * g] * inv, oacc[db][4 * g + 1] * inv, oacc[db][4 * g + 2] * inv,
                                 oacc[db][4 * g + 3] * inv);
          *reinterpret_cast<bf16x4*>(op + 32 * db + 8 * g + 4 * hh) = v;
        }
      if (hh == 0)
        p.lse[(int64_t)head * p.total_q + it.q_row0 + r] = (m_run * c + log2f(l_tot)) * 0.6931471805599453f;
    }
  }
}

template <int D>
static hipError_t launch_fwd_t(const FwdParams& p, int num_blocks, hipStream_t stream) {
  const size_t smem = (size_t)4 * 64 * D * 2;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&fwd_kernel<D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((fwd_kernel<D>), dim3(num_blocks), dim3(256), smem, stream, p);
  return hipGetLastError();
}

hipError_t launch_fwd(const FwdParams& p, int head_dim, int num_blocks, hipStream_t stream) {
  return head_dim == 128 ? launch_fwd_t<128>(p, num_blocks, stream) : launch_fwd_t<64>(p, num_blocks, stream);
}

}  // namespace chunk_attn
