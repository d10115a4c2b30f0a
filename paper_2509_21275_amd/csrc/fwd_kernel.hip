// Chunk attention forward for gfx950: O = softmax(scale Q K^T + mask) V and LSE, where the mask is the
// chunk mask of the paper's section 3.1 (each segment's queries see their own context and the causal
// part of their own slice; packed sequences see nothing of each other).
//
// A workgroup takes one forward work item -- a tile of query rows of one segment -- for the query heads of
// one group that share a key/value head, and streams that segment's visible keys/values through LDS in
// tiles of 64 rows: K row-major, V as the pre-transposed image (transpose_kernel.hip), both copied
// global->LDS without passing through registers and double-buffered.  Scores are computed transposed,
// S^T = K Q^T, so that after the MFMA every lane holds one query column: row maximum and row sum are a loop
// over the lane's own registers plus one exchange with the lane 32 away, and the bf16 probabilities are
// already laid out as the B operand of O^T += V^T P^T (device_common.hpp, "C-order").
//
// Two kernels:
//   fwd_kernel       online softmax with a lazily moved reference maximum, one 32-row query block per wave,
//                    two waves per SIMD.  Used for head_dim 64, and for head_dim 128 as the second pass below.
//   fwd_pipe_kernel  head_dim 128: one wave per SIMD with 64 query rows, software pipelined over the key
//                    tiles, reference maximum fixed by the first tile; rows whose scores outgrow it are
//                    flagged and recomputed by fwd_kernel, launched right after over the flagged items only.
#include <type_traits>

#include "kernels.hpp"
#include "tiles.hpp"

namespace chunk_attn {

template <int D, int WAVES>
__global__ __launch_bounds__(WAVES * 64, 8 / WAVES) void fwd_kernel(FwdParams p) {
  constexpr int QB = 1;        // 32-row query blocks per wave
  constexpr int NT = WAVES * 64;  // threads
  constexpr int BN = 64;       // key rows per LDS tile
  constexpr int KC = D / 8;    // 16-byte chunks per K row
  constexpr int DK = D / 16;   // k-steps of S^T = K Q^T
  constexpr int DB = D / 32;   // 32-row blocks of O^T
  constexpr int KT = BN * D;   // elements per K tile and per V^T image
  constexpr int WR = 32 * QB;  // query rows per wave
  if (p.redo && p.redo[blockIdx.x] == 0) return;  // second pass: only the items the pipelined kernel gave up on

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
  const int wave_row0 = (wave / p.heads_per_wg) * WR;  // first tile-local row of this wave

  const int n_wg = it.n0 + it.q_rows - 1;              // keys visible to the last valid row
  const int nt_wg = (n_wg + BN - 1) / BN;
  int nt_w = 0;
  if (wave_row0 < it.q_rows) {
    const int last = min(wave_row0 + WR, it.q_rows) - 1;
    nt_w = (it.n0 + last + BN - 1) / BN;
  }

  const int64_t q_stride = (int64_t)p.num_q_heads * D, kv_stride = (int64_t)p.num_kv_heads * D;
  const __bf16* __restrict__ Kg = p.k + (int64_t)it.kv_row0 * kv_stride + (int64_t)kvh * D;
  const __bf16* __restrict__ Vimg = p.vt + ((int64_t)kvh * p.total_kv_tiles + it.kv_tile0) * KT;

  // Per-lane source offsets of the global->LDS copies (elements).  A K tile is 64 rows x KC chunks; copy
  // instruction i of wave w fills LDS chunks [(WAVES i + w) 64, +64), so the lane fetches the chunk that the
  // swizzle puts there.  The V^T image is copied linearly.
  constexpr int NK = BN * KC / NT, NV = KT / 8 / NT;
  static_assert(NK >= 1 && NV >= 1, "every thread copies at least one chunk of each tile");
  unsigned k_src[NK];
  int k_row[NK];
#pragma unroll
  for (int i = 0; i < NK; ++i) {
    const int x = (i * WAVES + wave) * 64 + lane;
    k_row[i] = x / KC;
    k_src[i] = (unsigned)(k_row[i] * (int)kv_stride + unswz<KC>(k_row[i], x % KC) * 8);
  }
  auto dma_tile = [&](int t, int buf) {
    const __bf16* ksrc = Kg + (int64_t)(BN * t) * kv_stride;  // wave-uniform
    const int last_row = n_wg - 1 - BN * t;                   // rows past it are clamped (last tile only)
    __bf16* kdst = Ks + buf * KT;
    if (last_row >= BN - 1) {
#pragma unroll
      for (int i = 0; i < NK; ++i) dma16(ksrc + k_src[i], kdst + (i * WAVES + wave) * 512);
    } else {
#pragma unroll
      for (int i = 0; i < NK; ++i) {
        const unsigned off = k_src[i] - (unsigned)((k_row[i] - min(k_row[i], last_row)) * (int)kv_stride);
        dma16(ksrc + off, kdst + (i * WAVES + wave) * 512);
      }
    }
    const __bf16* vsrc = Vimg + (int64_t)t * KT;              // wave-uniform
    __bf16* vdst = Vs + buf * KT;
#pragma unroll
    for (int i = 0; i < NV; ++i)
      dma16(vsrc + (unsigned)(((i * WAVES + wave) * 64 + lane) * 8), vdst + (i * WAVES + wave) * 512);
  };

  dma_tile(0, 0);

  // Q fragments: B operand of S^T = K Q^T; lane holds Q[row = 32 qb + l32][16 ks + 8 hh ..+7]
  bf16x8 qf[QB][DK];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int r = min(wave_row0 + 32 * qb + l32, it.q_rows - 1);  // rows past the tile repeat the last one (never stored)
    const __bf16* qp = p.q + (int64_t)(it.q_row0 + r) * q_stride + (int64_t)head * D + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) qf[qb][ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
  }

  f32x16 oacc[QB][DB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[qb][db][i] = 0.f;
  float m_run[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) { m_run[qb] = -INFINITY; l_run[qb] = 0.f; }
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

  // One loop body for both LDS buffers: the operand addresses are toggled between the buffers with an XOR
  // (the buffers are KT elements = a power of two bytes apart), so the accumulators are carried by a single
  // loop and never pass through a conditional.
  static_assert((KT & (KT - 1)) == 0, "buffer pitch must be a power of two");
  int buf = 0;
  for (int t = 0; t < nt_wg; ++t) {
    if (t + 1 < nt_wg) dma_tile(t + 1, buf ^ 1);

    if (t < nt_w) {
      const __bf16* Kt = Ks;
      const __bf16* Vt = Vs;
      // ---- S^T = K Q^T : [64 keys] x [32 QB queries]; every K fragment feeds QB products ----
      f32x16 s0[QB], s1[QB];
#pragma unroll
      for (int ks = 0; ks < DK; ++ks) {
        const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(Kt + k_off[ks]);
        const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(Kt + k_off[ks] + 32 * D);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          s0[qb] = mfma32(a0, qf[qb][ks], ks == 0 ? zero16 : s0[qb]);
          s1[qb] = mfma32(a1, qf[qb][ks], ks == 0 ? zero16 : s1[qb]);
        }
      }
      bf16x8 pf[QB][4];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        // ---- mask: key j of the tile (j = 64 t + local) is visible to tile row r iff j < n0 + r ----
        if (BN * t + BN > it.n0 + wave_row0 + 32 * qb) {
          const int lim = it.n0 + wave_row0 + 32 * qb + l32 - BN * t;  // visible iff local key index < lim
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int j = 8 * (i >> 2) + 4 * hh + (i & 3);
            if (j >= lim) s0[qb][i] = -INFINITY;
            if (j + 32 >= lim) s1[qb][i] = -INFINITY;
          }
        }
        // ---- running max (refreshed lazily), probabilities, running sum ----
        float mx0 = fmaxf(fmaxf(s0[qb][0], s0[qb][1]), s0[qb][2]), mx1 = fmaxf(fmaxf(s1[qb][0], s1[qb][1]), s1[qb][2]);
#pragma unroll
        for (int i = 3; i < 15; i += 2) {
          mx0 = fmaxf(fmaxf(mx0, s0[qb][i]), s0[qb][i + 1]);
          mx1 = fmaxf(fmaxf(mx1, s1[qb][i]), s1[qb][i + 1]);
        }
        float mx = fmaxf(fmaxf(mx0, mx1), fmaxf(s0[qb][15], s1[qb][15]));
        mx = max_halves(mx);
        // The reference maximum only has to keep exp2 in range: it is moved when the tile maximum exceeds it
        // by more than 2^8 (first tile: from -inf), which spares the O^T rescale on almost every tile.
        if (__builtin_expect(__any((mx - m_run[qb]) * c > 8.0f), 0)) {
          const float m_new = fmaxf(m_run[qb], mx);
          const float alpha = __builtin_amdgcn_exp2f((m_run[qb] - m_new) * c);
          l_run[qb] *= alpha;
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[qb][db][i] *= alpha;
          m_run[qb] = m_new;
        }
        const float mc = m_run[qb] * c;
        {
          float e[16];
#pragma unroll
          for (int i = 0; i < 16; ++i) e[i] = __builtin_amdgcn_exp2f(s0[qb][i] * c - mc);
          pf[qb][0] = pack8(e[0], e[1], e[2], e[3], e[4], e[5], e[6], e[7]);
          pf[qb][1] = pack8(e[8], e[9], e[10], e[11], e[12], e[13], e[14], e[15]);
#pragma unroll
          for (int i = 0; i < 16; ++i) e[i] = __builtin_amdgcn_exp2f(s1[qb][i] * c - mc);
          pf[qb][2] = pack8(e[0], e[1], e[2], e[3], e[4], e[5], e[6], e[7]);
          pf[qb][3] = pack8(e[8], e[9], e[10], e[11], e[12], e[13], e[14], e[15]);
        }
        // row sum of the rounded probabilities (the same values the PV product uses), two per instruction
        float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          ps0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pf[qb][j], pf[qb][j], 0, 1), ones, ps0, false);
          ps1 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pf[qb][j], pf[qb][j], 2, 3), ones, ps1, false);
          ps0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pf[qb][j], pf[qb][j], 4, 5), ones, ps0, false);
          ps1 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pf[qb][j], pf[qb][j], 6, 7), ones, ps1, false);
        }
        l_run[qb] += ps0 + ps1;
      }
      // ---- O^T += V^T P^T : [D] x [32 QB queries], contraction over the 64 keys; every V^T fragment feeds QB products ----
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(Vt + v_off[ks] + db * 32 * 64);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) oacc[qb][db] = mfma32(a, pf[qb][ks], oacc[qb][db]);
        }
      }
    }

    buf ^= 1;
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) k_off[ks] ^= KT;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) v_off[ks] ^= KT;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  }

  // ---- epilogue: O = O^T / l, LSE = ln(l) + m scale ----
  auto oval = [&](int qb, int db, int i) { return oacc[qb][db][i]; };
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int r = wave_row0 + 32 * qb + l32;
    const float l_tot = sum_halves(l_run[qb]);
    if (r < it.q_rows) {
      const float inv = 1.0f / l_tot;
      __bf16* op = p.o + (int64_t)(it.q_row0 + r) * q_stride + (int64_t)head * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const bf16x4 v = pack4(oval(qb, db, 4 * g) * inv, oval(qb, db, 4 * g + 1) * inv, oval(qb, db, 4 * g + 2) * inv,
                                 oval(qb, db, 4 * g + 3) * inv);
          *reinterpret_cast<bf16x4*>(op + 32 * db + 8 * g + 4 * hh) = v;
        }
      if (hh == 0)
        p.lse[(int64_t)head * p.total_q + it.q_row0 + r] = (m_run[qb] * c + log2f(l_tot)) * 0.6931471805599453f;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Pipelined forward for head_dim 128: one wave per SIMD, 64 query rows per wave.
//
// Every K and V^T fragment read from LDS feeds two MFMAs (the wave's two 32-row query blocks), which halves
// the LDS traffic per MFMA.  That needs more than 256 registers per lane, so only one wave fits a SIMD and
// the overlap of matrix and vector work has to come from inside the wave: the loop is software pipelined.
// Iteration t runs   O^T += V^T(t-1) P^T(t-1)   next to the mask / row maximum of S^T(t), and
//                    S^T(t+1) = K(t+1) Q^T      next to the exponentials / row sums of S^T(t),
// matrix and vector instructions of each pair being independent.  The accumulators stay in accumulation
// registers for the whole loop (the rare rescale and the epilogue read them through opaque single-register
// moves, see device_common.hpp); the loop has one body for both LDS buffers (addresses toggled by XOR).
// ------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256, 1) void fwd_pipe_kernel(FwdParams p) {
  constexpr int WAVES = 4, QB = 2;
  constexpr int NT = WAVES * 64;
  constexpr int BN = 64;       // key rows per LDS tile
  constexpr int KC = D / 8;    // 16-byte chunks per K row
  constexpr int DK = D / 16;   // k-steps of S^T = K Q^T
  constexpr int DB = D / 32;   // 32-row blocks of O^T
  constexpr int KT = BN * D;   // elements per K tile and per V^T image
  constexpr int WR = 32 * QB;  // query rows per wave
  static_assert((KT & (KT - 1)) == 0, "buffer pitch must be a power of two");

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  __bf16* Ks = reinterpret_cast<__bf16*>(smem);  // [2][BN][D]  swizzled rows
  __bf16* Vs = Ks + 2 * KT;                      // [2][D][BN]  transposed image

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hh = lane >> 5;

  const int inner_n = p.num_kv_heads * p.head_splits;
  const int inner = blockIdx.x % inner_n;
  const FwdItem it = p.items[blockIdx.x / inner_n];
  const int kvh = inner % p.num_kv_heads, hs = inner / p.num_kv_heads;
  const int head = kvh * p.group + hs * p.heads_per_wg + wave % p.heads_per_wg;
  const int wave_row0 = (wave / p.heads_per_wg) * WR;

  const int n_wg = it.n0 + it.q_rows - 1;  // keys visible to the last valid row
  const int nt = (n_wg + BN - 1) / BN;     // every wave runs all tiles of the workgroup (masked ones give P = 0)

  const int64_t q_stride = (int64_t)p.num_q_heads * D, kv_stride = (int64_t)p.num_kv_heads * D;
  const __bf16* __restrict__ Kg = p.k + (int64_t)it.kv_row0 * kv_stride + (int64_t)kvh * D;
  const __bf16* __restrict__ Vimg = p.vt + ((int64_t)kvh * p.total_kv_tiles + it.kv_tile0) * KT;

  constexpr int NK = BN * KC / NT, NV = KT / 8 / NT;
  int k_chunk[NK], k_row[NK];  // element offset of the lane's chunk inside its row, and the row
#pragma unroll
  for (int i = 0; i < NK; ++i) {
    const int x = (i * WAVES + wave) * 64 + lane;
    k_row[i] = x / KC;
    k_chunk[i] = unswz<KC>(k_row[i], x % KC) * 8;
  }
  // branch-free (the loop body must stay one basic block): rows past the last key repeat it
  auto dma_k = [&](int t, int buf) {
    const __bf16* ksrc = Kg + (int64_t)(BN * t) * kv_stride;  // wave-uniform
    const int last_row = n_wg - 1 - BN * t;
    __bf16* kdst = Ks + buf * KT;
#pragma unroll
    for (int i = 0; i < NK; ++i)
      dma16(ksrc + (unsigned)(min(k_row[i], last_row) * (int)kv_stride + k_chunk[i]), kdst + (i * WAVES + wave) * 512);
  };
  auto dma_v = [&](int t, int buf) {
    const __bf16* vsrc = Vimg + (int64_t)t * KT;  // wave-uniform
    __bf16* vdst = Vs + buf * KT;
#pragma unroll
    for (int i = 0; i < NV; ++i)
      dma16(vsrc + (unsigned)(((i * WAVES + wave) * 64 + lane) * 8), vdst + (i * WAVES + wave) * 512);
  };

  dma_k(0, 0);
  if (nt > 1) dma_k(1, 1);
  // the first iteration multiplies P = 0 with "V^T(-1)": give it zeros rather than whatever LDS holds
  {
    bf16x8 z;
#pragma unroll
    for (int i = 0; i < 8; ++i) z[i] = (__bf16)0.0f;
#pragma unroll
    for (int i = 0; i < KT / 8 / NT; ++i) *reinterpret_cast<bf16x8*>(Vs + KT + (i * NT + tid) * 8) = z;
  }

  // Q fragments: B operand of S^T = K Q^T; lane holds Q[row = 32 qb + l32][16 ks + 8 hh ..+7]
  bf16x8 qf[QB][DK];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int r = min(wave_row0 + 32 * qb + l32, it.q_rows - 1);  // rows past the tile repeat the last one (never stored)
    const __bf16* qp = p.q + (int64_t)(it.q_row0 + r) * q_stride + (int64_t)head * D + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) qf[qb][ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
  }

  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 oacc[QB][DB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int db = 0; db < DB; ++db) oacc[qb][db] = zero16;
  float m_run[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) { m_run[qb] = 0.f; l_run[qb] = 0.f; }
  bool risk = false;
  const float c = p.scale_log2;

  // LDS operand addresses (elements); k_off addresses the K buffer of tile t + 1, v_off the V^T buffer of tile t - 1
  int k_off[DK], v_off[4];
#pragma unroll
  for (int ks = 0; ks < DK; ++ks) k_off[ks] = tile_elem<KC>(l32, 2 * ks + hh);
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) v_off[ks] = tile_elem<8>(l32, 2 * ks + hh) + KT;

  bf16x2 ones;
  ones[0] = (__bf16)1.0f; ones[1] = (__bf16)1.0f;

  // S^T = K Q^T of one tile: [64 keys] x [64 queries], dst[qb][kb].  Two score tiles live in the accumulation
  // registers: the one being computed (next tile) and the one whose exponentials are being taken.
  f32x16 s[2][QB][2];
  auto qk = [&](f32x16 (&dst)[QB][2]) {
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) {
      const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(Ks + k_off[ks]);
      const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(Ks + k_off[ks] + 32 * D);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        dst[qb][0] = mfma32(a0, qf[qb][ks], ks == 0 ? zero16 : dst[qb][0]);
        dst[qb][1] = mfma32(a1, qf[qb][ks], ks == 0 ? zero16 : dst[qb][1]);
      }
    }
  };
  bf16x8 pf[QB][4];  // P^T of the previous tile (B operands)
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int i = 0; i < 8; ++i) pf[qb][j][i] = (__bf16)0.0f;
  auto pv = [&]() {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(Vs + v_off[ks] + db * 32 * 64);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) oacc[qb][db] = mfma32(a, pf[qb][ks], oacc[qb][db]);
      }
  };

  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  qk(s[0]);  // S^T(0)
#pragma unroll
  for (int ks = 0; ks < DK; ++ks) k_off[ks] ^= KT;
  // The reference maximum only has to keep exp2 in range, so it is fixed by the first tile and never moved:
  // O^T is never rescaled and stays in the accumulation registers.  Should a later tile's probabilities
  // exceed 2^ref_limit, the workgroup raises its redo flag and the item is recomputed by the rescaling
  // kernel (fwd_kernel) launched right after this one.
  mfma_settle();
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int lim = it.n0 + wave_row0 + 32 * qb + l32;  // tile 0: visible iff local key index < lim (>= 1)
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int j = 8 * (i >> 2) + 4 * hh + (i & 3);
      const float a0 = read_acc_elem(s[0][qb][0], i), a1 = read_acc_elem(s[0][qb][1], i);
      if (j < lim) mx = fmaxf(mx, a0);
      if (j + 32 < lim) mx = fmaxf(mx, a1);
    }
    m_run[qb] = max_halves(mx);
  }
  const float big = __builtin_amdgcn_exp2f(p.ref_limit);
  __syncthreads();  // every wave has read K(0): its buffer may be refilled

  // One tile: O^T += V^T(t-1) P^T(t-1) and S^T(t+1) = K(t+1) Q^T (matrix pipe) next to P^T(t) = exp2(S^T(t) c - m c)
  // and its row sums (vector pipe).  cur holds S^T(t), nxt receives S^T(t+1).  The tile is cut into 32 steps
  // of one LDS operand fragment, the two MFMAs it feeds and the exponentials of two scores; every step also
  // issues the fragment read of the step four ahead (with one wave per SIMD nothing else would cover the LDS
  // latency).  Scheduling fences keep the steps apart, so that vector work is spread evenly under the MFMAs.
  auto tile = [&](int t, f32x16 (&cur)[QB][2], f32x16 (&nxt)[QB][2], auto masked_c) {
    constexpr bool MASKED = decltype(masked_c)::value;
    constexpr int AHEAD = 4;
    dma_k(min(t + 2, nt - 1), t & 1);  // past the end: the last tile again, into a buffer nobody reads
    dma_v(min(t, nt - 1), t & 1);
    bf16x8 fr[8];  // ring of operand fragments
    auto load_frag = [&](int m) {
      if (m < 16) return *reinterpret_cast<const bf16x8*>(Vs + v_off[m >> 2] + (m & 3) * 32 * 64);  // V^T(t-1): k-step, block
      const int mm = m - 16;                                                                          // K(t+1): k-step, key half
      return *reinterpret_cast<const bf16x8*>(Ks + k_off[mm >> 1] + (mm & 1) * 32 * D);
    };
    unsigned pw[QB][16];  // P^T(t) as packed pairs
    float ps[QB][2];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) ps[qb][0] = ps[qb][1] = 0.f;
#pragma unroll
    for (int m = 0; m < AHEAD; ++m) fr[m] = load_frag(m);
    // the last MFMA that wrote `cur` is far behind (end of the previous tile, a barrier and the copy set-up lie
    // between); the nop makes the required distance to the opaque reads explicit
    asm volatile("s_nop 15" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int m = 0; m < 32; ++m) {
      if (m + AHEAD < 32) fr[(m + AHEAD) & 7] = load_frag(m + AHEAD);
      const bf16x8 f = fr[m & 7];
      if (m < 16) {
        const int ks = m >> 2, db = m & 3;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) oacc[qb][db] = mfma32(f, pf[qb][ks], oacc[qb][db]);
      } else {
        const int ks = (m - 16) >> 1, kb = (m - 16) & 1;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) nxt[qb][kb] = mfma32(f, qf[qb][ks], ks == 0 ? zero16 : nxt[qb][kb]);
      }
      {  // scores 2 dw, 2 dw + 1 of block (qb, kb): exponentials, packed pair, row sum
        const int qb = m >> 4, kb = (m >> 3) & 1, dw = m & 7;
        const float mc = m_run[qb] * c;
        const int lim = it.n0 + wave_row0 + 32 * qb + l32 - BN * t;  // visible iff local key index < lim
        // opaque (ordered) reads of the scores, and the result pinned before the step's fence: otherwise the
        // compiler gathers the vector work of the whole tile in one place
        float e0 = __builtin_amdgcn_exp2f(read_acc_elem(cur[qb][kb], 2 * dw) * c - mc);
        float e1 = __builtin_amdgcn_exp2f(read_acc_elem(cur[qb][kb], 2 * dw + 1) * c - mc);
        if (MASKED) {
          const int j = 32 * kb + 8 * (dw >> 1) + 4 * hh + 2 * (dw & 1);
          if (j >= lim) e0 = 0.f;
          if (j + 1 >= lim) e1 = 0.f;
        }
        bf16x2 w;
        w[0] = (__bf16)e0; w[1] = (__bf16)e1;
        ps[qb][dw & 1] = __builtin_amdgcn_fdot2_f32_bf16(w, ones, ps[qb][dw & 1], false);
        unsigned wu = __builtin_bit_cast(unsigned, w);
        asm volatile("" : "+v"(wu));
        pw[qb][8 * kb + dw] = wu;
      }
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const float sum = ps[qb][0] + ps[qb][1];
      risk |= !(sum < big);
      l_run[qb] += sum;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        u32x4 v = {pw[qb][4 * j], pw[qb][4 * j + 1], pw[qb][4 * j + 2], pw[qb][4 * j + 3]};
        pf[qb][j] = __builtin_bit_cast(bf16x8, v);
      }
    }
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) k_off[ks] ^= KT;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) v_off[ks] ^= KT;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  };
  // Tiles are taken two at a time (the two score tiles swap roles without a copy), first the pairs every row
  // of the wave sees completely, then the ones that need the mask; a pair may run one tile past the end,
  // which the mask turns into P = 0.  The accumulators never pass through a conditional.
  const int t_full = min(nt, (it.n0 + wave_row0) / BN) & ~1;  // tiles [0, t_full) are complete for every row
  for (int t = 0; t < t_full; t += 2) {
    tile(t, s[0], s[1], std::false_type{});
    tile(t + 1, s[1], s[0], std::false_type{});
  }
  for (int t = t_full; t < nt; t += 2) {
    tile(t, s[0], s[1], std::true_type{});
    tile(t + 1, s[1], s[0], std::true_type{});
  }
  pv();  // O^T += V^T P^T of the last tile
  if (__any(risk) && lane == 0) p.redo[blockIdx.x] = 1;

  // ---- epilogue: O = O^T / l, LSE = ln(l) + m scale ----
  mfma_settle();
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int r = wave_row0 + 32 * qb + l32;
    const float l_tot = sum_halves(l_run[qb]);
    if (r < it.q_rows) {
      const float inv = 1.0f / l_tot;
      __bf16* op = p.o + (int64_t)(it.q_row0 + r) * q_stride + (int64_t)head * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const bf16x4 v = pack4(read_acc_elem(oacc[qb][db], 4 * g) * inv, read_acc_elem(oacc[qb][db], 4 * g + 1) * inv,
                                 read_acc_elem(oacc[qb][db], 4 * g + 2) * inv, read_acc_elem(oacc[qb][db], 4 * g + 3) * inv);
          *reinterpret_cast<bf16x4*>(op + 32 * db + 8 * g + 4 * hh) = v;
        }
      if (hh == 0)
        p.lse[(int64_t)head * p.total_q + it.q_row0 + r] = (m_run[qb] * c + log2f(l_tot)) * 0.6931471805599453f;
    }
  }
}

template <int D, int WAVES>
static hipError_t launch_fwd_t(const FwdParams& p, int num_blocks, hipStream_t stream);

static hipError_t launch_fwd_pipe(const FwdParams& p, int num_blocks, hipStream_t stream) {
  const size_t smem = (size_t)4 * 64 * 128 * 2;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&fwd_pipe_kernel<128>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((fwd_pipe_kernel<128>), dim3(num_blocks), dim3(256), smem, stream, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // second pass over the same items, 8 waves of 32 rows: a workgroup returns at once unless its flag is raised
  return launch_fwd_t<128, 8>(p, num_blocks, stream);
}

template <int D, int WAVES>
static hipError_t launch_fwd_t(const FwdParams& p, int num_blocks, hipStream_t stream) {
  const size_t smem = (size_t)4 * 64 * D * 2;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&fwd_kernel<D, WAVES>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((fwd_kernel<D, WAVES>), dim3(num_blocks), dim3(WAVES * 64), smem, stream, p);
  return hipGetLastError();
}

hipError_t launch_fwd(const FwdParams& p, int head_dim, int num_blocks, hipStream_t stream) {
  return head_dim == 128 ? launch_fwd_pipe(p, num_blocks, stream) : launch_fwd_t<64, 4>(p, num_blocks, stream);
}

}  // namespace chunk_attn
