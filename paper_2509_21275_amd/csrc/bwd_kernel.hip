// Chunk attention backward for gfx950 (gradients of L = sum(O .* dO) under the chunk mask of the
// paper's section 3.1; key/value gradients include the context rows, section 2.1 / 3.2.2).
//
// Two reductions are needed -- dQ sums over keys, dK/dV sum over queries -- and a workgroup can keep
// only one of them in registers.  Float atomics for the other one are far too slow on this chip at the
// rate an attention backward produces them, so each reduction gets its own kernel and every output
// element is written exactly once (the result is also bit-reproducible):
//
//   bwd_pre   D_i = <dO_i, O_i> and LSE_i log2(e) per (head, row), stored in arrays padded to 64-row
//             tiles per segment (+inf / 0 in the padding, so padded rows yield P = 0);
//   transposes (transpose_kernel.hip) of K (32-row tiles) and of Q, dO (64-row tiles);
//   bwd_dq    query-stationary, like the forward: S^T = K Q^T and dP^T = V dO^T per 32-key tile,
//             dS^T = P^T (dP^T - D), dQ^T += K^T dS^T with dS^T fed back from the accumulator registers;
//   bwd_dkv   key-stationary: one workgroup per 128 keys of one key/value head, K and V fragments in
//             registers, walking the query heads of the group and the 64-row query tiles that see
//             those keys: S = Q K^T, dP = dO V^T, dV^T += dO^T P, dK^T += Q^T dS with P and dS fed back
//             from the accumulator registers.
// P is recomputed from the saved log-sum-exp in both kernels.  All operands reach LDS by global->LDS
// copies and are read with 16-byte LDS reads from swizzled tiles (tiles.hpp).
#include <cstring>
#include <type_traits>

#include "kernels.hpp"
#include "tiles.hpp"

namespace chunk_attn {

namespace {

constexpr float kLog2e = 1.4426950408889634f;

// ------------------------------------------------------------------------------------------------
// bwd_pre: one workgroup per (64-row query tile, head); 4 threads per row.
// ------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void bwd_pre_kernel(const __bf16* __restrict__ o, const __bf16* __restrict__ d_o,
                                                      const float* __restrict__ lse, const TileJob* __restrict__ jobs,
                                                      int64_t total_q_tiles, int total_q, int num_q_heads,
                                                      float* __restrict__ lse2p, float* __restrict__ dsp) {
  const int head = blockIdx.x % num_q_heads;
  const TileJob job = jobs[blockIdx.x / num_q_heads];
  const int r = threadIdx.x >> 2, part = threadIdx.x & 3;
  float acc = 0.f;
  const bool valid = r < job.valid_rows;
  if (valid) {
    const int64_t base = ((int64_t)(job.src_row0 + r) * num_q_heads + head) * D + part * (D / 4);
#pragma unroll
    for (int c = 0; c < D / 32; ++c) {
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(o + base + c * 8);
      const bf16x8 b = *reinterpret_cast<const bf16x8*>(d_o + base + c * 8);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc += (float)a[i] * (float)b[i];
    }
  }
  acc += __shfl_xor(acc, 1);
  acc += __shfl_xor(acc, 2);
  if (part == 0) {
    const int64_t slot = ((int64_t)head * total_q_tiles + job.image) * 64 + r;
    dsp[slot] = valid ? acc : 0.f;
    lse2p[slot] = valid ? lse[(int64_t)head * total_q + job.src_row0 + r] * kLog2e : INFINITY;
  }
}

// zero `n16` 16-byte units starting at p
__global__ __launch_bounds__(256) void zero_fill_kernel(u32x4* __restrict__ p, int64_t n16) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n16) p[i] = u32x4{0u, 0u, 0u, 0u};
}

// ------------------------------------------------------------------------------------------------
// bwd_dq
// ------------------------------------------------------------------------------------------------
struct DqParams {
  const __bf16 *q, *k, *v, *d_o;
  const __bf16* kt;      // transposed K images [Hkv][total_kv32_tiles][D][32]
  const float* lse2p;    // [Hq][total_q_tiles * 64]
  const float* dsp;
  __bf16* dq;
  const DqItem* items;
  int64_t total_kv32_tiles, total_q_tiles;
  int32_t num_q_heads, num_kv_heads, group, heads_per_wg, head_splits;
  float scale, scale_log2;
};

template <int D>
__global__ __launch_bounds__(256, 2) void bwd_dq_kernel(DqParams p) {
  constexpr int BN = 32;       // key rows per LDS tile
  constexpr int KC = D / 8;    // 16-byte chunks per K / V row
  constexpr int DK = D / 16;   // k-steps over the head dimension
  constexpr int DB = D / 32;   // 32-row blocks of dQ^T
  constexpr int KT = BN * D;   // elements per tile

  constexpr int NS = 3;        // LDS stages: tiles are fetched NS - 1 iterations ahead

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  __bf16* Ks = reinterpret_cast<__bf16*>(smem);  // [NS][BN][D]
  __bf16* Vs = Ks + NS * KT;                     // [NS][BN][D]
  __bf16* Ts = Vs + NS * KT;                     // [NS][D][BN]  K^T image

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hh = lane >> 5;
  stagger_wave_priority();

  const int inner_n = p.num_kv_heads * p.head_splits;
  const int inner = blockIdx.x % inner_n;
  const DqItem it = p.items[blockIdx.x / inner_n];
  const int kvh = inner % p.num_kv_heads, hs = inner / p.num_kv_heads;
  const int head = kvh * p.group + hs * p.heads_per_wg + wave % p.heads_per_wg;
  const int wave_row0 = (wave / p.heads_per_wg) * 32;

  const int n_wg = it.n0 + it.q_rows - 1;
  const int nt_wg = (n_wg + BN - 1) / BN;
  int nt_w = 0;
  if (wave_row0 < it.q_rows) {
    const int last = min(wave_row0 + 32, it.q_rows) - 1;
    nt_w = (it.n0 + last + BN - 1) / BN;
  }

  const int64_t q_stride = (int64_t)p.num_q_heads * D, kv_stride = (int64_t)p.num_kv_heads * D;
  const __bf16* __restrict__ Kg = p.k + (int64_t)it.kv_row0 * kv_stride + (int64_t)kvh * D;
  const __bf16* __restrict__ Vg = p.v + (int64_t)it.kv_row0 * kv_stride + (int64_t)kvh * D;
  const __bf16* __restrict__ Timg = p.kt + ((int64_t)kvh * p.total_kv32_tiles + it.kv_tile0) * KT;

  constexpr int NK = BN * KC / 256, NT = KT / 8 / 256;
  unsigned k_src[NK];
  int k_row[NK];
#pragma unroll
  for (int i = 0; i < NK; ++i) {
    const int x = (i * 4 + wave) * 64 + lane;
    k_row[i] = x / KC;
    k_src[i] = (unsigned)(k_row[i] * (int)kv_stride + unswz<KC>(k_row[i], x % KC) * 8);
  }
  // One tile is copied by NK + NT pieces per lane (piece i < NK: a K and a V chunk; else a K^T image chunk), so
  // that the copies can be issued between MFMAs instead of in one burst.
  auto dma_piece = [&](int t, int buf, int i) {
    if (i < NK) {
      const int64_t toff = (int64_t)(BN * t) * kv_stride;  // wave-uniform
      const int last_row = n_wg - 1 - BN * t;
      unsigned off = k_src[i];
      if (last_row < BN - 1) off -= (unsigned)((k_row[i] - min(k_row[i], last_row)) * (int)kv_stride);
      dma16(Kg + toff + off, Ks + buf * KT + (i * 4 + wave) * 512);
      dma16(Vg + toff + off, Vs + buf * KT + (i * 4 + wave) * 512);
    } else {
      const int j = i - NK;
      const __bf16* tsrc = Timg + (int64_t)t * KT;
      dma16(tsrc + (unsigned)(((j * 4 + wave) * 64 + lane) * 8), Ts + buf * KT + (j * 4 + wave) * 512);
    }
  };
  auto dma_tile = [&](int t, int buf) {
#pragma unroll
    for (int i = 0; i < NK + NT; ++i) dma_piece(t, buf, i);
  };

  // Q and dO fragments (B operands): lane holds X[row = l32][16 ks + 8 hh ..+7]
  bf16x8 qf[DK], gf[DK];
  const int r_own = min(wave_row0 + l32, it.q_rows - 1);  // rows past the tile repeat the last one (never stored)
  {
    const int64_t off = (int64_t)(it.q_row0 + r_own) * q_stride + (int64_t)head * D + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) {
      qf[ks] = *reinterpret_cast<const bf16x8*>(p.q + off + 16 * ks);
      gf[ks] = *reinterpret_cast<const bf16x8*>(p.d_o + off + 16 * ks);
    }
  }
  const int64_t slot = (int64_t)head * p.total_q_tiles * 64 + it.q_slot0 + r_own;
  const float lse2 = p.lse2p[slot], dsum = p.dsp[slot];

  // prologue: the first NS - 1 tiles (issued after the register loads so that vmcnt below counts only copies)
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < nt_wg) dma_tile(s, s);

  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 dq[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) dq[db] = zero16;
  const float c = p.scale_log2;

  int k_off[DK], t_off[2];
#pragma unroll
  for (int ks = 0; ks < DK; ++ks) k_off[ks] = tile_elem<KC>(l32, 2 * ks + hh);
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) t_off[ks] = tile_elem<4>(l32, 2 * ks + hh);

  // wait until at most `tiles_in_flight` later tiles are still being copied (each is NK * 2 + NT copies per lane)
  auto wait_tiles = [&](int tiles_in_flight) {
    constexpr int PER = 2 * NK + NT;
    if (tiles_in_flight <= 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PER) : "memory");
  };
  wait_tiles(min(nt_wg, NS - 1) - 1);
  wg_barrier();

  auto tile_step = [&](int t, auto buf_c) {
    constexpr int buf = decltype(buf_c)::value;
    const bool prefetch = t + NS - 1 < nt_wg;
    if (t >= nt_w && prefetch) dma_tile(t + NS - 1, (buf + NS - 1) % NS);  // idle wave: still does its share of the copies

    if (t < nt_w) {
      const __bf16* Kt = Ks + buf * KT;
      const __bf16* Vt = Vs + buf * KT;
      const __bf16* Tt = Ts + buf * KT;
      // The loop body is laid out as stages separated by scheduling fences: each stage issues the LDS reads
      // of the next stage's operands together with the MFMAs of the current one, so the reads' latency is
      // covered by matrix work instead of stalling every MFMA on the read issued just before it.
      auto ldk = [&](int ks) { return *reinterpret_cast<const bf16x8*>(Kt + k_off[ks]); };
      auto ldv = [&](int ks) { return *reinterpret_cast<const bf16x8*>(Vt + k_off[ks]); };
      // ---- S^T = K Q^T, dP^T = V dO^T : [32 keys] x [32 queries] ----
      f32x16 s, dp;
      bf16x8 ak[2][2], av[2][2];  // [parity of the k-step pair][step in the pair]
      ak[0][0] = ldk(0); av[0][0] = ldv(0); ak[0][1] = ldk(1); av[0][1] = ldv(1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int g = 0; g < DK / 2; ++g) {
        const int cur = g & 1, nxt = cur ^ 1;
        if (g + 1 < DK / 2) {
          ak[nxt][0] = ldk(2 * g + 2); av[nxt][0] = ldv(2 * g + 2);
          ak[nxt][1] = ldk(2 * g + 3); av[nxt][1] = ldv(2 * g + 3);
        }
        s = mfma32(ak[cur][0], qf[2 * g], g == 0 ? zero16 : s);
        dp = mfma32(av[cur][0], gf[2 * g], g == 0 ? zero16 : dp);
        if (prefetch && g < NK + NT) dma_piece(t + NS - 1, (buf + NS - 1) % NS, g);
        s = mfma32(ak[cur][1], qf[2 * g + 1], s);
        dp = mfma32(av[cur][1], gf[2 * g + 1], dp);
        __builtin_amdgcn_sched_barrier(0);
      }
      // operands of dQ^T += K^T dS^T, fetched while the exponentials are computed
      bf16x8 at[2][DB];
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        at[0][db] = *reinterpret_cast<const bf16x8*>(Tt + t_off[0] + db * 32 * BN);
        at[1][db] = *reinterpret_cast<const bf16x8*>(Tt + t_off[1] + db * 32 * BN);
      }
      // ---- P = exp2(S c - LSE), dS = P (dP - D); masked keys give P = 0 ----
      float pe[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) pe[i] = __builtin_amdgcn_exp2f(s[i] * c - lse2);
      if (BN * t + BN > it.n0 + wave_row0) {
        const int lim = it.n0 + wave_row0 + l32 - BN * t;  // visible iff local key index < lim
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int j = 8 * (i >> 2) + 4 * hh + (i & 3);
          if (j >= lim) pe[i] = 0.f;
        }
      }
      float ds[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) ds[i] = pe[i] * (dp[i] - dsum);
      const bf16x8 f0 = pack8(ds[0], ds[1], ds[2], ds[3], ds[4], ds[5], ds[6], ds[7]);
      const bf16x8 f1 = pack8(ds[8], ds[9], ds[10], ds[11], ds[12], ds[13], ds[14], ds[15]);
      __builtin_amdgcn_sched_barrier(0);
      // ---- dQ^T += K^T dS^T : [D] x [32 queries], contraction over the 32 keys ----
#pragma unroll
      for (int db = 0; db < DB; ++db) dq[db] = mfma32(at[0][db], f0, dq[db]);
#pragma unroll
      for (int db = 0; db < DB; ++db) dq[db] = mfma32(at[1][db], f1, dq[db]);
    }
    // tile t + 1 must have landed; tiles t + 2 .. may still be in flight
    wait_tiles(min(nt_wg - 1, t + NS - 1) - (t + 1));
    wg_barrier();
  };

  for (int t = 0; t < nt_wg; t += NS) {
    tile_step(t, std::integral_constant<int, 0>{});
    if (t + 1 < nt_wg) tile_step(t + 1, std::integral_constant<int, 1>{});
    if (t + 2 < nt_wg) tile_step(t + 2, std::integral_constant<int, 2>{});
  }

  // ---- epilogue: dQ = scale * dQ^T ----
  {
    const int r = wave_row0 + l32;
    if (r < it.q_rows) {
      __bf16* op = p.dq + (int64_t)(it.q_row0 + r) * q_stride + (int64_t)head * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const bf16x4 v = pack4(dq[db][4 * g] * p.scale, dq[db][4 * g + 1] * p.scale, dq[db][4 * g + 2] * p.scale,
                                 dq[db][4 * g + 3] * p.scale);
          *reinterpret_cast<bf16x4*>(op + 32 * db + 8 * g + 4 * hh) = v;
        }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// bwd_dkv
// ------------------------------------------------------------------------------------------------
struct DkvParams {
  const __bf16 *q, *k, *v, *d_o;
  const __bf16* qt;     // transposed Q images  [Hq][total_q_tiles][D][64]
  const __bf16* gt;     // transposed dO images [Hq][total_q_tiles][D][64]
  const float* lse2p;   // [Hq][total_q_tiles * 64]
  const float* dsp;
  __bf16 *dk, *dv;
  const DkvItem* items;
  int64_t total_q_tiles;
  int32_t num_q_heads, num_kv_heads, group;
  float scale, scale_log2;
  int32_t accumulate;
};

template <int D>
__global__ __launch_bounds__(256) void bwd_dkv_kernel(DkvParams p) {
  constexpr int BM = 64;       // query rows per LDS tile
  constexpr int KC = D / 8;
  constexpr int DK = D / 16;
  constexpr int DB = D / 32;
  constexpr int QT = BM * D;   // elements per tile / image

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  __bf16* Qs = reinterpret_cast<__bf16*>(smem);  // [2][BM][D]  rows
  __bf16* Gs = Qs + 2 * QT;                      // [2][BM][D]  rows (dO)
  __bf16* QTs = Gs + 2 * QT;                     // [2][D][BM]  image
  __bf16* GTs = QTs + 2 * QT;                    // [2][D][BM]  image
  float* lse_s = reinterpret_cast<float*>(GTs + 2 * QT);  // [2][BM]
  float* dsum_s = lse_s + 2 * BM;                          // [2][BM]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hh = lane >> 5;

  const int kvh = blockIdx.x % p.num_kv_heads;
  const DkvItem it = p.items[blockIdx.x / p.num_kv_heads];
  const int G = p.group;
  const int64_t q_stride = (int64_t)p.num_q_heads * D, kv_stride = (int64_t)p.num_kv_heads * D;
  const float c = p.scale_log2;

  // this wave's K / V fragments (B operands): lane holds X[key = 32 wave + l32][16 ks + 8 hh ..+7]
  bf16x8 kf[DK], vf[DK];
  {
    const int64_t grow = it.kv_row0 + min(32 * wave + l32, it.kv_rows - 1);
    const int64_t off = grow * kv_stride + (int64_t)kvh * D + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) {
      kf[ks] = *reinterpret_cast<const bf16x8*>(p.k + off + 16 * ks);
      vf[ks] = *reinterpret_cast<const bf16x8*>(p.v + off + 16 * ks);
    }
  }

  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 dkacc[DB], dvacc[DB];  // dK^T, dV^T: [D] x [32 keys of this wave]
#pragma unroll
  for (int db = 0; db < DB; ++db) { dkacc[db] = zero16; dvacc[db] = zero16; }

  const int nqt = it.n_qt - it.qt_first;
  const int n_iter = nqt * G;

  // ---- staging of one (head, query tile): Q, dO rows; Q^T, dO^T images; LSE, D ----
  constexpr int NQ = BM * KC / 256, NI = QT / 8 / 256;
  unsigned q_src[NQ];
  int q_row[NQ];
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    const int x = (i * 4 + wave) * 64 + lane;
    q_row[i] = x / KC;
    q_src[i] = (unsigned)(q_row[i] * (int)q_stride + unswz<KC>(q_row[i], x % KC) * 8);
  }
  // The copies of one (head, query tile) stage are split into NQ + NI pieces per lane (piece i < NQ: a Q and a dO
  // row chunk; else a Q^T and a dO^T image chunk), so that they can be issued between MFMAs.
  struct StageSrc { int64_t roff, tile; int last_row; };
  auto stage_src = [&](int iter) {
    const int hg = iter / nqt, qt = it.qt_first + iter % nqt;
    const int head = kvh * G + hg;
    StageSrc ss;
    ss.last_row = it.q_len - 1 - qt * BM;  // >= 0
    ss.roff = (int64_t)(it.q_row_seg + qt * BM) * q_stride + (int64_t)head * D;  // wave-uniform
    ss.tile = (int64_t)head * p.total_q_tiles + it.q_tile0 + qt;                  // wave-uniform
    return ss;
  };
  auto dma_piece = [&](const StageSrc& ss, int buf, int i) {
    if (i < NQ) {
      unsigned off = q_src[i];
      if (ss.last_row < BM - 1) off -= (unsigned)((q_row[i] - min(q_row[i], ss.last_row)) * (int)q_stride);
      dma16(p.q + ss.roff + off, Qs + buf * QT + (i * 4 + wave) * 512);
      dma16(p.d_o + ss.roff + off, Gs + buf * QT + (i * 4 + wave) * 512);
    } else {
      const int j = i - NQ;
      const unsigned off = (unsigned)(((j * 4 + wave) * 64 + lane) * 8);
      dma16(p.qt + ss.tile * QT + off, QTs + buf * QT + (j * 4 + wave) * 512);
      dma16(p.gt + ss.tile * QT + off, GTs + buf * QT + (j * 4 + wave) * 512);
    }
  };
  auto dma_rowvals = [&](const StageSrc& ss, int buf) {
    if (wave == 0) dma4(p.lse2p + ss.tile * 64 + lane, lse_s + buf * BM);
    if (wave == 1) dma4(p.dsp + ss.tile * 64 + lane, dsum_s + buf * BM);
  };
  auto dma_stage = [&](int iter, int buf) {
    const StageSrc ss = stage_src(iter);
#pragma unroll
    for (int i = 0; i < NQ + NI; ++i) dma_piece(ss, buf, i);
    dma_rowvals(ss, buf);
  };

  int q_off[DK], t_off[4];
#pragma unroll
  for (int ks = 0; ks < DK; ++ks) q_off[ks] = tile_elem<KC>(l32, 2 * ks + hh);
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) t_off[ks] = tile_elem<8>(l32, 2 * ks + hh);

  // key index of this lane's column inside the segment, relative to the context: query i sees it iff i >= jrel
  const int jrel = it.j0 + 32 * wave + l32 - it.ctx;

  if (n_iter > 0) dma_stage(0, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  auto iter_step = [&](int iter, auto buf_c) {
    constexpr int buf = decltype(buf_c)::value;
    const bool prefetch = iter + 1 < n_iter;
    StageSrc nss{};
    if (prefetch) {
      nss = stage_src(iter + 1);
      dma_rowvals(nss, buf ^ 1);
    }
    const int qt = it.qt_first + iter % nqt;
    const __bf16* Qb = Qs + buf * QT;
    const __bf16* Gb = Gs + buf * QT;
    const __bf16* QTb = QTs + buf * QT;
    const __bf16* GTb = GTs + buf * QT;
    const int i0 = qt * BM;  // first query (inside the segment) of this tile

    // The 64 query rows are handled as two halves of 32; each half is a chain of stages separated by
    // scheduling fences, every stage issuing the LDS reads of the next one together with its own MFMAs (and
    // one piece of the next stage's global->LDS copies), so read latency hides behind matrix work.
    constexpr int PIECES = NQ + NI;
    int piece = 0;
    auto next_piece = [&]() {
      if (prefetch && piece < PIECES) dma_piece(nss, buf ^ 1, piece);
      ++piece;
    };
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      auto ldq = [&](int ks) { return *reinterpret_cast<const bf16x8*>(Qb + q_off[ks] + qb * 32 * D); };
      auto ldg = [&](int ks) { return *reinterpret_cast<const bf16x8*>(Gb + q_off[ks] + qb * 32 * D); };
      // ---- S = Q K^T and dP = dO V^T : [32 queries] x [32 keys of this wave] ----
      f32x16 s, dp;
      bf16x8 aq[2][2], ag[2][2];
      aq[0][0] = ldq(0); ag[0][0] = ldg(0); aq[0][1] = ldq(1); ag[0][1] = ldg(1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int g = 0; g < DK / 2; ++g) {
        const int cur = g & 1, nxt = cur ^ 1;
        if (g + 1 < DK / 2) {
          aq[nxt][0] = ldq(2 * g + 2); ag[nxt][0] = ldg(2 * g + 2);
          aq[nxt][1] = ldq(2 * g + 3); ag[nxt][1] = ldg(2 * g + 3);
        }
        s = mfma32(aq[cur][0], kf[2 * g], g == 0 ? zero16 : s);
        dp = mfma32(ag[cur][0], vf[2 * g], g == 0 ? zero16 : dp);
        next_piece();
        s = mfma32(aq[cur][1], kf[2 * g + 1], s);
        dp = mfma32(ag[cur][1], vf[2 * g + 1], dp);
        __builtin_amdgcn_sched_barrier(0);
      }
      // operands of the first k-step of dV^T / dK^T, fetched while the exponentials are computed
      bf16x8 tg[2][DB], tq[2][DB];
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        tg[0][db] = *reinterpret_cast<const bf16x8*>(GTb + t_off[2 * qb] + db * 32 * BM);
        tq[0][db] = *reinterpret_cast<const bf16x8*>(QTb + t_off[2 * qb] + db * 32 * BM);
      }
      // ---- P = exp2(S c - LSE), dS = P (dP - D); entries a query does not see give P = dS = 0 ----
      const bool need_mask = (i0 + 32 * qb) < (it.j0 + 32 * wave + 31 - it.ctx);
      float pv[16], dsv[16];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 l4 = *reinterpret_cast<const f32x4*>(lse_s + buf * BM + 32 * qb + 8 * g + 4 * hh);
        const f32x4 d4 = *reinterpret_cast<const f32x4*>(dsum_s + buf * BM + 32 * qb + 8 * g + 4 * hh);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int i = 4 * g + r;
          float pe = __builtin_amdgcn_exp2f(s[i] * c - l4[r]);
          if (need_mask) {
            const int qi = i0 + 32 * qb + 8 * g + 4 * hh + r;
            if (qi < jrel) pe = 0.f;
          }
          pv[i] = pe;
          dsv[i] = pe * (dp[i] - d4[r]);
        }
      }
      bf16x8 pfrag[2], dsfrag[2];  // B operands per k-step of 16 queries
      pfrag[0] = pack8(pv[0], pv[1], pv[2], pv[3], pv[4], pv[5], pv[6], pv[7]);
      pfrag[1] = pack8(pv[8], pv[9], pv[10], pv[11], pv[12], pv[13], pv[14], pv[15]);
      dsfrag[0] = pack8(dsv[0], dsv[1], dsv[2], dsv[3], dsv[4], dsv[5], dsv[6], dsv[7]);
      dsfrag[1] = pack8(dsv[8], dsv[9], dsv[10], dsv[11], dsv[12], dsv[13], dsv[14], dsv[15]);
      __builtin_amdgcn_sched_barrier(0);
      // ---- dV^T += dO^T P, dK^T += Q^T dS : [D] x [32 keys], contraction over this half's 32 queries ----
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        tg[1][db] = *reinterpret_cast<const bf16x8*>(GTb + t_off[2 * qb + 1] + db * 32 * BM);
        tq[1][db] = *reinterpret_cast<const bf16x8*>(QTb + t_off[2 * qb + 1] + db * 32 * BM);
      }
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        dvacc[db] = mfma32(tg[0][db], pfrag[0], dvacc[db]);
        dkacc[db] = mfma32(tq[0][db], dsfrag[0], dkacc[db]);
        next_piece();
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        dvacc[db] = mfma32(tg[1][db], pfrag[1], dvacc[db]);
        dkacc[db] = mfma32(tq[1][db], dsfrag[1], dkacc[db]);
        next_piece();
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    static_assert(2 * (DK / 2 + 2 * DB) >= PIECES, "not enough slots for the copies of one stage");

    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    wg_barrier();
  };

  for (int iter = 0; iter < n_iter; iter += 2) {
    iter_step(iter, std::integral_constant<int, 0>{});
    if (iter + 1 < n_iter) iter_step(iter + 1, std::integral_constant<int, 1>{});
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

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
size_t up256(size_t x) { return (x + 255) / 256 * 256; }

template <class K>
hipError_t set_smem(K kernel, size_t smem, bool* done) {
  if (*done) return hipSuccess;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)smem);
  if (e == hipSuccess) *done = true;
  return e;
}

template <int D>
hipError_t launch_bwd_t(const chunk_attn_desc* d, const BwdArgs& a, const BwdPlan& P, hipStream_t stream) {
  char* ws = a.workspace;
  const TileJob* qjobs = reinterpret_cast<const TileJob*>(ws + P.qjobs_off);
  const TileJob* kjobs = reinterpret_cast<const TileJob*>(ws + P.kjobs_off);
  float* lse2p = reinterpret_cast<float*>(ws + P.lse2p_off);
  float* dsp = reinterpret_cast<float*>(ws + P.dsp_off);
  __bf16* qt = reinterpret_cast<__bf16*>(ws + P.qt_off);
  __bf16* gt = reinterpret_cast<__bf16*>(ws + P.gt_off);
  __bf16* kt = reinterpret_cast<__bf16*>(ws + P.kt_off);
  hipError_t e;

  // pre-pass: D, scaled LSE, transposed operand images
  {
    const int64_t blocks = (int64_t)P.qjobs.size() * d->num_q_heads;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL((bwd_pre_kernel<D>), dim3((unsigned)blocks), dim3(256), 0, stream, a.o, a.d_o, a.lse, qjobs,
                       P.q_tiles, d->total_q, d->num_q_heads, lse2p, dsp);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if ((e = launch_transpose(a.q, d->num_q_heads, D, 64, qjobs, (int)P.qjobs.size(), P.q_tiles, qt, stream)) != hipSuccess) return e;
  if ((e = launch_transpose(a.d_o, d->num_q_heads, D, 64, qjobs, (int)P.qjobs.size(), P.q_tiles, gt, stream)) != hipSuccess) return e;
  if ((e = launch_transpose(a.k, d->num_kv_heads, D, 32, kjobs, (int)P.kjobs.size(), P.kv32_tiles, kt, stream)) != hipSuccess) return e;

  if (!a.accumulate) {  // rows no segment covers receive no gradient
    for (const auto& gap : uncovered_kv_ranges(d)) {
      const int64_t n16 = (int64_t)(gap.second - gap.first) * d->num_kv_heads * D / 8;
      for (__bf16* base : {a.dk, a.dv}) {
        u32x4* ptr = reinterpret_cast<u32x4*>(base + (int64_t)gap.first * d->num_kv_heads * D);
        hipLaunchKernelGGL(zero_fill_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, stream, ptr, n16);
      }
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
  }

  const int group = d->num_q_heads / d->num_kv_heads;
  {  // dQ
    DqParams p;
    p.q = a.q; p.k = a.k; p.v = a.v; p.d_o = a.d_o; p.kt = kt; p.lse2p = lse2p; p.dsp = dsp; p.dq = a.dq;
    p.items = reinterpret_cast<const DqItem*>(ws + P.dq_items_off);
    p.total_kv32_tiles = P.kv32_tiles; p.total_q_tiles = P.q_tiles;
    p.num_q_heads = d->num_q_heads; p.num_kv_heads = d->num_kv_heads; p.group = group;
    p.heads_per_wg = fwd_heads_per_wg(group); p.head_splits = group / p.heads_per_wg;
    p.scale = d->softmax_scale; p.scale_log2 = d->softmax_scale * kLog2e;
    const size_t smem = (size_t)9 * 32 * D * 2;  // 3 stages of K, V and K^T tiles
    static bool attr = false;
    if ((e = set_smem(&bwd_dq_kernel<D>, smem, &attr)) != hipSuccess) return e;
    const int64_t blocks = (int64_t)P.dq_items.size() * d->num_kv_heads * p.head_splits;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL((bwd_dq_kernel<D>), dim3((unsigned)blocks), dim3(256), smem, stream, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  {  // dK, dV
    DkvParams p;
    p.q = a.q; p.k = a.k; p.v = a.v; p.d_o = a.d_o; p.qt = qt; p.gt = gt; p.lse2p = lse2p; p.dsp = dsp;
    p.dk = a.dk; p.dv = a.dv;
    p.items = reinterpret_cast<const DkvItem*>(ws + P.dkv_items_off);
    p.total_q_tiles = P.q_tiles;
    p.num_q_heads = d->num_q_heads; p.num_kv_heads = d->num_kv_heads; p.group = group;
    p.scale = d->softmax_scale; p.scale_log2 = d->softmax_scale * kLog2e;
    p.accumulate = a.accumulate ? 1 : 0;
    const size_t smem = (size_t)8 * 64 * D * 2 + 4 * 64 * sizeof(float);
    static bool attr = false;
    if ((e = set_smem(&bwd_dkv_kernel<D>, smem, &attr)) != hipSuccess) return e;
    const int64_t blocks = (int64_t)P.dkv_items.size() * d->num_kv_heads;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    ProfileEvents pe = profile_events();
    profile_events() = ProfileEvents{};
    if (pe.start && (e = hipEventRecord(pe.start, stream)) != hipSuccess) return e;
    hipLaunchKernelGGL((bwd_dkv_kernel<D>), dim3((unsigned)blocks), dim3(256), smem, stream, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (pe.stop && (e = hipEventRecord(pe.stop, stream)) != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace

void bwd_layout(const chunk_attn_desc* d, BwdPlan& P, bool with_plan) {
  const int group = d->num_q_heads / d->num_kv_heads;
  const int dq_rows = fwd_tile_rows(group);
  P.q_tiles = count_tiles(d, false, 64);
  P.kv32_tiles = count_tiles(d, true, 32);
  size_t n_dq = 0, n_dkv = 0;
  if (with_plan) {
    P.dq_items = plan_dq(d, dq_rows);
    P.dkv_items = plan_dkv(d);
    P.qjobs = tile_jobs(d, false, 64, nullptr);
    P.kjobs = tile_jobs(d, true, 32, nullptr);
    n_dq = P.dq_items.size();
    n_dkv = P.dkv_items.size();
  } else {
    for (int t = 0; t < d->num_segments; ++t) {
      n_dq += (d->segments[t].q_len + dq_rows - 1) / dq_rows;
      n_dkv += (d->segments[t].kv_len + 127) / 128;
    }
  }
  P.dq_items_off = 0;
  P.dkv_items_off = up256(n_dq * sizeof(DqItem));
  P.qjobs_off = P.dkv_items_off + up256(n_dkv * sizeof(DkvItem));
  P.kjobs_off = P.qjobs_off + up256((size_t)P.q_tiles * sizeof(TileJob));
  P.blob_bytes = P.kjobs_off + up256((size_t)P.kv32_tiles * sizeof(TileJob));
  const size_t row_slots = (size_t)d->num_q_heads * P.q_tiles * 64;
  P.lse2p_off = P.blob_bytes;
  P.dsp_off = P.lse2p_off + up256(row_slots * sizeof(float));
  P.qt_off = P.dsp_off + up256(row_slots * sizeof(float));
  const size_t qimg = up256(row_slots * d->head_dim * sizeof(__bf16));
  P.gt_off = P.qt_off + qimg;
  P.kt_off = P.gt_off + qimg;
  P.total = P.kt_off + up256((size_t)d->num_kv_heads * P.kv32_tiles * 32 * d->head_dim * sizeof(__bf16));
}

std::vector<char> bwd_blob(const BwdPlan& P) {
  std::vector<char> blob(P.blob_bytes);
  std::memcpy(blob.data() + P.dq_items_off, P.dq_items.data(), P.dq_items.size() * sizeof(DqItem));
  std::memcpy(blob.data() + P.dkv_items_off, P.dkv_items.data(), P.dkv_items.size() * sizeof(DkvItem));
  std::memcpy(blob.data() + P.qjobs_off, P.qjobs.data(), P.qjobs.size() * sizeof(TileJob));
  std::memcpy(blob.data() + P.kjobs_off, P.kjobs.data(), P.kjobs.size() * sizeof(TileJob));
  return blob;
}

hipError_t launch_bwd(const chunk_attn_desc* d, const BwdArgs& a, const BwdPlan& P, hipStream_t stream) {
  return d->head_dim == 128 ? launch_bwd_t<128>(d, a, P, stream) : launch_bwd_t<64>(d, a, P, stream);
}

}  // namespace chunk_attn
