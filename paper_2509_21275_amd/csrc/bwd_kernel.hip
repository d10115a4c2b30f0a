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
//   transpose (transpose_kernel.hip) of K into 32-row tile images, for the dQ kernel;
//   bwd_dq    query-stationary, like the forward: S^T = K Q^T and dP^T = V dO^T per 32-key tile,
//             dS^T = P^T (dP^T - D), dQ^T += K^T dS^T with dS^T fed back from the accumulator registers;
//   bwd_dkv   key-stationary: one workgroup per 128 keys of one key/value head, walking the query heads of
//             the group and the 32-row query tiles that see those keys; two wave roles per key block,
//             S = Q K^T, P, dV^T += dO^T P  and  dP = dO V^T, dS, dK^T += Q^T dS (see the kernel).
// P is recomputed from the saved log-sum-exp in both kernels.  All operands reach LDS by global->LDS copies.
#include <cstring>
#include <cstdlib>
#include <type_traits>

#include "kernels.hpp"
#include "tiles.hpp"

namespace chunk_attn {

namespace {

constexpr float kLog2e = 1.4426950408889634f;

#ifndef DKV_PIPE_DIST
#define DKV_PIPE_DIST 3
#endif
#ifndef DQ_PIPE_DIST
#define DQ_PIPE_DIST 3  // stages the pipelined dQ kernel copies ahead
#endif

// ------------------------------------------------------------------------------------------------
// bwd_pre: one workgroup per (64-row query tile, head); D / 8 threads per row, one 16-byte chunk of O and of dO each, so
// that a wave reads whole rows (the kernel is bound by memory: it reads O and dO once).
// ------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void bwd_pre_kernel(const __bf16* __restrict__ o, const __bf16* __restrict__ d_o,
                                                      const float* __restrict__ lse, const TileJob* __restrict__ jobs,
                                                      int64_t total_q_tiles, int total_q, int num_q_heads,
                                                      float* __restrict__ lse2p, float* __restrict__ dsp) {
  constexpr int TPR = D / 8;         // threads per row
  constexpr int RPP = 256 / TPR;     // rows per pass
  const int head = blockIdx.x % num_q_heads;
  const TileJob job = jobs[blockIdx.x / num_q_heads];
  const int part = threadIdx.x % TPR;
#pragma unroll
  for (int pass = 0; pass < 64 / RPP; ++pass) {
    const int r = pass * RPP + threadIdx.x / TPR;
    const bool valid = r < job.valid_rows;
    float acc = 0.f;
    if (valid) {
      const int64_t base = ((int64_t)(job.src_row0 + r) * num_q_heads + head) * D + part * 8;
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(o + base);
      const bf16x8 b = *reinterpret_cast<const bf16x8*>(d_o + base);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc += (float)a[i] * (float)b[i];
    }
#pragma unroll
    for (int w = 1; w < TPR; w *= 2) acc += __shfl_xor(acc, w);
    if (part == 0) {
      const int64_t slot = ((int64_t)head * total_q_tiles + job.image) * 64 + r;
      dsp[slot] = valid ? -acc : 0.f;  // stored negated: the kernels add it (or start an accumulation from it)
      lse2p[slot] = valid ? lse[(int64_t)head * total_q + job.src_row0 + r] * kLog2e : INFINITY;
    }
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
  int32_t* taken;        // 8 block-queue counters of the pipelined kernel (zero before the launch)
  unsigned long long* clock_log;  // null, or where the pipelined kernel's workgroups log their clocks
};

template <int D, int WAVES>
__global__ __launch_bounds__(WAVES * 64, D > 128 ? 1 : 8 / WAVES) void bwd_dq_kernel(DqParams p) {
  constexpr int NTH = WAVES * 64;  // threads
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

  constexpr int NK = BN * KC / NTH, NT = KT / 8 / NTH;
  static_assert(NK >= 1 && NT >= 1, "every thread copies at least one chunk of each tile");
  unsigned k_src[NK];
  int k_row[NK];
#pragma unroll
  for (int i = 0; i < NK; ++i) {
    const int x = (i * WAVES + wave) * 64 + lane;
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
      dma16(Kg + toff + off, Ks + buf * KT + (i * WAVES + wave) * 512);
      dma16(Vg + toff + off, Vs + buf * KT + (i * WAVES + wave) * 512);
    } else {
      const int j = i - NK;
      const __bf16* tsrc = Timg + (int64_t)t * KT;
      dma16(tsrc + (unsigned)(((j * WAVES + wave) * 64 + lane) * 8), Ts + buf * KT + (j * WAVES + wave) * 512);
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
      for (int i = 0; i < 16; ++i) ds[i] = pe[i] * (dp[i] + dsum);
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
//
// One workgroup = 128 consecutive keys of one segment and one key/value head, 8 waves.  The four
// contractions of a (32-query, 32-key) block are split between two waves that share the block's keys:
//   wave A (waves 0..3): S = Q K^T, P = exp2(S c - LSE), dV^T += dO^T P;  hands P (bf16) to wave B through LDS
//   wave B (waves 4..7): dP = dO V^T, dS = P (dP - D),   dK^T += Q^T dS;  runs one step behind wave A
// so each wave keeps one fragment set (K or V) and one accumulator (dV^T or dK^T) and the whole kernel
// fits 256 registers per lane: two waves per SIMD, whose matrix and vector phases overlap.
// The workgroup walks the group's query heads and, per head, the 32-row query tiles that see its keys.
//
// Only the rows of Q and dO are streamed (global->LDS copies into 4-slot rings, two steps ahead); each tile
// serves both contractions that need it: as rows (16-byte reads, operand of Q K^T / dO V^T) and transposed
// (ds_read_b64_tr_b16, operand of Q^T dS / dO^T P).  A tile is stored chunk-major: 16-byte chunk c of row r
// sits at slot c * 32 + (r ^ 4 (c & 3)).  With that layout both kinds of read are bank-conflict free and
// their addresses are one per-lane base plus constants.
// ------------------------------------------------------------------------------------------------
struct DkvParams {
  const __bf16 *q, *k, *v, *d_o;
  const float* lse2p;   // [Hq][total_q_tiles * 64]
  const float* dsp;
  __bf16 *dk, *dv;
  const DkvItem* items;
  int64_t total_q_tiles;
  int32_t num_q_heads, num_kv_heads, group;
  float scale, scale_log2;
  int32_t accumulate;
  int32_t out_f32;      // dk / dv point to fp32 arrays of the same shape
  int32_t* taken;       // 8 block-queue counters of the pipelined kernel (zero before the launch)
  int32_t* ended;       // per queue, the blocks that have ended (zero before the launch)
  int32_t side_by_side; // blocks of a queue that run at the same time (DkvItem::in_step)
  unsigned long long* clock_log;  // null, or where the pipelined kernel's workgroups log their clocks
};

// Four consecutive elements of a dK / dV row: stored, or added to what is there, as bf16 or as fp32.
__device__ __forceinline__ void dkv_store4(const DkvParams& p, __bf16* out, int64_t elem, float v0, float v1, float v2,
                                           float v3) {
  if (p.out_f32) {
    f32x4* op = reinterpret_cast<f32x4*>(reinterpret_cast<float*>(out) + elem);
    if (p.accumulate) {
      const f32x4 old = *op;
      v0 += old[0]; v1 += old[1]; v2 += old[2]; v3 += old[3];
    }
    const f32x4 nv = {v0, v1, v2, v3};
    *op = nv;
  } else {
    bf16x4* op = reinterpret_cast<bf16x4*>(out + elem);
    if (p.accumulate) {
      const bf16x4 old = *op;
      v0 += (float)old[0]; v1 += (float)old[1]; v2 += (float)old[2]; v3 += (float)old[3];
    }
    *op = pack4(v0, v1, v2, v3);
  }
}


template <int D, int KB>  // KB: 32-key blocks per workgroup (2 KB waves)
__global__ __launch_bounds__(KB * 128, D > 128 ? 1 : 4 / KB) void bwd_dkv_kernel(DkvParams p) {
  constexpr int NW = 2 * KB;   // waves
  constexpr int NTH = NW * 64; // threads
  constexpr int BM = 32;       // query rows per step
  constexpr int KC = D / 8;    // 16-byte chunks per operand row
  constexpr int DK = D / 16;   // k-steps over the head dimension
  constexpr int DB = D / 32;   // 32-row blocks of dK^T / dV^T
  constexpr int QT = BM * D;   // elements per operand tile
  constexpr int NS = 4;        // ring slots
  constexpr int PT = KB * 64 * 16;     // elements of one P hand-over slot: KB key blocks x 64 lanes x 16 values
  constexpr int CH = BM * KC;          // 16-byte chunks per operand tile
  constexpr int PER = 2 * CH / NTH;    // global->LDS copies per thread and stage
  constexpr int NP = CH / 64;          // 64-slot pieces per tile
  constexpr int RV = 64;               // floats per slot of the LSE / D rows (32 used; a whole wave copies them)
  static_assert(PER >= 1 && 2 * NP % NW == 0, "the pieces of the two tiles divide evenly among the waves");

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  lds_bf16* const L = (lds_bf16*)smem;
  constexpr int Q_OFF = 0;                 // [NS][QT]  Q rows of stage n in slot n % NS   (wave A: step n, wave B: step n + 1)
  constexpr int G_OFF = Q_OFF + NS * QT;   // [NS][QT]  dO rows                            (both waves: step n)
  constexpr int P_OFF = G_OFF + NS * QT;   // [2][PT]   P hand-over
  lds_f32* const lse_s = (lds_f32*)(L + P_OFF + 2 * PT);  // [NS][RV]  slot n % NS        (wave A, step n)
  lds_f32* const dsum_s = lse_s + NS * RV;                // [NS][RV]  slot n % NS        (wave B, step n + 1)

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int role = wave / KB, kb = wave % KB;
  const int l32 = lane & 31, hh = lane >> 5;

  const int kvh = blockIdx.x % p.num_kv_heads;
  const DkvItem it = p.items[blockIdx.x / p.num_kv_heads];
  const int G = p.group;
  const int64_t q_stride = (int64_t)p.num_q_heads * D, kv_stride = (int64_t)p.num_kv_heads * D;
  const float c = p.scale_log2;

  // this wave's K (wave A) or V (wave B) fragments, B operands: lane holds X[key = 32 kb + l32][16 ks + 8 hh ..+7]
  bf16x8 bfrag[DK];
  {
    const __bf16* src = role ? p.v : p.k;
    const int64_t grow = it.kv_row0 + min(32 * kb + l32, it.kv_rows - 1);
    const int64_t off = grow * kv_stride + (int64_t)kvh * D + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) bfrag[ks] = *reinterpret_cast<const bf16x8*>(src + off + 16 * ks);
  }

  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 acc[DB];  // dV^T (wave A) or dK^T (wave B): [D] x [32 keys of this wave]
#pragma unroll
  for (int db = 0; db < DB; ++db) acc[db] = zero16;

  const int nqt = it.n_qt - it.qt_first;
  const int n_iter = nqt * G;  // stages: (head in group, query tile), head-major

  // ---- staging: a copy instruction of a wave fills 64 consecutive slots of a tile = two chunk columns of 32 rows;
  // the lane fetches the chunk that belongs in its slot.  The 2 NP pieces of a stage (NP of Q, then NP of dO) are
  // dealt to the waves round robin.  Wave 0 also copies the stage's LSE rows, wave 1 its D rows. ----
  int s_off[PER];  // element offset of the lane's chunk inside its row ...
  int s_row[PER];  // ... and the row, per piece
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int x = ((i * NW + wave) % NP) * 64 + lane;
    s_off[i] = (x >> 5) * 8;
    s_row[i] = (x & 31) ^ (((x >> 5) & 3) << 2);
  }
  int d_qt = it.qt_first, d_hg = 0;  // (query tile, head in group) of the next stage to copy
  auto dma_stage = [&](auto slot_c) {
    constexpr int sl = decltype(slot_c)::value;
    const int head = kvh * G + d_hg;
    const int last_row = it.q_len - 1 - d_qt * BM;  // >= 0; rows past it repeat it (their P is 0)
    const int64_t roff = (int64_t)(it.q_row_seg + d_qt * BM) * q_stride + (int64_t)head * D;
    const int64_t slot = ((int64_t)head * p.total_q_tiles + it.q_tile0) * 64 + d_qt * BM;
    if (wave == 0) dma4(p.lse2p + slot + lane, lse_s + sl * RV);
    if (wave == 1) dma4(p.dsp + slot + lane, dsum_s + sl * RV);
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int piece = i * NW + wave;  // wave-uniform: < NP: Q, else dO
      const unsigned row_off = (unsigned)(min(s_row[i], last_row) * (int)q_stride + s_off[i]);
      if (piece < NP) dma16(p.q + roff + row_off, L + Q_OFF + sl * QT + piece * 512);
      else dma16(p.d_o + roff + row_off, L + G_OFF + sl * QT + (piece - NP) * 512);
    }
    if (++d_qt == it.n_qt) { d_qt = it.qt_first; ++d_hg; }
  };

  // ---- per-lane operand addresses (elements) inside a tile ----
  // rows: A operand of the first contraction, X[row = l32][chunk 2 ks + hh]; k-steps of equal parity are a constant apart
  int x_off[2];
#pragma unroll
  for (int par = 0; par < 2; ++par) x_off[par] = cm_elem(l32, 2 * par + hh);
  // transposed: A operand of the second contraction, X^T[32 db + l32][k-slots of 16 ks2 ..] in accumulator order.
  // Lane j of a 16-lane group addresses the 8 bytes (row k0 + j / 4, elements 16 grp + 4 (j % 4) ..+3); the low and
  // the high half of the operand come from rows 8 apart.  Blocks db and k-steps ks2 are a constant apart.
  int t_off[2];
  {
    const int j = lane & 15, grp = (lane >> 4) & 1;
    const int cl = 2 * grp + ((j & 3) >> 1);  // chunk (mod 4) of the lane's 8 bytes
    const int r0 = 4 * hh + (j >> 2);
#pragma unroll
    for (int half = 0; half < 2; ++half) t_off[half] = cm_elem(r0 + 8 * half, cl) + 4 * (j & 1);
  }
  auto load_rows = [&](const lds_bf16* tile, bf16x8 (&a)[DK]) {
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) a[ks] = lds_load8(tile + x_off[ks & 1] + (ks >> 1) * (4 * 32 * 8));
  };
  auto load_transposed = [&](const lds_bf16* tile, bf16x8 (&t)[2][DB]) {
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const s16x4 lo = lds_read_tr(tile + t_off[0] + ks * (16 * 8) + db * (4 * 32 * 8));
        const s16x4 hi = lds_read_tr(tile + t_off[1] + ks * (16 * 8) + db * (4 * 32 * 8));
        t[ks][db] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
      }
  };

  // key index of this lane's column relative to the context: query i of the segment sees it iff i >= jrel
  const int jrel = it.j0 + 32 * kb + l32 - it.ctx;
  const int jrel_lo = it.j0 + 32 * kb - it.ctx;  // of the wave's first key

  // prologue: stages 0 and 1 (after the fragment loads, so that the waits below count only copies)
  dma_stage(std::integral_constant<int, 0>{});
  if (n_iter > 1) {
    dma_stage(std::integral_constant<int, 1>{});
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PER) : "memory");
  } else {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  wg_barrier();

  int c_qt = it.qt_first, p_qt = it.qt_first;  // query tile of stage g and of stage g - 1
  // end of step g: stage g + 1 must have landed and wave A's P must be visible; the copies issued in this
  // step (stage g + 2) may still be in flight
  auto end_step = [&](bool more) {
    p_qt = c_qt;
    if (++c_qt == it.n_qt) c_qt = it.qt_first;
    if (more) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(PER) : "memory");
    else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    wg_barrier();
  };

  // Wave A defers the second contraction of a block to the beginning of the next step: its operands are in
  // registers by then, so its step opens with eight MFMAs that need nothing from LDS and cover the latency of
  // the operand reads issued at the top of the step.  (The same order measured slower for wave B, which opens
  // with the vector work of the previous block instead.)
  if (role == 0) {
    // ================= wave A: S = Q K^T, P, dV^T += dO^T P =================
    const lds_f32* const rv = lse_s + 4 * hh;
    lds_bf16* const pex = L + P_OFF + kb * 1024 + lane * 8;
    bf16x8 tp[2][DB], fp[2];  // dO^T operands and P of the block whose dV^T product is pending
    bool pend = false;
    auto second = [&]() {
#pragma unroll
      for (int db = 0; db < DB; ++db) acc[db] = mfma32(tp[0][db], fp[0], acc[db]);
#pragma unroll
      for (int db = 0; db < DB; ++db) acc[db] = mfma32(tp[1][db], fp[1], acc[db]);
    };

    auto step = [&](int g, auto u_c) {
      constexpr int u = decltype(u_c)::value;
      const bool more = g + 2 < n_iter;
      const int i0 = c_qt * BM;  // first query (inside the segment) of block g
      const bool vis = g < n_iter && i0 + BM - 1 >= jrel_lo;  // else: no block, or nothing of it visible to this wave
      bf16x8 a[DK], t[2][DB];
      f32x4 r4[4];  // LSE of rows 8 g4 + 4 hh + 0..3
      if (vis) {
        load_rows(L + Q_OFF + u * QT, a);
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) r4[g4] = lds_load4f(rv + u * RV + 8 * g4);
        load_transposed(L + G_OFF + u * QT, t);
      }
      if (pend) second();
      pend = vis;
      if (vis) {
        f32x16 s;
#pragma unroll
        for (int ks = 0; ks < DK; ++ks) s = mfma32(a[ks], bfrag[ks], ks == 0 ? zero16 : s);
        __builtin_amdgcn_sched_barrier(0);
        if (more) dma_stage(std::integral_constant<int, (u + 2) % NS>{});
        __builtin_amdgcn_sched_barrier(0);
        // P = exp2(S c - LSE); entries a query does not see give P = 0
        float w[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) w[i] = __builtin_amdgcn_exp2f(s[i] * c - r4[i >> 2][i & 3]);
        if (i0 < jrel_lo + 31) {
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int qi = i0 + 8 * (i >> 2) + 4 * hh + (i & 3);
            if (qi < jrel) w[i] = 0.f;
          }
        }
        fp[0] = pack8(w[0], w[1], w[2], w[3], w[4], w[5], w[6], w[7]);
        fp[1] = pack8(w[8], w[9], w[10], w[11], w[12], w[13], w[14], w[15]);
        lds_store8(pex + (u & 1) * PT, fp[0]);
        lds_store8(pex + (u & 1) * PT + 512, fp[1]);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
          for (int db = 0; db < DB; ++db) tp[ks][db] = t[ks][db];
      } else if (more) {
        dma_stage(std::integral_constant<int, (u + 2) % NS>{});
      }
      end_step(more);
    };
    for (int g = 0; g <= n_iter; g += NS) {
      step(g, std::integral_constant<int, 0>{});
      if (g + 1 <= n_iter) step(g + 1, std::integral_constant<int, 1>{});
      if (g + 2 <= n_iter) step(g + 2, std::integral_constant<int, 2>{});
      if (g + 3 <= n_iter) step(g + 3, std::integral_constant<int, 3>{});
    }
    if (pend) second();
  } else {
    // ================= wave B: dP = dO V^T, dS = P (dP - D), dK^T += Q^T dS =================
    // In step g it first finishes block g - 1 (vector work with wave A's P, then dK^T) and then starts block g
    // (dP): right after the barrier one wave of each SIMD begins with matrix work and the other with vector work.
    const lds_f32* const rv = dsum_s + 4 * hh;
    const lds_bf16* const pex = L + P_OFF + kb * 1024 + lane * 8;
    f32x16 dp = zero16;  // dP of the block whose dS is formed in the next step

    auto step = [&](int g, auto u_c) {
      constexpr int u = decltype(u_c)::value;
      constexpr int up = (u + NS - 1) % NS;  // slot of stage g - 1
      const bool more = g + 2 < n_iter;
      const bool cur_vis = g < n_iter && (c_qt * BM + BM - 1 >= jrel_lo);
      const bool prev_vis = g >= 1 && (p_qt * BM + BM - 1 >= jrel_lo);
      bf16x8 a[DK];
      if (cur_vis) load_rows(L + G_OFF + u * QT, a);
      if (prev_vis) {
        // ---- dS = P (dP - D) with wave A's P of block g - 1, then dK^T += Q^T dS ----
        const bf16x8 p0 = lds_load8(pex + ((u & 1) ^ 1) * PT);
        const bf16x8 p1 = lds_load8(pex + ((u & 1) ^ 1) * PT + 512);
        f32x4 r4[4];  // D of rows 8 g4 + 4 hh + 0..3
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) r4[g4] = lds_load4f(rv + up * RV + 8 * g4);
        bf16x8 t[2][DB];  // Q^T operands
        load_transposed(L + Q_OFF + up * QT, t);
        float w[16];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          w[i] = (float)p0[i] * (dp[i] + r4[i >> 2][i & 3]);
          w[8 + i] = (float)p1[i] * (dp[8 + i] + r4[2 + (i >> 2)][i & 3]);
        }
        const bf16x8 f0 = pack8(w[0], w[1], w[2], w[3], w[4], w[5], w[6], w[7]);
        const bf16x8 f1 = pack8(w[8], w[9], w[10], w[11], w[12], w[13], w[14], w[15]);
#pragma unroll
        for (int db = 0; db < DB; ++db) acc[db] = mfma32(t[0][db], f0, acc[db]);
#pragma unroll
        for (int db = 0; db < DB; ++db) acc[db] = mfma32(t[1][db], f1, acc[db]);
      }
      __builtin_amdgcn_sched_barrier(0);
      if (more) dma_stage(std::integral_constant<int, (u + 2) % NS>{});
      __builtin_amdgcn_sched_barrier(0);
      if (cur_vis) {
#pragma unroll
        for (int ks = 0; ks < DK; ++ks) dp = mfma32(a[ks], bfrag[ks], ks == 0 ? zero16 : dp);
      }
      end_step(more);
    };
    for (int g = 0; g <= n_iter; g += NS) {
      step(g, std::integral_constant<int, 0>{});
      if (g + 1 <= n_iter) step(g + 1, std::integral_constant<int, 1>{});
      if (g + 2 <= n_iter) step(g + 2, std::integral_constant<int, 2>{});
      if (g + 3 <= n_iter) step(g + 3, std::integral_constant<int, 3>{});
    }
  }

  // ---- epilogue: dV = dV^T (wave A), dK = scale * dK^T (wave B), written (or added) as bf16 ----
  {
    const int kr = 32 * kb + l32;
    if (kr < it.kv_rows) {
      const int64_t off = ((int64_t)it.kv_row0 + kr) * kv_stride + (int64_t)kvh * D;
      __bf16* const out = role ? p.dk : p.dv;
      const float f = role ? p.scale : 1.0f;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          dkv_store4(p, out, off + 32 * db + 8 * g + 4 * hh, acc[db][4 * g] * f, acc[db][4 * g + 1] * f,
                     acc[db][4 * g + 2] * f, acc[db][4 * g + 3] * f);
        }
    }
  }
}

// LDS instructions of one step of bwd_dkv_pipe_kernel in program order, per wave role, and the waits that follow from
// it.  Mini-step m issues the read of fragment m + 4 (two instructions for a transposed fragment: the first NT of a step;
// fragments past the end are the next step's first ones), then E0(m) instructions after its first MFMA and E1(m) after
// its second: role A spreads its four hand-over stores and four row-value reads over mini-steps 0 .. 3 (issued in one go
// they keep the matrix pipe waiting), role B reads the hand-over in mini-step 0 and its row values in mini-step 1.
// LDS operations of a wave complete in order, so "fragment m has arrived" = "at most wait(m) LDS instructions issued
// since its read are outstanding".  The vector work starts in mini-step 4, which therefore also waits for the last of
// the hand-over / row-value instructions.
template <int ROLE, int NF, int NT>
struct DkvLdsOrder {
  static constexpr int cost(int k) { return ((k % NF + NF) % NF) < NT ? 2 : 1; }
  static constexpr int e0(int m) { return ROLE == 0 ? (m < 4 ? 1 : 0) : (m < 2 ? 4 : 0); }
  static constexpr int e1(int m) { return ROLE == 0 ? (m < 2 ? 2 : 0) : 0; }
  static constexpr int after_fragment(int m) {
    int n = m >= 4 ? e0(m - 4) + e1(m - 4) : 0;
    for (int i = m - 3; i < m; ++i) n += cost(i + 4) + (i >= 0 ? e0(i) + e1(i) : 0);
    return n;
  }
  static constexpr int after_extras() {  // instructions between the last E0 / E1 instruction and mini-step 4
    int n = 0;
    for (int i = 3; i >= 0; --i) {
      if (e0(i) + e1(i) > 0) return n;  // nothing of mini-step i follows its last extra instruction
      n += cost(i + 4);
    }
    return n;
  }
  static constexpr int wait(int m) {
    const int a = after_fragment(m);
    return m == 4 && after_extras() < a ? after_extras() : a;
  }
};
// (pins: the counts worked out by hand for head_dim 128, where a step has 16 fragments of which the first 8 are transposed)
static_assert(DkvLdsOrder<1, 16, 8>::wait(0) == 6 && DkvLdsOrder<1, 16, 8>::wait(1) == 10 && DkvLdsOrder<1, 16, 8>::wait(2) == 14 &&
              DkvLdsOrder<1, 16, 8>::wait(3) == 14 && DkvLdsOrder<1, 16, 8>::wait(4) == 4 && DkvLdsOrder<1, 16, 8>::wait(6) == 4 &&
              DkvLdsOrder<1, 16, 8>::wait(7) == 3 && DkvLdsOrder<1, 16, 8>::wait(12) == 3 && DkvLdsOrder<1, 16, 8>::wait(13) == 4 &&
              DkvLdsOrder<1, 16, 8>::wait(14) == 5 && DkvLdsOrder<1, 16, 8>::wait(15) == 6, "role B");
static_assert(DkvLdsOrder<0, 16, 8>::wait(0) == 6 && DkvLdsOrder<0, 16, 8>::wait(1) == 9 && DkvLdsOrder<0, 16, 8>::wait(2) == 12 &&
              DkvLdsOrder<0, 16, 8>::wait(3) == 13 && DkvLdsOrder<0, 16, 8>::wait(4) == 0 && DkvLdsOrder<0, 16, 8>::wait(6) == 6 &&
              DkvLdsOrder<0, 16, 8>::wait(7) == 4 && DkvLdsOrder<0, 16, 8>::wait(8) == 3 && DkvLdsOrder<0, 16, 8>::wait(15) == 6, "role A");

// ------------------------------------------------------------------------------------------------
// bwd_dkv_pipe (head_dim 128)
//
// Same work split as bwd_dkv_kernel, laid out for one wave per SIMD: a workgroup of 4 waves covers 128
// keys; each wave owns 64 keys (two 32-key blocks), waves 0, 1 in role A (S, P, dV^T), waves 2, 3 in role B
// (dP, dS, dK^T).  Every operand fragment read from LDS feeds two MFMAs (the wave's two key blocks), and
// with nobody else on the SIMD the wave overlaps its own matrix and vector work by software pipelining:
// in step g it runs
//     role A:  S(g) = Q K^T           P(g-1) = exp2(S(g-1) c - LSE)       dV^T += dO^T P(g-2)
//     role B:  dP(g-2) = dO V^T       dS(g-3) = P(g-3) (dP(g-3) - D)      dK^T += Q^T dS(g-4)
// (stage n = the n-th (head, 32-row query tile) of the workgroup's walk).  The three pieces of a step are
// independent of each other.  A wave issues at most one instruction every four cycles and an MFMA holds the
// matrix pipe for 32, so the step is laid out instruction by instruction: 16 mini-steps of one operand
// fragment and the two MFMAs it feeds, each MFMA followed by its share of everything else (the vector work
// of one score, an LDS read, a copy), so that the next MFMA finds the pipe just free.  Fragments are fetched
// four mini-steps ahead (the first four of a step before the barrier that ends the previous one).  Role A
// writes P(g-2) to LDS in step g, role B picks it up one step later.  Stages live in a ring of DIST + 5 slots
// (5 in use, DIST on their way from global memory).
// A step runs the same straight-line code whatever the stage.  Stages outside the walk compute on zeros or
// on stale (finite) data and contribute nothing: LDS starts zeroed, and role A starts the S accumulation of
// such a stage from -inf (P = 0), just as it does for the entries a query does not see.
// S and dP are kept in vector registers, where the vector work reads them directly; the compiler would keep
// every MFMA result of a kernel this size in accumulation registers (one extra move per element), so those
// MFMAs are written as opaque instructions.
// ------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256, 1) void bwd_dkv_pipe_kernel(DkvParams p, int num_blocks) {
  constexpr int NW = 4;        // waves
  constexpr int BM = 32;       // query rows per stage
  constexpr int KC = D / 8;    // 16-byte chunks per operand row
  constexpr int DK = D / 16;   // k-steps over the head dimension
  constexpr int DB = D / 32;   // 32-row blocks of dK^T / dV^T
  constexpr int QT = BM * D;   // elements per operand tile
  constexpr int DIST = DKV_PIPE_DIST;  // stages copied ahead of the step that first reads them
  constexpr int NS = DIST + 5; // ring slots: stages g - 4 .. g in use, g + 1 .. g + DIST on their way
  constexpr int NF = 2 * DB + DK;      // operand fragments (mini-steps) per step
  constexpr int AHEAD = 4;             // fragments in flight
  constexpr int PS = 2 * 4 * 64 * 8;   // elements of one P hand-over slot: 2 wave pairs x 4 fragments x 64 lanes x 8
  constexpr int CH = BM * KC;          // 16-byte chunks per operand tile
  constexpr int NP = CH / 64;          // 64-slot pieces per tile
  // global->LDS copies per wave and stage: the 2 NP operand pieces and the two sets of row values (LSE, D) are dealt
  // unevenly, because issuing a copy costs a wave about as long as an MFMA and role A (the exponentials) is the one the
  // step waits for: a role A wave copies two pieces and one set of row values, a role B wave six pieces
  constexpr int PER_A = 2, PER_B = (2 * NP - 2 * PER_A) / 2;  // pieces per wave
  constexpr int CPS_A = PER_A + 1, CPS_B = PER_B;              // copies per wave and stage
  constexpr int RV = 64;               // floats per slot of the LSE / D rows (32 used; a whole wave copies them)
  static_assert(D == 128 && NF == 16 && PER_B == 6, "the mini-step schedule below is written for head_dim 128");

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  lds_bf16* const L = (lds_bf16*)smem;
  constexpr int Q_OFF = 0;                 // [NS][QT]  Q rows of stage n in slot n % NS
  constexpr int G_OFF = Q_OFF + NS * QT;   // [NS][QT]  dO rows
  constexpr int P_OFF = G_OFF + NS * QT;   // [2][PS]   P hand-over
  constexpr int R_OFF = P_OFF + 2 * PS;    // [NS][RV] floats LSE rows, then [NS][RV] floats D rows
  lds_f32* const lse_s = (lds_f32*)(L + R_OFF);
  lds_f32* const dsum_s = lse_s + NS * RV;
  constexpr int LDS_ELEMS = R_OFF + 2 * NS * RV * 2;  // in bf16 units

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int role = wave >> 1, pair = wave & 1;
  const int l32 = lane & 31, hh = lane >> 5;

  // The workgroup is persistent: it claims one block (128 keys of one key/value head) after the other
  // (device_common.hpp) until none is left.  The next block is claimed before the current one's last few steps: early
  // enough for the answer to arrive by the time it is needed, and not earlier (that would fix the order of the blocks
  // before it is known which workgroup is free first).
  __shared__ int next_block;
  const int xcd = xcd_of_this_wave();
  clock_log_stamp(p.clock_log, 0);
  int blk = 0;
  // blocks that walk the same rows as the others of their group wait for the groups before them (DkvItem::in_step)
  auto start_in_step = [&](int b) __attribute__((always_inline)) {
    if (b >= 0 && p.items[b / p.num_kv_heads].in_step) wait_for_earlier_groups(p.ended, b, p.side_by_side);
  };
  if (wave == 0) {
    blk = block_claim_finish(p.taken, num_blocks, xcd, block_claim_issue(p.taken, xcd));
    start_in_step(blk);
  }
  blk = broadcast_from_wave0(&next_block, blk);
  while (blk >= 0) {
  int pending_claim = 0;
  const int kvh = blk % p.num_kv_heads;
  const DkvItem it = p.items[blk / p.num_kv_heads];
  const int G = p.group;
  const int64_t q_stride = (int64_t)p.num_q_heads * D, kv_stride = (int64_t)p.num_kv_heads * D;
  const float c = p.scale_log2;

  // zero everything but the ring slots the prologue fills
  {
    bf16x8 z;
#pragma unroll
    for (int i = 0; i < 8; ++i) z[i] = (__bf16)0.0f;
    for (int x = tid; x < (NS - DIST) * QT / 8; x += NW * 64) {
      lds_store8(L + Q_OFF + DIST * QT + x * 8, z);
      lds_store8(L + G_OFF + DIST * QT + x * 8, z);
    }
    for (int x = tid; x < (LDS_ELEMS - P_OFF) / 8; x += NW * 64) lds_store8(L + P_OFF + x * 8, z);
  }

  const int nqt = it.n_qt - it.qt_first;
  // stages: (query tile, head in group), the heads of a tile one after the other, the tiles upwards from the first one
  // that sees the block's keys or (it.reverse, the host's choice) downwards from the segment's last one.  Workgroups that walk the same rows at
  // about the same time (the key blocks of one key/value head run on one XCD) then touch, per query row, one run of
  // G x D contiguous elements, and blocks of different walk lengths stay side by side for the whole of their common
  // part instead of drifting apart head by head.
  const int n_iter = nqt * G;

  // ---- staging: copy i of a role A wave is piece `pair` of Q (i = 0) or of dO (i = 1), the first of the two waves
  // also copies the stage's LSE rows, the second its D rows; copy i of a role B wave is piece 2 + 2 (i % 3) + pair of Q
  // (i < 3) or of dO.  Past the last stage the last one is copied again (into a slot nobody reads any more), so
  // that every step issues the same number of copies. ----
  // byte offset of the lane's chunk of copy i from the tile's first row, for a full tile and for the segment's
  // last tile (rows past the last query repeat it; their P is 0)
  auto piece_in_tile = [&](int i) { return role == 0 ? pair : 2 + 2 * (i % 3) + pair; };
  unsigned v_full[PER_B], v_last[PER_B];
  {
    const int last_row = it.q_len - 1 - (it.n_qt - 1) * BM;
#pragma unroll
    for (int i = 0; i < PER_B; ++i) {
      const int x = piece_in_tile(i) * 64 + lane;
      const int off = (x >> 5) * 8, row = (x & 31) ^ (((x >> 5) & 3) << 2);
      v_full[i] = (unsigned)(row * (int)q_stride + off) * 2u;
      v_last[i] = (unsigned)(min(row, last_row) * (int)q_stride + off) * 2u;
    }
  }
  // Wave-uniform state of the copies, kept as running byte pointers so that a step spends only a handful of scalar
  // instructions on it: the first row of the next stage to copy in Q and in dO, its LSE / D rows, the stages left in
  // the current head's walk (counting that one), the heads left (counting the current one), the ring slot.
  const bool down = it.reverse != 0;
  const int qt_start = down ? it.n_qt - 1 : it.qt_first;
  const int64_t roff0 = (int64_t)(it.q_row_seg + qt_start * BM) * q_stride + (int64_t)(kvh * G) * D;
  const int64_t rv0 = ((int64_t)(kvh * G) * p.total_q_tiles + it.q_tile0) * 64 + qt_start * BM;
  const char* d_q = reinterpret_cast<const char*>(p.q + roff0);
  const char* d_g = reinterpret_cast<const char*>(p.d_o + roff0);
  const char* d_r = reinterpret_cast<const char*>(((wave & 1) ? p.dsp : p.lse2p) + rv0);
  const int64_t head_bytes = (int64_t)D * 2;                             // to the next head of the group, same tile
  const int64_t head_rows_bytes = p.total_q_tiles * 64 * 4;
  const int64_t tile_bytes = (down ? -1 : 1) * (int64_t)BM * q_stride * 2 - (G - 1) * head_bytes;   // from the last head to the first, next tile
  const int64_t tile_rows_bytes = (down ? -1 : 1) * (int64_t)BM * 4 - (G - 1) * head_rows_bytes;
  int d_heads = G, d_tiles = nqt;
  const int d_ragged = down ? nqt : 1;  // d_tiles while the segment's last query tile is the one to copy
  unsigned d_slot = 0;  // element offset of the ring slot inside the Q / dO rings (slot index x QT)
  const unsigned lane4 = (unsigned)lane * 4u;
  lds_f32* const rows_dst = (wave & 1) ? dsum_s : lse_s;
  auto dma_rows = [&]() __attribute__((always_inline)) { dma4(d_r + lane4, rows_dst + d_slot / (QT / RV)); };
  auto dma_piece = [&](int i) __attribute__((always_inline)) {
    const bool of_q = role == 0 ? i == 0 : i < PER_B / 2;
    const unsigned voff = d_tiles == d_ragged ? v_last[i] : v_full[i];  // the segment's last query tile
    const char* base = of_q ? d_q : d_g;
    lds_bf16* dst = L + (of_q ? Q_OFF : G_OFF) + piece_in_tile(i) * 512 + d_slot;
    dma16(base + voff, dst);
  };
  auto dma_advance = [&]() __attribute__((always_inline)) {
    if (d_heads > 1) {
      --d_heads;
      d_q += head_bytes; d_g += head_bytes; d_r += head_rows_bytes;
    } else {  // on to the next query tile; after the last stage, stay on it
      const bool more = d_tiles > 1;
      d_tiles -= more ? 1 : 0;
      d_heads = more ? G : 1;
      const int64_t tb = more ? tile_bytes : 0, tr = more ? tile_rows_bytes : 0;
      d_q += tb; d_g += tb; d_r += tr;
    }
    d_slot = d_slot == (unsigned)((NS - 1) * QT) ? 0u : d_slot + (unsigned)QT;
  };

  // ---- per-lane operand addresses (elements) inside a tile, as in bwd_dkv_kernel ----
  int x_off[2];
#pragma unroll
  for (int par = 0; par < 2; ++par) x_off[par] = cm_elem(l32, 2 * par + hh);
  int t_off[2];
  {
    const int j = lane & 15, grp = (lane >> 4) & 1;
    const int cl = 2 * grp + ((j & 3) >> 1);
    const int r0 = 4 * hh + (j >> 2);
#pragma unroll
    for (int half = 0; half < 2; ++half) t_off[half] = cm_elem(r0 + 8 * half, cl) + 4 * (j & 1);
  }
  auto prev_slot = [&](int s) __attribute__((always_inline)) { return s == 0 ? NS - 1 : s - 1; };

  // Everything from here on is instantiated once per role, with its own accumulators.
  auto body = [&](auto role_c) __attribute__((always_inline)) {
    constexpr int ROLE = decltype(role_c)::value;
    const lds_bf16* const a_tile = L + (ROLE ? G_OFF : Q_OFF);  // rows operand: Q (role A) or dO (role B)
    const lds_bf16* const t_tile = L + (ROLE ? Q_OFF : G_OFF);  // transposed operand: dO^T (role A) or Q^T (role B)
    const lds_f32* const rv_rows = (ROLE ? dsum_s : lse_s) + 4 * hh;
    lds_bf16* const pex = L + P_OFF + pair * (4 * 512) + lane * 8;

    // this wave's K (role A) or V (role B) fragments, B operands: lane holds X[key = 64 pair + 32 kb + l32][16 ks + 8 hh ..+7]
    bf16x8 bfrag[2][DK];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const __bf16* src = ROLE ? p.v : p.k;
      const int64_t grow = it.kv_row0 + min(64 * pair + 32 * kb + l32, it.kv_rows - 1);
      const int64_t off = grow * kv_stride + (int64_t)kvh * D + 8 * hh;
#pragma unroll
      for (int ks = 0; ks < DK; ++ks) bfrag[kb][ks] = *reinterpret_cast<const bf16x8*>(src + off + 16 * ks);
    }

    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 acc[2][DB];  // dV^T (role A) or dK^T (role B): [D] x [32 keys of block kb]
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int db = 0; db < DB; ++db) acc[kb][db] = zero16;

    // key index of this lane's column of block 0 relative to the context: query i of the segment sees the column of
    // block kb iff i >= jrel + 32 kb
    const int jrel = it.j0 + 64 * pair + l32 - it.ctx;
    const int jrel_hi = it.j0 + 64 * pair + 63 - it.ctx;  // of the wave's last key

    // prologue: stages 0 .. DIST - 1 (after the fragment loads, so that the waits below count only copies)
    constexpr int CPS = ROLE ? CPS_B : CPS_A;      // copies of this wave per stage
    constexpr int PIECES = ROLE ? PER_B : PER_A;
#pragma unroll
    for (int s = 0; s < DIST; ++s) {
      if (ROLE == 0) dma_rows();
#pragma unroll
      for (int i = 0; i < PIECES; ++i) dma_piece(i);
      dma_advance();
    }
    // A wait the compiler can see, for all copies and loads issued so far: without it the compiler's own bookkeeping
    // of outstanding loads makes it put a full vmcnt(0) wait inside the loop (before role A's first S MFMA).
    __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
    wg_barrier();

    // pipeline state
    int sA = ROLE ? NS - 2 : 0;  // slot of stage g - 2 ROLE (rows operand); one before: row values and the next step's
                                 // transposed operand; two before: this step's transposed operand
    int s_qt = qt_start;         // role A: query tile of stage g (whose S is computed in step g)
    int s_heads = G;             //         and the heads of that tile still to come, counting stage g's
    // Role A masks through the accumulator: the first MFMA of S starts from a tile that holds -inf where the query
    // does not see the key (and everywhere for a stage past the end of the walk) and 0 elsewhere.  The tile is
    // rebuilt only for the stages that need it.
    f32x16 mask_c[2] = {zero16, zero16};
    bool mask_set = false;
    f32x16 x[2][2];              // S or dP: [buffer][key block]
    bf16x8 f[2][2][2];           // P or dS as B operands: [buffer][key block][k-step]
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) x[b][kb][i] = ROLE ? 0.f : -INFINITY;  // role A: P = 0 before the first stage
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
          for (int i = 0; i < 8; ++i) f[b][kb][ks][i] = (__bf16)0.0f;
      }
    bf16x8 fr[8];  // ring of operand fragments

    // byte addresses of this lane's operand reads inside slot 0
    const unsigned t_lo0 = lds_addr(t_tile + t_off[0]), t_hi0 = lds_addr(t_tile + t_off[1]);
    const unsigned a_ev0 = lds_addr(a_tile + x_off[0]), a_od0 = lds_addr(a_tile + x_off[1]);
    const unsigned rv0 = lds_addr(rv_rows), pex0 = lds_addr(pex);
    constexpr unsigned SLOT = QT * 2;  // bytes per ring slot
    // transposed fragment m = ks2 * DB + db of the tile at (lo, hi)
    auto load_t = [&](unsigned lo_addr, unsigned hi_addr, auto m_c) __attribute__((always_inline)) {
      constexpr int m = decltype(m_c)::value;
      constexpr int off = ((m / DB) * (16 * 8) + (m % DB) * (4 * 32 * 8)) * 2;
      const s16x4 lo = lds_asm_read_tr<off>(lo_addr);
      const s16x4 hi = lds_asm_read_tr<off>(hi_addr);
      return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    // rows fragment of k-step ks of the tile at (even, odd)
    auto load_a = [&](unsigned ev_addr, unsigned od_addr, auto ks_c) __attribute__((always_inline)) {
      constexpr int ks = decltype(ks_c)::value;
      constexpr int off = (ks >> 1) * (4 * 32 * 8) * 2;
      return lds_asm_read16<off>((ks & 1) ? od_addr : ev_addr);
    };

    // the first fragments of step 0 (zeros)
    {
      const unsigned sT = prev_slot(prev_slot(sA)) * SLOT;
      static_for<0, AHEAD>([&](auto m_c) __attribute__((always_inline)) {
        fr[decltype(m_c)::value] = load_t(t_lo0 + sT, t_hi0 + sT, m_c);
      });
    }

    using Lds = DkvLdsOrder<ROLE, NF, 2 * DB>;  // the waits for LDS data (see there)
    auto step = [&](int g, f32x16 (&cur)[2], f32x16 (&nxt)[2], bf16x8 (&f_old)[2][2],
                    bf16x8 (&f_new)[2][2]) __attribute__((always_inline)) {
      const int sR = prev_slot(sA), sT = prev_slot(sR);
      const unsigned oA = sA * SLOT, oR = sR * SLOT, oT = sT * SLOT;
      const unsigned t_lo = t_lo0 + oT, t_hi = t_hi0 + oT, a_ev = a_ev0 + oA, a_od = a_od0 + oA;
      const unsigned n_lo = t_lo0 + oR, n_hi = t_hi0 + oR;
      if (ROLE == 0) {
        // entry (query 8 (i / 4) + 4 hh + i % 4 of the tile, column of block kb) is visible iff 8 (i / 4) + i % 4 >= lim[kb]
        const bool valid = g < n_iter;
        if (__builtin_expect(!valid || s_qt * BM < jrel_hi, 0)) {  // rare: keep it out of the loop's straight line
          const int lim0 = valid ? jrel - s_qt * BM - 4 * hh : 0x40000000;
          const int lim1 = valid ? lim0 + 32 : 0x40000000;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            mask_c[0][i] = 8 * (i >> 2) + (i & 3) < lim0 ? -INFINITY : 0.f;
            mask_c[1][i] = 8 * (i >> 2) + (i & 3) < lim1 ? -INFINITY : 0.f;
          }
          mask_set = true;
        } else if (__builtin_expect(mask_set, 0)) {
          mask_c[0] = zero16;
          mask_c[1] = zero16;
          mask_set = false;
        }
      }
      // hand-over and row values are issued between the MFMAs of the first mini-steps, so that the matrix pipe restarts
      // right after the barrier; the vector work starts at mini-step 4
      bf16x8 ph[2][2];
      f32x4 r4[4];  // LSE (role A) or -D (role B) of rows 8 g4 + 4 hh + 0..3
      const unsigned pa = pex0 + (ROLE == 0 ? (g & 1) : ((g & 1) ^ 1)) * (PS * 2);
      const unsigned ra = rv0 + sR * (RV * 4);
      unsigned pw[2][8];
      float e_hold[2];  // role A: exponentials of the previous pair (converted one mini-step later: a transcendental
                        // result cannot be consumed by the very next instruction)
      // vector work of score 2 dw + q of block kb (pair j = 8 kb + dw), pinned to where it is written (the compiler
      // would gather the vector work elsewhere)
      auto vec_half = [&](auto j_c, auto q_c) __attribute__((always_inline)) {
        constexpr int j = decltype(j_c)::value, q = decltype(q_c)::value;
        constexpr int kb = j >> 3, dw = j & 7, i = 2 * dw + q;
        if (ROLE == 0) {
          if constexpr (j > 0 && q == 0) {  // the previous pair's exponentials
            bf16x2 w;
            w[0] = (__bf16)e_hold[0]; w[1] = (__bf16)e_hold[1];
            unsigned wu = __builtin_bit_cast(unsigned, w);
            asm volatile("" : "+v"(wu));
            pw[(j - 1) >> 3][(j - 1) & 7] = wu;
          }
          e_hold[q] = __builtin_amdgcn_exp2f(cur[kb][i] * c - r4[i >> 2][i & 3]);
          asm volatile("" : "+v"(e_hold[q]));
        } else {
          const float e = (float)ph[kb][i >> 3][i & 7] * (cur[kb][i] + r4[i >> 2][i & 3]);  // r4 = -D
          if constexpr (q == 0) {
            e_hold[0] = e;
            asm volatile("" : "+v"(e_hold[0]));
          } else {
            bf16x2 w;
            w[0] = (__bf16)e_hold[0]; w[1] = (__bf16)e;
            unsigned wu = __builtin_bit_cast(unsigned, w);
            asm volatile("" : "+v"(wu));
            pw[kb][dw] = wu;
          }
        }
      };
      auto vec_pair = [&](auto j_c) __attribute__((always_inline)) {
        vec_half(j_c, std::integral_constant<int, 0>{});
        vec_half(j_c, std::integral_constant<int, 1>{});
      };
      asm volatile("s_nop 7" ::: "memory");
      __builtin_amdgcn_sched_barrier(0);
      static_for<0, NF>([&](auto m_c) __attribute__((always_inline)) {
        constexpr int m = decltype(m_c)::value;
        {  // wait for fragment m (and, in mini-step 4, for the hand-over and the row values)
          constexpr int lgkm = Lds::wait(m);
          static_assert(lgkm >= 0 && lgkm <= 15, "lgkmcnt is a 4-bit counter");
          if constexpr (m == 4) {
            if (ROLE == 0)
              asm volatile("s_waitcnt lgkmcnt(%5)" : "+v"(fr[m & 7]), "+v"(r4[0]), "+v"(r4[1]), "+v"(r4[2]), "+v"(r4[3]) : "n"(lgkm));
            else
              asm volatile("s_waitcnt lgkmcnt(%9)" : "+v"(fr[m & 7]), "+v"(r4[0]), "+v"(r4[1]), "+v"(r4[2]), "+v"(r4[3]),
                           "+v"(ph[0][0]), "+v"(ph[0][1]), "+v"(ph[1][0]), "+v"(ph[1][1]) : "n"(lgkm));
          } else {
            asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(fr[m & 7]) : "n"(lgkm));
          }
        }
        {  // read the fragment of mini-step m + AHEAD (past the end: the next step's first transposed fragments)
          constexpr int mm = m + AHEAD;
          if constexpr (mm < 2 * DB) fr[mm & 7] = load_t(t_lo, t_hi, std::integral_constant<int, mm>{});
          else if constexpr (mm < NF) fr[mm & 7] = load_a(a_ev, a_od, std::integral_constant<int, mm - 2 * DB>{});
          else fr[mm & 7] = load_t(n_lo, n_hi, std::integral_constant<int, mm - NF>{});
        }
        const bf16x8 fa = fr[m & 7];
        // S / dP live in vector registers (the vector work reads them directly) and K / V fragments in accumulation
        // registers; written as opaque instructions since the compiler keeps every MFMA result of a kernel with more
        // than 256 registers in accumulation registers.  Their results are first read one step later.
        auto mma = [&](auto kb_c) __attribute__((always_inline)) {
          constexpr int kb = decltype(kb_c)::value;
          if constexpr (m < 2 * DB) {
            constexpr int ks = m / DB, db = m % DB;
            acc[kb][db] = mfma32(fa, f_old[kb][ks], acc[kb][db]);
          } else {
            constexpr int ks = m - 2 * DB;
            if (ks == 0 && ROLE == 0)
              asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(nxt[kb]) : "v"(fa), "a"(bfrag[kb][ks]), "v"(mask_c[kb]));
            else if (ks == 0)
              asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(nxt[kb]) : "v"(fa), "a"(bfrag[kb][ks]));
            else
              asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(nxt[kb]) : "v"(fa), "a"(bfrag[kb][ks]));
          }
        };
        // The mini-step's two MFMAs are kept apart by half of its other work: issued back to back, the second one would
        // hold up the wave (the only one on this SIMD) until the first has left the matrix pipe.
        constexpr std::integral_constant<int, 0> c0{};
        constexpr std::integral_constant<int, 1> c1{};
        mma(c0);
        // hand-over and row values (DkvLdsOrder: E0)
        if constexpr (ROLE == 0) {
          if constexpr (m < 4) lds_asm_write16<1024 * m>(pa, f_old[m >> 1][m & 1]);
        } else {
          if constexpr (m == 0) {
            ph[0][0] = lds_asm_read16<0>(pa);
            ph[0][1] = lds_asm_read16<1024>(pa);
            ph[1][0] = lds_asm_read16<2048>(pa);
            ph[1][1] = lds_asm_read16<3072>(pa);
          }
          if constexpr (m == 1) {
            r4[0] = lds_asm_read16f<0>(ra);
            r4[1] = lds_asm_read16f<32>(ra);
            r4[2] = lds_asm_read16f<64>(ra);
            r4[3] = lds_asm_read16f<96>(ra);
          }
        }
        if (m == 2 && ROLE == 0) dma_rows();
        // Vector work next to the MFMAs: one pair (two scores of a key block) after each MFMA of the second half of the
        // step; the MFMAs of the first half run unhindered.  Measured for role A (fma + exponential) against an even
        // spread over the whole step (2.1 % slower), one score per MFMA from mini-step 4 on and two in the last four
        // mini-steps (0.5 - 1 % slower) and everything in the last four mini-steps (9.6 % slower); for role B against
        // the second of these (1.2 % slower).
        if constexpr (m >= 8) vec_pair(std::integral_constant<int, 2 * (m - 8)>{});
        __builtin_amdgcn_sched_barrier(0);
        mma(c1);
        if constexpr (ROLE == 0 && m < 2) {  // (E1)
          r4[2 * m] = lds_asm_read16f<64 * m>(ra);
          r4[2 * m + 1] = lds_asm_read16f<64 * m + 32>(ra);
        }
        if (m >= 3 && m < 3 + 2 * PIECES && ((m - 3) & 1) == 0) dma_piece((m - 3) >> 1);
        if constexpr (m >= 8) vec_pair(std::integral_constant<int, 2 * (m - 8) + 1>{});
        if constexpr (m == 14) {  // bookkeeping for the next step (the copies of this step have been issued)
          dma_advance();
          sA = sA == NS - 1 ? 0 : sA + 1;
          if (ROLE == 0 && --s_heads == 0) {
            s_heads = G;
            s_qt += down ? -1 : 1;
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      });
      if (ROLE == 0) {
        bf16x2 w;
        w[0] = (__bf16)e_hold[0]; w[1] = (__bf16)e_hold[1];
        pw[1][7] = __builtin_bit_cast(unsigned, w);
      }
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          u32x4 v = {pw[kb][4 * ks], pw[kb][4 * ks + 1], pw[kb][4 * ks + 2], pw[kb][4 * ks + 3]};
          f_new[kb][ks] = __builtin_bit_cast(bf16x8, v);
        }
      // Stage g + 1 must have landed; the copies of the DIST - 1 stages after it may still be in flight.  This wave's
      // hand-over stores completed long ago (mini-step 4 waited for them).
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((DIST - 1) * CPS) : "memory");
      wg_barrier();
    };
    // role A's last product is dV^T of stage n - 1 in step n + 1, role B's dK^T of stage n - 1 in step n + 3
    const int n_steps = n_iter + 4;
    const int claim_at = max(0, n_steps - 4) & ~1;  // the step pair before which wave 0 claims the next block
    for (int g = 0; g < n_steps; g += 2) {
      if (g == claim_at && wave == 0) pending_claim = block_claim_issue(p.taken, xcd);
      step(g, x[0], x[1], f[0], f[1]);
      step(g + 1, x[1], x[0], f[1], f[0]);
    }
    // every copy of this wave has landed (the last ones rewrote a slot nobody reads): once all waves have met at the
    // barrier that hands out the next block, the ring may be filled again
    __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)

    // ---- epilogue: dV = dV^T (role A), dK = scale * dK^T (role B), written (or added) as bf16 ----
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const int kr = 64 * pair + 32 * kb + l32;
      if (kr < it.kv_rows) {
        const int64_t off = ((int64_t)it.kv_row0 + kr) * kv_stride + (int64_t)kvh * D;
        __bf16* const out = ROLE ? p.dk : p.dv;
        const float fs = ROLE ? p.scale : 1.0f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            dkv_store4(p, out, off + 32 * db + 8 * g + 4 * hh, acc[kb][db][4 * g] * fs, acc[kb][db][4 * g + 1] * fs,
                       acc[kb][db][4 * g + 2] * fs, acc[kb][db][4 * g + 3] * fs);
          }
      }
    }
  };
  if (role == 0) body(std::integral_constant<int, 0>{});
  else body(std::integral_constant<int, 1>{});
  // on to the next block; the stores of the epilogue are not waited for here
  int nb = 0;
  if (wave == 0) {
    if (lane == 0) __hip_atomic_fetch_add(p.ended + (blk & 7), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    nb = block_claim_finish(p.taken, num_blocks, xcd, pending_claim);
    start_in_step(nb);
  }
  blk = broadcast_from_wave0(&next_block, nb);
  }
  clock_log_stamp(p.clock_log, 1);
}

// ------------------------------------------------------------------------------------------------
// bwd_dq_pipe (head_dim 128)
//
// The dQ kernel in the style of bwd_dkv_pipe_kernel: one wave per SIMD, a workgroup of 4 waves, each wave
// owning two 32-row query blocks ("units": the workgroup's 8 units are the same (head, row block) pairs the
// 8 waves of bwd_dq_kernel take), so that every K / V fragment read from LDS feeds two MFMAs.  Stage t is
// the t-th 32-key tile of the segment; in step t a wave runs
//     dP^T(t) = V(t) dO^T        S^T(t+1) = K(t+1) Q^T        dQ^T += K(t-1)^T dS^T(t-1)      (matrix pipe)
//     P^T(t) = exp2(S^T(t) c - LSE)  and, once dP^T(t) is complete,  dS^T(t) = P^T(t) (dP^T(t) - D)   (vector)
// as 24 mini-steps of one LDS operand fragment and the two MFMAs it feeds (one per unit), each MFMA followed
// by its share of the vector work.  K^T is read from the K tile itself with the LDS transpose read (tiles
// are stored chunk-major as in the dK/dV kernels), so no transposed image of K is needed.  K and V tiles
// live in a ring of DIST + 3 slots.  Steps whose tile needs the causal mask (the last one or two of the
// walk) or lies past the end run a second variant of the step that masks in the vector work.
// ------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256, 1) void bwd_dq_pipe_kernel(DqParams p, int num_blocks) {
  constexpr int NW = 4;        // waves
  constexpr int BN = 32;       // key rows per stage
  constexpr int KC = D / 8;    // 16-byte chunks per K / V row
  constexpr int DK = D / 16;   // k-steps over the head dimension
  constexpr int DB = D / 32;   // 32-row blocks of dQ^T
  constexpr int KT = BN * D;   // elements per tile
  constexpr int DIST = DQ_PIPE_DIST;  // stages copied ahead
  constexpr int NS = DIST + 3; // ring slots: stages t - 1 .. t + 1 in use, t + 2 .. t + 1 + DIST on their way
  constexpr int NF = 2 * DK + 2 * DB;  // operand fragments (mini-steps) per step: V rows, K rows, K^T
  constexpr int AHEAD = 4;             // fragments in flight
  constexpr int NP = BN * KC / 64;     // 64-slot pieces per tile
  constexpr int PER = 2 * NP / NW;     // global->LDS copies per wave and stage
  static_assert(D == 128 && NF == 24 && PER == 4, "the mini-step schedule below is written for head_dim 128");

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  lds_bf16* const L = (lds_bf16*)smem;
  constexpr int K_OFF = 0;               // [NS][KT]  K rows of stage n in slot n % NS (chunk-major)
  constexpr int V_OFF = K_OFF + NS * KT; // [NS][KT]  V rows
  // [NW][64][D] staging of a wave's 64 rows of dQ on their way out, rows of 16-byte chunks, swizzled (tile_elem<KC>):
  // global memory is then written in whole rows (four per instruction) instead of 32 rows with 16 bytes each, which
  // costs the address unit several times as long.  Its first word doubles as the slot through which wave 0 announces
  // the next block, between the last read of one block and the first write of the next.
  constexpr int ST_OFF = V_OFF + NS * KT;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hh = lane >> 5;
  int* const next_block = (int*)((__bf16*)smem + ST_OFF);

  // The workgroup is persistent: it claims one block (work item x key/value head x head split) after the other
  // (device_common.hpp) until none is left.  The next block is claimed before the current one's last few steps: early
  // enough for the answer to arrive by the time it is needed, and not earlier (that would fix the order of the blocks
  // before it is known which workgroup is free first).
  const int xcd = xcd_of_this_wave();
  clock_log_stamp(p.clock_log, 0);
  int blk = 0;
  if (wave == 0) blk = block_claim_finish(p.taken, num_blocks, xcd, block_claim_issue(p.taken, xcd));
  blk = broadcast_from_wave0(next_block, blk);
  while (blk >= 0) {
  wg_barrier();  // every wave has read the announcement: the staging area may be written again
  const int inner_n = p.num_kv_heads * p.head_splits;
  const int inner = blk % inner_n;
  const DqItem it = p.items[blk / inner_n];
  const int kvh = inner % p.num_kv_heads, hs = inner / p.num_kv_heads;
  int head[2], row0[2];  // of the wave's two units
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int unit = 2 * wave + u;
    head[u] = kvh * p.group + hs * p.heads_per_wg + unit % p.heads_per_wg;
    row0[u] = (unit / p.heads_per_wg) * 32;
  }

  const int n_wg = it.n0 + it.q_rows - 1;    // keys visible to the last valid row
  const int nt = (n_wg + BN - 1) / BN;       // stages

  const int64_t q_stride = (int64_t)p.num_q_heads * D, kv_stride = (int64_t)p.num_kv_heads * D;
  const __bf16* __restrict__ Kg = p.k + (int64_t)it.kv_row0 * kv_stride + (int64_t)kvh * D;
  const __bf16* __restrict__ Vg = p.v + (int64_t)it.kv_row0 * kv_stride + (int64_t)kvh * D;

  // the ring slots the prologue does not fill are read before anything is copied into them (K(-1) in step 0)
  {
    bf16x8 z;
#pragma unroll
    for (int i = 0; i < 8; ++i) z[i] = (__bf16)0.0f;
    for (int x = tid; x < (NS - DIST - 1) * KT / 8; x += NW * 64) {
      lds_store8(L + K_OFF + (DIST + 1) * KT + x * 8, z);
      lds_store8(L + V_OFF + (DIST + 1) * KT + x * 8, z);
    }
  }

  // ---- staging: the 2 NP pieces of a stage (NP of K, then NP of V) are dealt to the waves round robin; a piece is
  // 64 consecutive slots of a chunk-major tile = two chunk columns of 32 rows.  Past the last stage the last one is
  // copied again (into a slot nobody reads for anything that counts). ----
  unsigned v_full[PER], v_last[PER];  // byte offset of the lane's chunk from the tile's first row: full tile, last tile
  {
    const int last_row = n_wg - 1 - (nt - 1) * BN;  // rows past the last key repeat it (masked)
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int x = ((i * NW + wave) % NP) * 64 + lane;
      const int off = (x >> 5) * 8, row = (x & 31) ^ (((x >> 5) & 3) << 2);
      v_full[i] = (unsigned)(row * (int)kv_stride + off) * 2u;
      v_last[i] = (unsigned)(min(row, last_row) * (int)kv_stride + off) * 2u;
    }
  }
  int d_t = 0, d_slot = 0;   // stage to copy next (clamped to the last one) and its slot
  int64_t d_off = 0;         // element offset of its first row
  auto dma_piece = [&](int i) __attribute__((always_inline)) {
    const int piece = i * NW + wave;  // wave-uniform; i < NP / NW: a piece of K, else of V
    const unsigned voff = d_t == nt - 1 ? v_last[i] : v_full[i];
    const char* base = reinterpret_cast<const char*>((i < NP / NW ? Kg : Vg) + d_off);
    lds_bf16* dst = L + (i < NP / NW ? K_OFF + piece * 512 : V_OFF + (piece - NP) * 512) + d_slot * KT;
    dma16(base + voff, dst);
  };
  auto dma_advance = [&]() __attribute__((always_inline)) {
    if (d_t + 1 < nt) {
      ++d_t;
      d_off += BN * kv_stride;
    }
    d_slot = d_slot == NS - 1 ? 0 : d_slot + 1;
  };

  // per-lane operand addresses inside a tile (as in the dK/dV kernels)
  int x_off[2], t_off[2];
#pragma unroll
  for (int par = 0; par < 2; ++par) x_off[par] = cm_elem(l32, 2 * par + hh);
  {
    const int j = lane & 15, grp = (lane >> 4) & 1;
    const int cl = 2 * grp + ((j & 3) >> 1);
    const int r0 = 4 * hh + (j >> 2);
#pragma unroll
    for (int half = 0; half < 2; ++half) t_off[half] = cm_elem(r0 + 8 * half, cl) + 4 * (j & 1);
  }
  const unsigned k_ev0 = lds_addr(L + K_OFF + x_off[0]), k_od0 = lds_addr(L + K_OFF + x_off[1]);
  const unsigned v_ev0 = lds_addr(L + V_OFF + x_off[0]), v_od0 = lds_addr(L + V_OFF + x_off[1]);
  const unsigned t_lo0 = lds_addr(L + K_OFF + t_off[0]), t_hi0 = lds_addr(L + K_OFF + t_off[1]);
  constexpr unsigned SLOT = KT * 2;  // bytes per ring slot
  auto load_rows = [&](unsigned ev_addr, unsigned od_addr, auto ks_c) __attribute__((always_inline)) {
    constexpr int ks = decltype(ks_c)::value;
    constexpr int off = (ks >> 1) * (4 * 32 * 8) * 2;
    return lds_asm_read16<off>((ks & 1) ? od_addr : ev_addr);
  };
  auto load_t = [&](unsigned lo_addr, unsigned hi_addr, auto m_c) __attribute__((always_inline)) {
    constexpr int m = decltype(m_c)::value;  // ks2 * DB + db
    constexpr int off = ((m / DB) * (16 * 8) + (m % DB) * (4 * 32 * 8)) * 2;
    const s16x4 lo = lds_asm_read_tr<off>(lo_addr);
    const s16x4 hi = lds_asm_read_tr<off>(hi_addr);
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };

  // prologue: the copies of stages 0 .. DIST first, then the fragments, so that both travel at the same time
#pragma unroll
  for (int s = 0; s <= DIST; ++s) {
#pragma unroll
    for (int i = 0; i < PER; ++i) dma_piece(i);
    dma_advance();
  }
  // Q and dO fragments (B operands): lane holds X[row = l32 of the unit][16 ks + 8 hh ..+7]; LSE and D of that row
  bf16x8 qf[2][DK], gf[2][DK];
  float lse2[2], dsum[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int r_own = min(row0[u] + l32, it.q_rows - 1);  // rows past the tile repeat the last one (never stored)
    const int64_t off = (int64_t)(it.q_row0 + r_own) * q_stride + (int64_t)head[u] * D + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) {
      qf[u][ks] = *reinterpret_cast<const bf16x8*>(p.q + off + 16 * ks);
      gf[u][ks] = *reinterpret_cast<const bf16x8*>(p.d_o + off + 16 * ks);
    }
    const int64_t slot = (int64_t)head[u] * p.total_q_tiles * 64 + it.q_slot0 + r_own;
    lse2[u] = p.lse2p[slot];
    dsum[u] = p.dsp[slot];
  }
  // -D of the unit's row in every element of a tile: the accumulation of dP^T starts from it, so that the vector work
  // gets dP - D straight from the matrix pipe (a column of dP^T belongs to one query row)
  f32x16 dneg[2];
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int i = 0; i < 16; ++i) dneg[u][i] = dsum[u];
  // One wait the compiler can see for everything issued so far (loads complete in order: the copies have landed when
  // the fragments have), so that it puts no full waits for outstanding loads into the loop
  __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
  wg_barrier();

  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 dq[2][DB];
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int db = 0; db < DB; ++db) dq[u][db] = zero16;
  f32x16 x[2][2];   // S^T: [buffer][unit]
  f32x16 dp[2];     // dP^T: [unit]
  bf16x8 f[2][2][2];  // dS^T as B operands: [buffer][unit][k-step]
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int i = 0; i < 8; ++i) f[b][u][ks][i] = (__bf16)0.0f;
  const float c = p.scale_log2;
  bf16x8 fr[8];  // ring of operand fragments

  // S^T(0) = K(0) Q^T, then the first fragments of step 0 (V rows of stage 0)
  {
    bf16x8 a[DK];
    static_for<0, DK>([&](auto ks_c) __attribute__((always_inline)) { a[decltype(ks_c)::value] = load_rows(k_ev0, k_od0, ks_c); });
    static_for<0, AHEAD>([&](auto ks_c) __attribute__((always_inline)) { fr[decltype(ks_c)::value] = load_rows(v_ev0, v_od0, ks_c); });
    asm volatile("s_waitcnt lgkmcnt(%8)" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7]) : "n"(AHEAD));
#pragma unroll
    for (int ks = 0; ks < DK; ++ks)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        if (ks == 0) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(x[0][u]) : "v"(a[ks]), "a"(qf[u][ks]));
        else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(x[0][u]) : "v"(a[ks]), "a"(qf[u][ks]));
      }
    mfma_settle();
  }

  // In program order mini-step m reads fragment m + 4: one instruction for the rows fragments (0 .. 15 of this step,
  // 0 .. 3 of the next), two for the transposed ones (16 .. 23).  lgkm_wait(m) = number of LDS instructions between the
  // read of fragment m and the start of mini-step m, where the wait stands.
  auto lgkm_wait = [](int m) {
    constexpr int tab[24] = {3, 3, 3, 3, 3, 3, 3, 3, 3, 3, 3, 3, 3, 4, 5, 6, 6, 6, 6, 6, 6, 5, 4, 3};
    return tab[m];
  };
  int sV = 0;  // slot of stage t
  auto step = [&](int t, f32x16 (&cur)[2], f32x16 (&nxt)[2], bf16x8 (&f_old)[2][2], bf16x8 (&f_new)[2][2],
                  auto masked_c) __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(masked_c)::value;
    const int sK = sV == NS - 1 ? 0 : sV + 1;   // stage t + 1
    const int sM = sV == 0 ? NS - 1 : sV - 1;   // stage t - 1
    const unsigned v_ev = v_ev0 + sV * SLOT, v_od = v_od0 + sV * SLOT, k_ev = k_ev0 + sK * SLOT, k_od = k_od0 + sK * SLOT;
    const unsigned t_lo = t_lo0 + sM * SLOT, t_hi = t_hi0 + sM * SLOT, n_ev = v_ev0 + sK * SLOT, n_od = v_od0 + sK * SLOT;
    // MASKED: element i (key 8 (i / 4) + 4 hh + i % 4 of the tile) of unit u is visible iff 8 (i / 4) + i % 4 < lim[u]
    int lim[2];
    if (MASKED) {
#pragma unroll
      for (int u = 0; u < 2; ++u) lim[u] = t < nt ? it.n0 + row0[u] + l32 - BN * t - 4 * hh : -0x40000000;
    }
    float pf[2][16];   // P^T(t)
    unsigned pw[2][8]; // dS^T(t), packed pairs
    auto exp_half = [&](auto j_c, auto q_c) __attribute__((always_inline)) {  // P of element 2 dw + q of unit u (pair j = 8 u + dw)
      constexpr int j = decltype(j_c)::value, q = decltype(q_c)::value;
      constexpr int u = j >> 3, i = 2 * (j & 7) + q;
      float tt = cur[u][i] * c - lse2[u];
      if (MASKED) {
        if (8 * (i >> 2) + (i & 3) >= lim[u]) tt = -INFINITY;
      }
      pf[u][i] = __builtin_amdgcn_exp2f(tt);
      asm volatile("" : "+v"(pf[u][i]));  // pinned here (the compiler would gather the vector work elsewhere)
    };
    auto ds_pair = [&](auto j_c) __attribute__((always_inline)) {
      constexpr int j = decltype(j_c)::value;
      constexpr int u = j >> 3, dw = j & 7;
      bf16x2 w;
      w[0] = (__bf16)(pf[u][2 * dw] * dp[u][2 * dw]);  // dp holds dP - D: its accumulation starts from -D
      w[1] = (__bf16)(pf[u][2 * dw + 1] * dp[u][2 * dw + 1]);
      unsigned wu = __builtin_bit_cast(unsigned, w);
      asm volatile("" : "+v"(wu));
      pw[u][dw] = wu;
    };
    asm volatile("s_nop 7" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    static_for<0, NF>([&](auto m_c) __attribute__((always_inline)) {
      constexpr int m = decltype(m_c)::value;
      asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(fr[m & 7]) : "n"(lgkm_wait(m)));
      {  // read the fragment of mini-step m + AHEAD (past the end: the next step's first V fragments)
        constexpr int mm = m + AHEAD;
        if constexpr (mm < DK) fr[mm & 7] = load_rows(v_ev, v_od, std::integral_constant<int, mm>{});
        else if constexpr (mm < 2 * DK) fr[mm & 7] = load_rows(k_ev, k_od, std::integral_constant<int, mm - DK>{});
        else if constexpr (mm < NF) fr[mm & 7] = load_t(t_lo, t_hi, std::integral_constant<int, mm - 2 * DK>{});
        else fr[mm & 7] = load_rows(n_ev, n_od, std::integral_constant<int, mm - NF>{});
      }
      const bf16x8 fa = fr[m & 7];
      // dP^T and S^T are kept in vector registers, the Q / dO fragments in accumulation registers (opaque MFMAs, see
      // bwd_dkv_pipe_kernel); dP^T is first read three mini-steps after its last MFMA, S^T in the next step
      auto mma = [&](auto u_c) __attribute__((always_inline)) {
        constexpr int u = decltype(u_c)::value;
        const bf16x8& a_ = fa;  // (named references: variables used only inside an asm statement are not captured)
        if constexpr (m < DK) {
          f32x16& d_ = dp[u];
          const bf16x8& b_ = gf[u][m];
          const f32x16& n_ = dneg[u];
          if (m == 0) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(d_) : "v"(a_), "a"(b_), "v"(n_));
          else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d_) : "v"(a_), "a"(b_));
        } else if constexpr (m < 2 * DK) {
          constexpr int ks = m - DK;
          f32x16& d_ = nxt[u];
          const bf16x8& b_ = qf[u][ks];
          if (ks == 0) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d_) : "v"(a_), "a"(b_));
          else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d_) : "v"(a_), "a"(b_));
        } else {
          constexpr int ks = (m - 2 * DK) / DB, db = (m - 2 * DK) % DB;
          dq[u][db] = mfma32(fa, f_old[u][ks], dq[u][db]);
        }
      };
      constexpr std::integral_constant<int, 0> c0{};
      constexpr std::integral_constant<int, 1> c1{};
      // exponentials: pair j in mini-step 6 + j (the first six mini-steps are left to the MFMAs alone: measured 1 %
      // faster than starting with mini-step 0, and faster than starting with 2, 4 or 8); dS: pairs 0 .. 11 in
      // mini-steps 10 .. 21, then two per mini-step
      mma(c0);
      if constexpr (m >= 6 && m < 22) exp_half(std::integral_constant<int, m - 6>{}, c0);
      if constexpr (m >= 10 && m < 22) ds_pair(std::integral_constant<int, m - 10>{});
      if constexpr (m >= 22) ds_pair(std::integral_constant<int, 12 + 2 * (m - 22)>{});
      __builtin_amdgcn_sched_barrier(0);
      mma(c1);
      if constexpr (m >= 6 && m < 22) exp_half(std::integral_constant<int, m - 6>{}, c1);
      if constexpr (m >= 3 && m < 3 + 2 * PER && ((m - 3) & 1) == 0) dma_piece((m - 3) >> 1);
      if constexpr (m >= 22) ds_pair(std::integral_constant<int, 13 + 2 * (m - 22)>{});
      if constexpr (m == 12) {  // bookkeeping for the next step (this step's copies have been issued)
        dma_advance();
        sV = sK;
      }
      __builtin_amdgcn_sched_barrier(0);
    });
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        u32x4 v = {pw[u][4 * ks], pw[u][4 * ks + 1], pw[u][4 * ks + 2], pw[u][4 * ks + 3]};
        f_new[u][ks] = __builtin_bit_cast(bf16x8, v);
      }
    // stage t + 2 must have landed; the copies of the DIST - 1 stages after it may still be in flight
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((DIST - 1) * PER) : "memory");
    wg_barrier();
  };

  // Steps are taken two at a time (the two S^T buffers and the two dS^T buffers swap roles without a copy): first the
  // pairs whose tiles every row of the wave sees completely, then the rest with the mask, up to step nt (whose only
  // real work is the dQ^T product of the last tile); a pair may run one step past that, which contributes nothing.
  const int t_full = min(nt, (it.n0 + min(row0[0], row0[1])) / BN) & ~1;
  int t = 0;
  for (; t < t_full; t += 2) {
    step(t, x[0], x[1], f[0], f[1], std::false_type{});
    step(t + 1, x[1], x[0], f[1], f[0], std::false_type{});
  }
  int pending_claim = 0;
  if (wave == 0) pending_claim = block_claim_issue(p.taken, xcd);
  for (; t <= nt; t += 2) {
    step(t, x[0], x[1], f[0], f[1], std::true_type{});
    step(t + 1, x[1], x[0], f[1], f[0], std::true_type{});
  }

  // every copy of this wave has landed (the last ones rewrote a slot nobody reads): after the barrier below the next
  // block may fill the ring again
  __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
  // ---- epilogue: dQ = scale * dQ^T, through the wave's staging tile (one unit after the other) ----
  lds_bf16* const stage = L + ST_OFF + wave * (64 * D);
  // (the lane index is made opaque here: the addresses below depend on nothing else, and computed ahead of the loop
  // they would take registers the loop has no room for)
  int lane_e = lane;
  asm volatile("" : "+v"(lane_e));
  const int l32_e = lane_e & 31, hh_e = lane_e >> 5;
#pragma unroll
  for (int u = 0; u < 2; ++u) {
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const bf16x4 v = pack4(dq[u][db][4 * g] * p.scale, dq[u][db][4 * g + 1] * p.scale, dq[u][db][4 * g + 2] * p.scale,
                               dq[u][db][4 * g + 3] * p.scale);
        *(__attribute__((address_space(3))) bf16x4*)(stage + tile_elem<KC>(32 * u + l32_e, 4 * db + g) + 4 * hh_e) = v;
      }
    __bf16* obase = p.dq + (int64_t)(it.q_row0 + row0[u]) * q_stride + (int64_t)head[u] * D;
#pragma unroll 2
    for (int i = 0; i < 32 * KC / 64; ++i) {
      const int x = (u * 32 * KC / 64 + i) * 64 + lane_e;
      const int row = x / KC, c = unswz<KC>(row, x % KC);  // row of the staging tile: 32 u + row of the unit
      const bf16x8 v = lds_load8(stage + x * 8);
      const int ru = row - 32 * u;
      if (row0[u] + ru < it.q_rows) *reinterpret_cast<bf16x8*>(obase + (int64_t)ru * q_stride + c * 8) = v;
    }
  }
  // on to the next block; the stores above are not waited for here
  int nb = 0;
  if (wave == 0) nb = block_claim_finish(p.taken, num_blocks, xcd, pending_claim);
  blk = broadcast_from_wave0(next_block, nb);
  }
  clock_log_stamp(p.clock_log, 1);
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
size_t up256(size_t x) { return (x + 255) / 256 * 256; }
size_t n_dkv_blocks(const chunk_attn_desc* d) {
  size_t n = 0;
  for (int t = 0; t < d->num_segments; ++t) n += (d->segments[t].kv_len + dkv_keys(d->head_dim) - 1) / dkv_keys(d->head_dim);
  return n;
}

// Raises a kernel's dynamic-LDS limit; callers keep the result in a function-local static, so that it happens once per
// process and is safe from several threads.
template <class K>
hipError_t raise_smem_limit(K kernel, size_t smem) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
}

template <int D>
hipError_t launch_bwd_t(const chunk_attn_desc* d, const BwdArgs& a, const BwdPlan& P, hipStream_t stream) {
  char* ws = a.workspace;
  const TileJob* qjobs = reinterpret_cast<const TileJob*>(ws + P.qjobs_off);
  const TileJob* kjobs = reinterpret_cast<const TileJob*>(ws + P.kjobs_off);
  float* lse2p = reinterpret_cast<float*>(ws + P.lse2p_off);
  float* dsp = reinterpret_cast<float*>(ws + P.dsp_off);
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
  if constexpr (D != 128) {  // the head_dim 128 dQ kernel reads K^T from its K tiles
    if ((e = launch_transpose(a.k, d->num_kv_heads, D, 32, kjobs, (int)P.kjobs.size(), P.kv32_tiles, kt, stream)) != hipSuccess) return e;
  }

  if (!a.accumulate) {  // rows no segment covers receive no gradient
    for (const auto& gap : uncovered_kv_ranges(d)) {
      const int esz = a.dkv_f32 ? 4 : 2;  // bytes per element of dK / dV
      const int64_t n16 = (int64_t)(gap.second - gap.first) * d->num_kv_heads * D * esz / 16;
      for (__bf16* base : {a.dk, a.dv}) {
        u32x4* ptr = reinterpret_cast<u32x4*>(reinterpret_cast<char*>(base) + (int64_t)gap.first * d->num_kv_heads * D * esz);
        hipLaunchKernelGGL(zero_fill_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, stream, ptr, n16);
      }
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
  }

  const int group = d->num_q_heads / d->num_kv_heads;
  if constexpr (D == 128) {
    if (P.fused) return launch_bwd_fused(d, a, P, lse2p, dsp, stream);
  }
  {  // dQ
    DqParams p;
    p.q = a.q; p.k = a.k; p.v = a.v; p.d_o = a.d_o; p.kt = kt; p.lse2p = lse2p; p.dsp = dsp; p.dq = a.dq;
    p.items = reinterpret_cast<const DqItem*>(ws + P.dq_items_off);
    p.total_kv32_tiles = P.kv32_tiles; p.total_q_tiles = P.q_tiles;
    p.num_q_heads = d->num_q_heads; p.num_kv_heads = d->num_kv_heads; p.group = group;
    p.heads_per_wg = heads_per_wg(group, dq_waves(D)); p.head_splits = group / p.heads_per_wg;
    p.scale = d->softmax_scale; p.scale_log2 = d->softmax_scale * kLog2e;
    p.taken = reinterpret_cast<int32_t*>(ws + P.queues_off);
    p.clock_log = clock_log(1);
    const int64_t blocks = (int64_t)P.dq_items.size() * d->num_kv_heads * p.head_splits;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    if constexpr (D == 128) {
      // ring slots of a K and a V tile, then the staging tiles of the four waves (64 rows each)
      const size_t smem = (size_t)2 * (DQ_PIPE_DIST + 3) * 32 * D * 2 + (size_t)4 * 64 * D * 2;
      static const hipError_t attr = raise_smem_limit(&bwd_dq_pipe_kernel<D>, smem);
      if (attr != hipSuccess) return attr;
      hipLaunchKernelGGL((bwd_dq_pipe_kernel<D>), dim3((unsigned)persistent_grid(blocks)), dim3(256), smem, stream, p, (int)blocks);
    } else {
      const size_t smem = (size_t)9 * 32 * D * 2;  // 3 stages of K, V and K^T tiles
      constexpr int DQW = 4;
      static const hipError_t attr = raise_smem_limit(&bwd_dq_kernel<D, DQW>, smem);
      if (attr != hipSuccess) return attr;
      hipLaunchKernelGGL((bwd_dq_kernel<D, DQW>), dim3((unsigned)blocks), dim3(DQW * 64), smem, stream, p);
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  {  // dK, dV
    DkvParams p;
    p.q = a.q; p.k = a.k; p.v = a.v; p.d_o = a.d_o; p.lse2p = lse2p; p.dsp = dsp;
    p.dk = a.dk; p.dv = a.dv;
    p.items = reinterpret_cast<const DkvItem*>(ws + P.dkv_items_off);
    p.total_q_tiles = P.q_tiles;
    p.num_q_heads = d->num_q_heads; p.num_kv_heads = d->num_kv_heads; p.group = group;
    p.scale = d->softmax_scale; p.scale_log2 = d->softmax_scale * kLog2e;
    p.accumulate = a.accumulate ? 1 : 0;
    p.out_f32 = a.dkv_f32 ? 1 : 0;
    p.taken = reinterpret_cast<int32_t*>(ws + P.queues_off) + kBlockQueues;
    p.ended = p.taken + kBlockQueues;
    p.side_by_side = std::max(1, persistent_grid(0x7fffffff) / kBlockQueues);
    p.clock_log = clock_log(2);
    static_assert(DKV_KEYS == 128, "the head_dim 64 and 128 kernels cover 128 keys per workgroup");
    const int64_t blocks = (int64_t)P.dkv_items.size() * d->num_kv_heads;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    ProfileEvents pe = profile_events();
    profile_events() = ProfileEvents{};
    if constexpr (D == 128) {
      // ring slots of two 32-row operand tiles, 2 P hand-over slots, one slot of LSE and D rows per ring slot
      constexpr int NS = DKV_PIPE_DIST + 5;
      const size_t smem = (size_t)2 * NS * 32 * D * 2 + 2 * 4096 * 2 + 2 * NS * 64 * sizeof(float);
      static const hipError_t attr = raise_smem_limit(&bwd_dkv_pipe_kernel<D>, smem);
      if (attr != hipSuccess) return attr;
      if (pe.start && (e = hipEventRecord(pe.start, stream)) != hipSuccess) return e;
      hipLaunchKernelGGL((bwd_dkv_pipe_kernel<D>), dim3((unsigned)persistent_grid(blocks)), dim3(256), smem, stream, p, (int)blocks);
    } else {
      // 4 ring slots of two 32-row operand tiles, 2 P hand-over slots, 4 slots of LSE and D rows
      constexpr int KB = (D > 128 ? 64 : DKV_KEYS) / 32;   // as dkv_keys(D)
      const size_t smem = (size_t)8 * 32 * D * 2 + 2 * KB * 1024 * 2 + 2 * 4 * 64 * sizeof(float);
      static const hipError_t attr = raise_smem_limit(&bwd_dkv_kernel<D, KB>, smem);
      if (attr != hipSuccess) return attr;
      if (pe.start && (e = hipEventRecord(pe.start, stream)) != hipSuccess) return e;
      hipLaunchKernelGGL((bwd_dkv_kernel<D, KB>), dim3((unsigned)blocks), dim3(KB * 128), smem, stream, p);
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (pe.stop && (e = hipEventRecord(pe.stop, stream)) != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace

void bwd_layout(const chunk_attn_desc* d, BwdPlan& P, bool with_plan) {
  const int group = d->num_q_heads / d->num_kv_heads;
  const int dq_rows = tile_rows(group, dq_waves(d->head_dim));
  P.q_tiles = count_tiles(d, false, 64);
  P.kv32_tiles = count_tiles(d, true, 32);
  P.qt32_tiles = count_tiles(d, false, 32);
  P.fused = d->head_dim == 128 && bwd_mode() == 2;
  size_t n_dq = 0, n_dkv = 0;
  if (with_plan) {
    if (P.fused) {
      P.fplan = plan_fused(d, dkv_keys(d->head_dim), kNumXcd, fused_num_bufs(d, dkv_keys(d->head_dim)));
    } else {
      P.dq_items = plan_dq(d, dq_rows);
      // head_dim 128: the pipelined kernel walks either way; the key blocks of one key/value head that run at the same time
      // are the workgroups of the launch (one per CU) over the number of key/value heads
      const int side_by_side = d->head_dim == 128 ? std::max(1, persistent_grid(0x7fffffff) / d->num_kv_heads) : 0;
      P.dkv_items = plan_dkv(d, dkv_keys(d->head_dim), side_by_side);
    }
    P.qjobs = tile_jobs(d, false, 64, nullptr);
    P.kjobs = tile_jobs(d, true, 32, nullptr);
  }
  // the layout does not depend on which backward runs: item counts follow from the segment table
  for (int t = 0; t < d->num_segments; ++t) {
    n_dq += (d->segments[t].q_len + dq_rows - 1) / dq_rows;
    n_dkv += (d->segments[t].kv_len + dkv_keys(d->head_dim) - 1) / dkv_keys(d->head_dim);
  }
  P.dq_items_off = 0;
  P.dkv_items_off = up256(n_dq * sizeof(DqItem));
  P.qjobs_off = P.dkv_items_off + up256(n_dkv * sizeof(DkvItem));
  P.kjobs_off = P.qjobs_off + up256((size_t)P.q_tiles * sizeof(TileJob));
  P.fitems_off = P.kjobs_off + up256((size_t)P.kv32_tiles * sizeof(TileJob));
  // the workspace is sized for either backward (the mode may change between the size query and the call): the one-pass
  // backward has one item per (key block, key/value head) and at most 8 x that many workgroup slots
  const size_t n_fused = d->head_dim == 128 ? n_dkv_blocks(d) * (size_t)d->num_kv_heads : 0;
  P.forder_off = P.fitems_off + up256(n_fused * sizeof(FusedItem));
  P.q32jobs_off = P.forder_off + up256(n_fused * kNumXcd * sizeof(int32_t));
  // block-queue counters of the dQ and of the dK/dV kernel (zero in the blob)
  P.queues_off = P.q32jobs_off + (d->head_dim == 128 ? up256((size_t)P.qt32_tiles * sizeof(DqTileJob)) : 0);
  P.blob_bytes = P.queues_off + up256(3 * kBlockQueues * sizeof(int32_t));  // dQ queues, dK/dV queues, dK/dV blocks ended
  const size_t row_slots = (size_t)d->num_q_heads * P.q_tiles * 64;
  P.fprog_off = P.blob_bytes;
  // progress counters, then the status word (its own 256 bytes), then a scratch tile
  P.fprog_bytes = up256(n_fused * 4 * sizeof(unsigned)) + 256 + kFusedSinkBytes;
  P.lse2p_off = P.fprog_off + P.fprog_bytes;
  P.dsp_off = P.lse2p_off + up256(row_slots * sizeof(float));
  P.kt_off = P.dsp_off + up256(row_slots * sizeof(float));
  // transposed K images only for head_dim 64 (the head_dim 128 dQ kernel reads K^T from its K tiles)
  // (256 bytes remain in any case: the dK/dV kernels copy the LSE / D rows 64 at a time, up to 32 past a segment's last)
  P.fdq_off = P.kt_off + (d->head_dim == 128 ? 256 : up256((size_t)d->num_kv_heads * P.kv32_tiles * 32 * d->head_dim * sizeof(__bf16)));
  P.total = P.fdq_off + (d->head_dim == 128 ? (size_t)fused_num_bufs(d, dkv_keys(128)) * d->num_q_heads * P.qt32_tiles * 4096 * sizeof(float) : 0);
}

std::vector<char> bwd_blob(const BwdPlan& P) {
  std::vector<char> blob(P.blob_bytes);
  std::memcpy(blob.data() + P.dq_items_off, P.dq_items.data(), P.dq_items.size() * sizeof(DqItem));
  std::memcpy(blob.data() + P.dkv_items_off, P.dkv_items.data(), P.dkv_items.size() * sizeof(DkvItem));
  std::memcpy(blob.data() + P.qjobs_off, P.qjobs.data(), P.qjobs.size() * sizeof(TileJob));
  std::memcpy(blob.data() + P.kjobs_off, P.kjobs.data(), P.kjobs.size() * sizeof(TileJob));
  if (P.fused) {
    std::memcpy(blob.data() + P.fitems_off, P.fplan.items.data(), P.fplan.items.size() * sizeof(FusedItem));
    std::memcpy(blob.data() + P.forder_off, P.fplan.order.data(), P.fplan.order.size() * sizeof(int32_t));
    std::memcpy(blob.data() + P.q32jobs_off, P.fplan.tiles.data(), P.fplan.tiles.size() * sizeof(DqTileJob));
  }
  return blob;
}

hipError_t launch_bwd(const chunk_attn_desc* d, const BwdArgs& a, const BwdPlan& P, hipStream_t stream) {
  return d->head_dim == 128 ? launch_bwd_t<128>(d, a, P, stream)
         : d->head_dim == 256 ? launch_bwd_t<256>(d, a, P, stream) : launch_bwd_t<64>(d, a, P, stream);
}

}  // namespace chunk_attn
