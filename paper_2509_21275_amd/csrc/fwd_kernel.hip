// Chunk attention forward for gfx950: O = softmax(scale Q K^T + mask) V and LSE, where the mask is the
// chunk mask of the paper's section 3.1 (each segment's queries see their own context and the causal
// part of their own slice; packed sequences see nothing of each other).
//
// A workgroup takes one forward work item -- a tile of query rows of one segment -- for the query heads of
// one group that share a key/value head, and streams that segment's visible keys/values through LDS, copied
// global->LDS without passing through registers.  Scores are computed transposed, S^T = K Q^T, so that after
// the MFMA every lane holds one query column: row maximum and row sum are a loop over the lane's own
// registers plus one exchange with the lane 32 away, and the bf16 probabilities are already laid out as the
// B operand of O^T += V^T P^T (device_common.hpp, "C-order").
//
// Two kernels:
//   fwd_kernel       online softmax with a lazily moved reference maximum, one 32-row query block per wave,
//                    two waves per SIMD, tiles of 64 keys (K row-major, V as the pre-transposed image of
//                    transpose_kernel.hip, double-buffered).  Used for head_dim 64, and for head_dim 128 as the
//                    second pass below.
//   fwd_pipe_kernel  head_dim 128: one wave per SIMD with 64 query rows, software pipelined over stages of 32
//                    keys, reference maximum fixed by the first stage; rows whose scores outgrow it are
//                    flagged and recomputed by fwd_kernel, launched right after over the flagged items only.
#include <type_traits>

#include "kernels.hpp"

#ifndef FWD_PIPE_DIST
#define FWD_PIPE_DIST 3  // stages the pipelined forward copies ahead of the one it computes on
#endif
#include "tiles.hpp"

namespace chunk_attn {

template <int D, int WAVES>
__global__ __launch_bounds__(WAVES * 64, D > 128 ? 1 : 8 / WAVES) void fwd_kernel(FwdParams p) {
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
// Pipelined forward for head_dim 128: one wave per SIMD, 64 query rows per wave (two 32-row "units"), keys
// streamed in stages of 32.
//
// A wave issues at most one instruction every four cycles and an MFMA holds the matrix pipe for 32, so the loop
// is laid out instruction by instruction.  In step t a wave runs
//     O^T += V(t-1)^T P^T(t-1)        S^T(t+1) = K(t+1) Q^T        (matrix pipe)
//     P^T(t) = exp2(S^T(t) c - m c) and its row sums                (vector pipe)
// as 16 mini-steps of one LDS operand fragment and the two MFMAs it feeds (one per unit), each MFMA followed by
// the vector work of one score.  K and V tiles are copied global->LDS into a ring of DIST + 3 slots, stored
// chunk-major; V^T is read from the V tile itself with the LDS transpose read.  Fragments are fetched four
// mini-steps ahead with opaque LDS reads and explicit lgkmcnt waits; S^T lives in vector registers, where the
// vector work reads it directly, the Q fragments and O^T in accumulation registers (tiles.hpp).
// The reference maximum of the softmax is fixed by the first stage, so O^T is never rescaled in the loop; a row
// whose later scores outgrow it raises the workgroup's redo flag and the item is recomputed by fwd_kernel.
// Steps whose stage needs the causal mask (the last few of the walk) or lies past the end run a second variant of
// the step that masks in the vector work.
// ------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256, 1) void fwd_pipe_kernel(FwdParams p, int num_blocks) {
  constexpr int NW = 4;        // waves
  constexpr int BN = 32;       // key rows per stage
  constexpr int KC = D / 8;    // 16-byte chunks per K / V row
  constexpr int DK = D / 16;   // k-steps of S^T = K Q^T
  constexpr int DB = D / 32;   // 32-row blocks of O^T
  constexpr int KT = BN * D;   // elements per tile
  constexpr int DIST = FWD_PIPE_DIST;  // stages copied ahead
  constexpr int NS = DIST + 3; // ring slots: stages t - 1 .. t + 1 in use, t + 2 .. t + 1 + DIST on their way
  constexpr int NF = 2 * DB + DK;      // operand fragments (mini-steps) per step: V^T, then K rows
  constexpr int AHEAD = 4;             // fragments in flight
  constexpr int NP = BN * KC / 64;     // 64-slot pieces per tile
  constexpr int PER = 2 * NP / NW;     // global->LDS copies per wave and stage
  static_assert(D == 128 && NF == 16 && PER == 4, "the mini-step schedule below is written for head_dim 128");

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  lds_bf16* const L = (lds_bf16*)smem;
  constexpr int K_OFF = 0;               // [NS][KT]  K rows of stage n in slot n % NS (chunk-major)
  constexpr int V_OFF = K_OFF + NS * KT; // [NS][KT]  V rows
  // [NW][64][D] staging of a wave's 64 rows of Q on their way in and of O on their way out, rows of 16-byte chunks,
  // swizzled (tile_elem<KC>): global memory is then touched in whole rows (four per instruction) instead of 32 rows
  // with 32 bytes each, which costs the address unit eight times as long.  Its first word doubles as the slot through
  // which wave 0 announces the next block, between the last read of one block and the first copy of the next.
  constexpr int ST_OFF = V_OFF + NS * KT;
  constexpr int ST_ROWS = 64;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hh = lane >> 5;
  __bf16* const stage = (__bf16*)smem + ST_OFF + wave * (ST_ROWS * D);  // this wave's staging tile (generic pointer)
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
  const FwdItem it = p.items[blk / inner_n];
  const int kvh = inner % p.num_kv_heads, hs = inner / p.num_kv_heads;
  const int head = kvh * p.group + hs * p.heads_per_wg + wave % p.heads_per_wg;
  const int wave_row0 = (wave / p.heads_per_wg) * 64;  // the wave's units are rows wave_row0 + 32 u .. + 31 of `head`

  const int n_wg = it.n0 + it.q_rows - 1;    // keys visible to the last valid row
  const int nt = (n_wg + BN - 1) / BN;       // stages

  const int64_t q_stride = (int64_t)p.num_q_heads * D, kv_stride = (int64_t)p.num_kv_heads * D;
  const __bf16* __restrict__ Kg = p.k + (int64_t)it.kv_row0 * kv_stride + (int64_t)kvh * D;
  const __bf16* __restrict__ Vg = p.v + (int64_t)it.kv_row0 * kv_stride + (int64_t)kvh * D;

  // the ring slots the prologue does not fill are read before anything is copied into them (V(-1) in step 0)
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
  // copied again. ----
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

  // per-lane operand addresses inside a tile
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
  const unsigned t_lo0 = lds_addr(L + V_OFF + t_off[0]), t_hi0 = lds_addr(L + V_OFF + t_off[1]);
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

  // prologue: the copies of stages 0 .. DIST first, then the Q fragments, so that both travel at the same time
#pragma unroll
  for (int s = 0; s <= DIST; ++s) {
#pragma unroll
    for (int i = 0; i < PER; ++i) dma_piece(i);
    dma_advance();
  }
  // the wave's 64 rows of Q (its two units) into its staging tile: slot x = 16 row + position holds the chunk that
  // belongs there; rows past the tile repeat the last one (never stored)
  {
    const __bf16* qbase = p.q + (int64_t)it.q_row0 * q_stride + (int64_t)head * D;
#pragma unroll 4
    for (int i = 0; i < ST_ROWS * KC / 64; ++i) {
      const int x = i * 64 + lane;
      const int row = x / KC, c = unswz<KC>(row, x % KC);
      const int r = min(wave_row0 + row, it.q_rows - 1);
      dma16(qbase + (int64_t)r * q_stride + c * 8, stage + i * 512);
    }
  }
  // One wait the compiler can see for everything issued so far: it then has no reason to put full waits for outstanding
  // loads into the loop.
  __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
  // Q fragments (B operands of S^T = K Q^T): lane holds Q[row = l32 of the unit][16 ks + 8 hh ..+7]
  bf16x8 qf[2][DK];
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) qf[u][ks] = lds_chunk<KC>(stage, 32 * u + l32, 2 * ks + hh);
  wg_barrier();

  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 oacc[2][DB];
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int db = 0; db < DB; ++db) oacc[u][db] = zero16;
  f32x16 x[2][2];      // S^T: [buffer][unit]
  bf16x8 f[2][2][2];   // P^T as B operands: [buffer][unit][k-step]
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

  // S^T(0) = K(0) Q^T and the reference maximum of each row; then the first fragments of step 0 (zeros)
  float mc[2], l_run[2];
  {
    bf16x8 a[DK];
    static_for<0, DK>([&](auto ks_c) __attribute__((always_inline)) { a[decltype(ks_c)::value] = load_rows(k_ev0, k_od0, ks_c); });
    {
      const unsigned sT = (NS - 1) * SLOT;
      static_for<0, AHEAD>([&](auto m_c) __attribute__((always_inline)) { fr[decltype(m_c)::value] = load_t(t_lo0 + sT, t_hi0 + sT, m_c); });
    }
    asm volatile("s_waitcnt lgkmcnt(%8)" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7]) : "n"(2 * AHEAD));
#pragma unroll
    for (int ks = 0; ks < DK; ++ks)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        f32x16& d_ = x[0][u];
        const bf16x8& b_ = qf[u][ks];
        if (ks == 0) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d_) : "v"(a[ks]), "a"(b_));
        else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d_) : "v"(a[ks]), "a"(b_));
      }
    mfma_settle();
    asm volatile("s_nop 15" : "+v"(x[0][0]), "+v"(x[0][1]));  // the reads below come after the MFMAs have written
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int lim = it.n0 + wave_row0 + 32 * u + l32;  // stage 0: visible iff local key index < lim (>= 1)
      float mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int j = 8 * (i >> 2) + 4 * hh + (i & 3);
        if (j < lim) mx = fmaxf(mx, x[0][u][i]);
      }
      mc[u] = max_halves(mx) * c;
      l_run[u] = 0.f;
    }
  }
  bool risk = false;
  const float big = __builtin_amdgcn_exp2f(p.ref_limit);

  // In program order mini-step m reads fragment m + 4: two instructions for the transposed fragments (0 .. 7 of this
  // step, 0 .. 3 of the next), one for the rows fragments (8 .. 15).  lgkm_wait(m) = number of LDS instructions between
  // the read of fragment m and the start of mini-step m, where the wait stands.
  auto lgkm_wait = [](int m) {
    constexpr int tab[16] = {6, 6, 6, 6, 6, 5, 4, 3, 3, 3, 3, 3, 3, 4, 5, 6};
    return tab[m];
  };
  int sV = 0;  // slot of stage t
  auto step = [&](int t, f32x16 (&cur)[2], f32x16 (&nxt)[2], bf16x8 (&f_old)[2][2], bf16x8 (&f_new)[2][2],
                  auto masked_c) __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(masked_c)::value;
    const int sK = sV == NS - 1 ? 0 : sV + 1;   // stage t + 1
    const int sM = sV == 0 ? NS - 1 : sV - 1;   // stage t - 1
    const unsigned k_ev = k_ev0 + sK * SLOT, k_od = k_od0 + sK * SLOT;
    const unsigned t_lo = t_lo0 + sM * SLOT, t_hi = t_hi0 + sM * SLOT, n_lo = t_lo0 + sV * SLOT, n_hi = t_hi0 + sV * SLOT;
    // MASKED: element i (key 8 (i / 4) + 4 hh + i % 4 of the stage) of unit u is visible iff 8 (i / 4) + i % 4 < lim[u]
    int lim[2];
    if (MASKED) {
#pragma unroll
      for (int u = 0; u < 2; ++u) lim[u] = t < nt ? it.n0 + wave_row0 + 32 * u + l32 - BN * t - 4 * hh : -0x40000000;
    }
    unsigned pw[2][8];  // P^T(t), packed pairs
    float ps[2] = {0.f, 0.f};
    float e_hold[2];
    // vector work of score 2 dw + q of unit u (pair j = 8 u + dw), pinned to where it is written; a pair is converted
    // one mini-step after its exponentials (a transcendental result cannot be consumed by the very next instruction)
    auto finish_pair = [&](int jp) __attribute__((always_inline)) {
      bf16x2 w;
      w[0] = (__bf16)e_hold[0]; w[1] = (__bf16)e_hold[1];
      // row sums with plain adds: a dot-product instruction next to MFMAs holds the wave up (it costs about as much
      // as 14 cycles of the matrix pipe, an add 1 - 2)
      ps[jp >> 3] += e_hold[0] + e_hold[1];
      asm volatile("" : "+v"(ps[jp >> 3]));
      unsigned wu = __builtin_bit_cast(unsigned, w);
      asm volatile("" : "+v"(wu));
      pw[jp >> 3][jp & 7] = wu;
    };
    auto vec_half = [&](auto j_c, auto q_c) __attribute__((always_inline)) {
      constexpr int j = decltype(j_c)::value, q = decltype(q_c)::value;
      constexpr int u = j >> 3, i = 2 * (j & 7) + q;
      if constexpr (j > 0 && q == 0) finish_pair(j - 1);
      float tt = cur[u][i] * c - mc[u];
      if (MASKED) {
        if (8 * (i >> 2) + (i & 3) >= lim[u]) tt = -INFINITY;
      }
      e_hold[q] = __builtin_amdgcn_exp2f(tt);
      asm volatile("" : "+v"(e_hold[q]));
    };
    asm volatile("s_nop 7" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    static_for<0, NF>([&](auto m_c) __attribute__((always_inline)) {
      constexpr int m = decltype(m_c)::value;
      asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(fr[m & 7]) : "n"(lgkm_wait(m)));
      {  // read the fragment of mini-step m + AHEAD (past the end: the next step's first transposed fragments)
        constexpr int mm = m + AHEAD;
        if constexpr (mm < 2 * DB) fr[mm & 7] = load_t(t_lo, t_hi, std::integral_constant<int, mm>{});
        else if constexpr (mm < NF) fr[mm & 7] = load_rows(k_ev, k_od, std::integral_constant<int, mm - 2 * DB>{});
        else fr[mm & 7] = load_t(n_lo, n_hi, std::integral_constant<int, mm - NF>{});
      }
      const bf16x8 fa = fr[m & 7];
      auto mma = [&](auto u_c) __attribute__((always_inline)) {
        constexpr int u = decltype(u_c)::value;
        if constexpr (m < 2 * DB) {
          constexpr int ks = m / DB, db = m % DB;
          oacc[u][db] = mfma32(fa, f_old[u][ks], oacc[u][db]);
        } else {
          constexpr int ks = m - 2 * DB;
          const bf16x8& a_ = fa;  // (named references: variables used only inside an asm statement are not captured)
          f32x16& d_ = nxt[u];
          const bf16x8& b_ = qf[u][ks];
          if (ks == 0) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d_) : "v"(a_), "a"(b_));
          else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d_) : "v"(a_), "a"(b_));
        }
      };
      constexpr std::integral_constant<int, 0> c0{};
      constexpr std::integral_constant<int, 1> c1{};
      mma(c0);
      vec_half(m_c, c0);
      __builtin_amdgcn_sched_barrier(0);
      mma(c1);
      vec_half(m_c, c1);
      if constexpr (m >= 3 && m < 3 + 2 * PER && ((m - 3) & 1) == 0) dma_piece((m - 3) >> 1);
      if constexpr (m == 12) {  // bookkeeping for the next step (this step's copies have been issued)
        dma_advance();
        sV = sK;
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    finish_pair(15);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      risk |= !(ps[u] < big);
      l_run[u] += ps[u];
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        u32x4 v = {pw[u][4 * ks], pw[u][4 * ks + 1], pw[u][4 * ks + 2], pw[u][4 * ks + 3]};
        f_new[u][ks] = __builtin_bit_cast(bf16x8, v);
      }
    }
    // stage t + 2 must have landed; the copies of the DIST - 1 stages after it may still be in flight
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((DIST - 1) * PER) : "memory");
    wg_barrier();
  };

  // Steps are taken two at a time (the two S^T buffers and the two P^T buffers swap roles without a copy): first the
  // pairs whose stages every row of the wave sees completely, then the rest with the mask, up to step nt (whose only
  // real work is the O^T product of the last stage); a pair may run one step past that, which contributes nothing.
  const int t_full = min(nt, (it.n0 + wave_row0) / BN) & ~1;
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
  if (__any(risk) && lane == 0) {
    p.redo[blk] = 1;
    *p.any_redo = 1;
  }

  // ---- epilogue: O = O^T / l, LSE = ln(l) + m scale ----
  // (through the wave's staging tile: the lane that holds four values of a row writes them there, then every lane
  // moves one 16-byte chunk of a row to global memory, four whole rows per instruction; one unit after the other, so
  // that few values are in flight at a time)
  {
    // (the lane index is made opaque here: the addresses below depend on nothing else, and computed ahead of the loop
    // they would take registers for its whole length)
    int lane_e = lane;
    asm volatile("" : "+v"(lane_e));
    const int l32_e = lane_e & 31, hh_e = lane_e >> 5;
    __bf16* obase = p.o + (int64_t)it.q_row0 * q_stride + (int64_t)head * D;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int r = wave_row0 + 32 * u + l32_e;
      const float l_tot = sum_halves(l_run[u]);
      const float inv = 1.0f / l_tot;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const bf16x4 v = pack4(oacc[u][db][4 * g] * inv, oacc[u][db][4 * g + 1] * inv, oacc[u][db][4 * g + 2] * inv,
                                 oacc[u][db][4 * g + 3] * inv);
          *reinterpret_cast<bf16x4*>(stage + tile_elem<KC>(32 * u + l32_e, 4 * db + g) + 4 * hh_e) = v;
        }
      if (r < it.q_rows && hh_e == 0)
        p.lse[(int64_t)head * p.total_q + it.q_row0 + r] = (mc[u] + log2f(l_tot)) * 0.6931471805599453f;
#pragma unroll 2
      for (int i = 0; i < 32 * KC / 64; ++i) {
        const int x = (u * 32 * KC / 64 + i) * 64 + lane_e;
        const int row = x / KC, c = unswz<KC>(row, x % KC);
        const bf16x8 v = *reinterpret_cast<const bf16x8*>(stage + x * 8);
        if (wave_row0 + row < it.q_rows) *reinterpret_cast<bf16x8*>(obase + (int64_t)(wave_row0 + row) * q_stride + c * 8) = v;
      }
    }
  }
  // on to the next block; the stores above are not waited for here
  int nb = 0;
  if (wave == 0) nb = block_claim_finish(p.taken, num_blocks, xcd, pending_claim);
  blk = broadcast_from_wave0(next_block, nb);
  }
  clock_log_stamp(p.clock_log, 1);
}

// The dynamic-LDS limit of a kernel is raised once per process (thread-safe: a function-local static).
template <class K>
static hipError_t raise_smem_limit(K kernel, size_t smem) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
}

template <int D, int WAVES>
static hipError_t launch_fwd_t(const FwdParams& p, int num_blocks, hipStream_t stream) {
  const size_t smem = (size_t)4 * 64 * D * 2;
  static const hipError_t attr = raise_smem_limit(&fwd_kernel<D, WAVES>, smem);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL((fwd_kernel<D, WAVES>), dim3(num_blocks), dim3(WAVES * 64), smem, stream, p);
  return hipGetLastError();
}

hipError_t launch_fwd(const FwdParams& p, int head_dim, int num_blocks, const TileJob* vjobs, int num_vjobs, hipStream_t stream) {
  hipError_t e;
  if (head_dim != 128) {
    if ((e = launch_transpose(p.v, p.num_kv_heads, head_dim, 64, vjobs, num_vjobs, p.total_kv_tiles, const_cast<__bf16*>(p.vt),
                              stream)) != hipSuccess) return e;
    return head_dim == 256 ? launch_fwd_t<256, 4>(p, num_blocks, stream) : launch_fwd_t<64, 4>(p, num_blocks, stream);
  }
  // ring slots of a K and a V tile, then the staging tiles of the four waves (64 rows each)
  const size_t smem = (size_t)2 * (FWD_PIPE_DIST + 3) * 32 * 128 * 2 + (size_t)4 * 64 * 128 * 2;
  static const hipError_t attr = raise_smem_limit(&fwd_pipe_kernel<128>, smem);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL((fwd_pipe_kernel<128>), dim3(persistent_grid(num_blocks)), dim3(256), smem, stream, p, num_blocks);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  // Second pass over the same items, 8 waves of 32 rows: a workgroup returns at once unless its flag is raised, and the
  // transposed V images it reads are only made if any flag is.
  if ((e = launch_transpose(p.v, p.num_kv_heads, head_dim, 64, vjobs, num_vjobs, p.total_kv_tiles, const_cast<__bf16*>(p.vt),
                            stream, p.any_redo)) != hipSuccess) return e;
  return launch_fwd_t<128, 8>(p, num_blocks, stream);
}

}  // namespace chunk_attn
