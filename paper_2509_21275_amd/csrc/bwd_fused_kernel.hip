// One-pass chunk-attention backward for head_dim 128 on gfx950: dK, dV and dQ from one walk (gradients of
// L = sum(O .* dO) under the chunk mask of the paper's section 3.1; key/value gradients include the context
// rows, section 2.1 / 3.2.2).
//
// The key-stationary kernel of bwd_kernel.hip (a workgroup owns 128 keys of one key/value head and walks the
// group's query heads x the 32-row query tiles that see them; S, P, dP, dS are computed once) is extended by the
// fifth contraction, dQ^T(tile) = K^T dS^T over the workgroup's 128 keys.  dQ sums over ALL keys, i.e. over
// workgroups.  Float atomics are far too slow for that on this chip (0.34 T/s measured, about a third of what the
// kernel produces), so the sum is kept in float32 tiles in the workspace that the workgroups update with plain
// loads and stores, one after the other in a fixed order:
//   * all key blocks of one (segment, key/value head) form a chain (plan.hpp); the whole chain runs on one XCD, so
//     that every update of a tile goes through the same L2 (loads bypass the per-CU cache);
//   * a block adds its share to a tile only after its predecessor has published that it is done with the tile
//     (a per-wave progress counter in the workspace, written after the tile's stores have completed); the chain's
//     first block sees every tile and writes instead of adding, so the tiles need no clearing;
//   * waits are bounded: a wave that gives up raises a status bit and carries on (the result is then wrong, but
//     every workgroup ends); workgroups are handed out in index order and a predecessor always has the smaller index,
//     so a waiting workgroup's predecessor is running or done.
//   * a long chain is dealt round robin to 2 or 4 sub-chains, each adding into a tile array of its own (summed by the
//     conversion): a link costs about two steps, and the further apart the workgroups of an XCD are in their walks, the
//     less of the Q / dO stream they share in the L2 (measured on the last-but-four slice of the 128K sequence: 208 GB
//     fetched per launch with one chain of 32 workgroups per XCD, 41 GB with four of 8).
// The order of additions is fixed by the plan: results are bit-reproducible.
// A tile is stored in the order the matrix pipe delivers it (wave = 32-wide slice of the head dimension, then
// the accumulator's register order), which makes every load and store of the walk one contiguous kilobyte;
// dq_convert_kernel turns the tiles into bf16 rows afterwards.
//
// Per step (stage n = n-th (head, query tile) of the walk) a wave runs, software pipelined as in bwd_dkv_pipe_kernel,
//     role A:  S(g) = Q K^T           P(g-1) = exp2(S(g-1) c - LSE)       dV^T += dO^T P(g-2)
//     role B:  dP(g-2) = dO V^T       dS(g-3) = P(g-3) (dP(g-3) - D)      dK^T += Q^T dS(g-4)    dS(g-4) -> LDS
//     all:     dQ^T(g-5) = K^T dS^T(g-5)   (8 MFMAs on the wave's 32 rows of the head dimension), load the tile of g-5,
//              add, store and publish dQ^T(g-6)
// as 24 mini-steps of one LDS operand fragment and the one or two MFMAs it feeds.
#include <cstring>
#include <type_traits>

#include "kernels.hpp"
#include "tiles.hpp"

namespace chunk_attn {

namespace {

constexpr int FUSED_DIST = 2;  // stages copied ahead of the step that first reads them

struct FusedParams {
  const __bf16 *q, *k, *v, *d_o;
  const float* lse2p;   // [Hq][total_q_tiles * 64]
  const float* dsp;
  __bf16 *dk, *dv;
  const FusedItem* items;
  const int32_t* order;  // item of workgroup b, -1: none
  float* dq_acc;         // [Hq][total_qt32] tiles of 4096 floats
  unsigned* progress;    // [items][4]: stages whose dQ update wave w of the item has completed
  unsigned* status;      // bit 0: a bounded wait expired; bit 1: an XCD received more workgroups than planned;
                         // words 8 .. 15: workgroups started per XCD; word 32: scratch
  int32_t num_slots;     // entries of `order`
  float* sink;           // 64 scratch dQ tiles of 16 KB
  int64_t total_q_tiles, total_qt32;
  int64_t buf_bytes;     // size of one dQ tile array (a chain is split into sub-chains, each with its own array)
  int32_t num_q_heads, num_kv_heads, group;
  float scale, scale_log2;
  int32_t accumulate, out_f32;
  int32_t spin_limit;
};

__device__ __forceinline__ void dkv_store4(const FusedParams& p, __bf16* out, int64_t elem, float v0, float v1, float v2,
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

// ---- the step's schedule, as data: 24 mini-steps; T = transposed fragment (two LDS reads) feeding the two dV^T / dK^T
// MFMAs, R = rows fragment (one read) feeding the two S / dP MFMAs, Q = dS^T fragment (two reads) feeding one dQ^T MFMA.
// A fragment is read four mini-steps before it is used (the first four of a step at the end of the step before).  The
// dS^T fragments are written by other waves in the step before and must be read inside the step: none sits in the
// first four mini-steps. ----
enum : int { MS_T = 0, MS_R = 1, MS_Q = 2 };
struct MiniStep { int kind, idx; };
constexpr int NMS = 24, MS_AHEAD = 4;
constexpr MiniStep kSeq[NMS] = {{MS_T, 0}, {MS_T, 1}, {MS_T, 2}, {MS_T, 3}, {MS_Q, 0}, {MS_T, 4}, {MS_T, 5}, {MS_Q, 1},
                                {MS_T, 6}, {MS_T, 7}, {MS_Q, 2}, {MS_R, 0}, {MS_R, 1}, {MS_Q, 3}, {MS_R, 2}, {MS_R, 3},
                                {MS_Q, 4}, {MS_R, 4}, {MS_R, 5}, {MS_Q, 5}, {MS_R, 6}, {MS_Q, 6}, {MS_R, 7}, {MS_Q, 7}};
static_assert(kSeq[0].kind == MS_T && kSeq[1].kind == MS_T && kSeq[2].kind == MS_T && kSeq[3].kind == MS_T,
              "a step opens with four transposed fragments (read at the end of the step before)");
constexpr int frag_reads(int m) { return kSeq[(m + NMS) % NMS].kind == MS_R ? 1 : 2; }
// LDS instructions a mini-step issues besides its fragment read: the P hand-over (role A writes, role B reads) in
// mini-step 0, the row values in mini-step 1, role B's dS hand-over in mini-step 2
constexpr int extras(int role, int m) {
  m = (m + NMS) % NMS;
  return m == 0 ? 4 : m == 1 ? 4 : (m == 2 && role == 1) ? 4 : 0;
}
// LDS instructions issued between the read of mini-step m's fragment and the start of mini-step m (where its wait stands)
constexpr int lgkm_after_frag(int role, int m) {
  int n = extras(role, m - MS_AHEAD);
  for (int k = m - MS_AHEAD + 1; k < m; ++k) n += frag_reads(k + MS_AHEAD) + extras(role, k);
  return n;
}
constexpr int VEC_START = 4;  // first mini-step with vector work: hand-over and row values must have arrived
// LDS instructions issued after the row-value reads (the last of what the vector work needs) up to the start of VEC_START
constexpr int lgkm_after_rows(int role) {
  int n = 0;
  for (int k = 2; k < VEC_START; ++k) n += frag_reads(k + MS_AHEAD) + extras(role, k);
  return n;
}
constexpr int lgkm_wait(int role, int m) {
  int w = lgkm_after_frag(role, m);
  if (m == VEC_START) {
    const int r = lgkm_after_rows(role);
    w = r < w ? r : w;
  }
  return w > 15 ? 15 : w;  // a 4-bit counter: waiting for fewer outstanding operations is always safe
}
// halves of the vector work (one score each) done before mini-step m: one after every MFMA from VEC_START on
constexpr int halves_before(int m) {
  int n = 0;
  for (int k = VEC_START; k < m; ++k) n += kSeq[k].kind == MS_Q ? 1 : 2;
  return n;
}
static_assert(halves_before(NMS) == 32, "32 scores per lane and step");
// memory operation (0 .. 14, -1: none) issued in mini-step m: tile stores, tile loads, row values, three operand copies,
// progress store, progress fetch, the fourth copy
constexpr int kVmSlot[15] = {0, 1, 2, 3, 5, 6, 8, 9, 11, 12, 14, 15, 17, 18, 20};  // two-MFMA mini-steps only
constexpr int vm_of(int m) {
  for (int k = 0; k < 15; ++k)
    if (kVmSlot[k] == m) return k;
  return -1;
}

template <int D>
__global__ __launch_bounds__(256, 1) void bwd_fused_pipe_kernel(FusedParams p) {
  constexpr int NW = 4;        // waves
  constexpr int BM = 32;       // query rows per stage
  constexpr int KC = D / 8;    // 16-byte chunks per operand row
  constexpr int DK = D / 16;   // k-steps over the head dimension
  constexpr int DB = D / 32;   // 32-row blocks of dK^T / dV^T
  constexpr int QT = BM * D;   // elements per operand tile
  constexpr int DIST = FUSED_DIST;
  constexpr int NS = DIST + 5; // ring slots: stages g - 4 .. g in use, g + 1 .. g + DIST on their way
  constexpr int PS = 2 * 4 * 64 * 8;   // elements of one P hand-over slot: 2 wave pairs x 4 fragments x 64 lanes x 8
  constexpr int DS = 128 * 32;         // elements of one dS hand-over slot: 128 keys x 32 queries
  constexpr int CH = BM * KC;          // 16-byte chunks per operand tile
  constexpr int NP = CH / 64;          // 64-slot pieces per tile
  constexpr int PER = 2 * NP / NW;     // global->LDS copies of operand pieces per wave and stage
  constexpr int RV = 64;               // floats per slot of the LSE / D rows (32 used; a whole wave copies them)
  constexpr int VM_OPS = 10 + 1 + PER; // memory operations per wave and step: 10 for dQ, the row values, the operand copies
  static_assert(D == 128 && PER == 4, "the mini-step schedule is written for head_dim 128");

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  lds_bf16* const L = (lds_bf16*)smem;
  constexpr int Q_OFF = 0;                 // [NS][QT]  Q rows of stage n in slot n % NS
  constexpr int G_OFF = Q_OFF + NS * QT;   // [NS][QT]  dO rows
  constexpr int P_OFF = G_OFF + NS * QT;   // [2][PS]   P hand-over
  constexpr int S_OFF = P_OFF + 2 * PS;    // [2][DS]   dS hand-over: row = key (32 queries, 64 bytes)
  constexpr int R_OFF = S_OFF + 2 * DS;    // [NS][RV] floats LSE rows, then [NS][RV] floats D rows
  lds_f32* const lse_s = (lds_f32*)(L + R_OFF);
  lds_f32* const dsum_s = lse_s + NS * RV;
  constexpr int LDS_ELEMS = R_OFF + 2 * NS * RV * 2;  // in bf16 units

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int role = wave >> 1, pair = wave & 1;
  const int l32 = lane & 31, hh = lane >> 5;

  // The slot of this workgroup in the order: column = the XCD it runs on, row = how many workgroups of that XCD came
  // before it (a counter per XCD, zero before the launch).  A grid's workgroups are dealt to the XCDs round robin, so
  // every XCD receives as many workgroups as its column has rows, whichever XCD the first one lands on; taking the
  // column from the hardware register instead of the workgroup index keeps a chain inside one L2 in any case, and
  // the predecessor of a slot (an earlier row of the same column) has always started before it.
  __shared__ int my_slot;
  if (tid == 0) {
    const unsigned xcc = __builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 20) & 7u;  // XCC_ID
    const unsigned row = __hip_atomic_fetch_add(p.status + 8 + xcc, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int64_t sl = (int64_t)row * kNumXcd + xcc;
    if (sl >= p.num_slots) atomicOr(p.status, 2u);  // more workgroups on this XCD than its column has rows
    my_slot = sl < p.num_slots ? (int)sl : -1;
  }
  __syncthreads();
  const int slot = my_slot;
  if (slot < 0) return;
  const int item_id = p.order[slot];
  if (item_id < 0) return;
  const FusedItem it = p.items[item_id];
  const int kvh = it.kvh;
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
  const int n_iter = nqt * G;  // stages: (query tile, head in group), the heads of a tile one after the other

  // ---- staging of Q / dO / LSE / D, as in bwd_dkv_pipe_kernel ----
  unsigned v_full[PER], v_last[PER];
  {
    const int last_row = it.q_len - 1 - (it.n_qt - 1) * BM;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int x = ((i * NW + wave) % NP) * 64 + lane;
      const int off = (x >> 5) * 8, row = (x & 31) ^ (((x >> 5) & 3) << 2);
      v_full[i] = (unsigned)(row * (int)q_stride + off) * 2u;
      v_last[i] = (unsigned)(min(row, last_row) * (int)q_stride + off) * 2u;
    }
  }
  const int64_t roff0 = (int64_t)(it.q_row_seg + it.qt_first * BM) * q_stride + (int64_t)(kvh * G) * D;
  const int64_t rv0g = ((int64_t)(kvh * G) * p.total_q_tiles + it.q_tile0) * 64 + it.qt_first * BM;
  const char* d_q = reinterpret_cast<const char*>(p.q + roff0);
  const char* d_g = reinterpret_cast<const char*>(p.d_o + roff0);
  const char* d_r = reinterpret_cast<const char*>(((wave & 1) ? p.dsp : p.lse2p) + rv0g);
  const int64_t head_bytes = (int64_t)D * 2;                             // to the next head of the group, same tile
  const int64_t head_rows_bytes = p.total_q_tiles * 64 * 4;
  const int64_t tile_bytes = (int64_t)BM * q_stride * 2 - (G - 1) * head_bytes;   // from the last head to the first, next tile
  const int64_t tile_rows_bytes = (int64_t)BM * 4 - (G - 1) * head_rows_bytes;
  int d_heads = G, d_tiles = nqt;
  unsigned d_slot = 0;
  const unsigned lane4 = (unsigned)lane * 4u;
  lds_f32* const rows_dst = (wave & 1) ? dsum_s : lse_s;
  auto dma_rows = [&]() __attribute__((always_inline)) { dma4(d_r + lane4, rows_dst + d_slot / (QT / RV)); };
  auto dma_piece = [&](int i) __attribute__((always_inline)) {
    const int piece = i * NW + wave;
    const unsigned voff = d_tiles == 1 ? v_last[i] : v_full[i];
    const char* base = i < NP / NW ? d_q : d_g;
    lds_bf16* dst = L + (i < NP / NW ? Q_OFF + piece * 512 : G_OFF + (piece - NP) * 512) + d_slot;
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

  // ---- per-lane operand addresses (elements) inside a tile, as in bwd_dkv_pipe_kernel ----
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

  // ---- dQ: the wave's 32 rows of the head dimension (block `wave`) ----
  // K^T fragments (A operands): lane holds K^T[d = 32 wave + l32][key slots of k-step ks], the 8 slots of half hh being
  // keys 16 ks + 4 hh + 0..3 and 16 ks + 8 + 4 hh + 0..3 (the order in which the transposed LDS read delivers dS^T).
  // Keys past the item's last one count as zero: their dS is not.
  bf16x8 ktf[8];
  {
    const unsigned short* kb16 = reinterpret_cast<const unsigned short*>(p.k) + (int64_t)it.kv_row0 * kv_stride + (int64_t)kvh * D +
                                 32 * wave + l32;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      s16x8 raw;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int key = 16 * ks + 8 * (e >> 2) + 4 * hh + (e & 3);
        raw[e] = key < it.kv_rows ? (short)kb16[(int64_t)key * kv_stride] : (short)0;
      }
      ktf[ks] = __builtin_bit_cast(bf16x8, raw);
    }
    // Pinned here, in accumulation registers: left to itself the compiler may move some of these loads down to their first
    // use inside the walk, where its count of outstanding loads does not include the walk's copies and dQ traffic
    // (issued as opaque instructions), so that its wait would be too short.
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+a"(ktf[ks]));
  }
  // dS hand-over tile: row = key (64 bytes = 32 queries), the four 16-byte pieces of a row swapped by (key / 4) % 4.
  // Column position of query 16 a + 8 b + 4 h + r of the stage is 16 a + 8 h + 4 b + r: role B's operand registers
  // go out as they are, 16 bytes each.  Reader: lane j of a 16-lane group (half hh, column group grp) addresses the 8 bytes
  // (key k0 + 4 hh + j / 4 [+ 8], columns 16 grp + 4 (j % 4) ..+3) and receives column 16 grp + j for four keys.
  unsigned ds_rd[2];   // byte address inside a dS slot for k-step 0: low and high half of the fragment
  {
    const int j = lane & 15, grp = (lane >> 4) & 1;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int key = 4 * hh + (j >> 2) + 8 * half;              // + 16 ks
      const int piece = (2 * grp + ((j & 3) >> 1)) ^ ((hh + 2 * half) & 3);
      ds_rd[half] = lds_addr(L + S_OFF) + (unsigned)(key * 64 + piece * 16 + (j & 1) * 8);
    }
  }
  // the dQ^T tile column this lane holds: query of the stage
  // (column position l32 = 16 a + 8 h + 4 b + r  ->  query 16 a + 8 b + 4 h + r)
  // chain state (wave-uniform)
  const bool has_pred = it.pred >= 0;
  unsigned* const my_prog = p.progress + (int64_t)item_id * 4 + wave;
  const unsigned* const pred_prog = p.progress + (int64_t)(has_pred ? it.pred : item_id) * 4 + wave;
  // tile of a stage: ((kvh G + head in group) total_qt32 + dq_tile0 + query tile) x 16 KB, this wave's 4 KB of it, 16 bytes per
  // lane per register group (4 groups, 1 KB apart)
  const int64_t acc_tile0 = it.buf * p.buf_bytes + ((int64_t)(kvh * G) * p.total_qt32 + it.dq_tile0 + it.qt_first) * 16384 + wave * 4096;
  const int64_t acc_head_bytes = p.total_qt32 * 16384;                    // to the same tile of the next head
  const int64_t acc_tile_bytes = 16384 - (G - 1) * acc_head_bytes;        // from the last head to the first, next tile
  const unsigned lane16 = (unsigned)lane * 16u;

  auto body = [&](auto role_c) __attribute__((always_inline)) {
    constexpr int ROLE = decltype(role_c)::value;
    const lds_bf16* const a_tile = L + (ROLE ? G_OFF : Q_OFF);
    const lds_bf16* const t_tile = L + (ROLE ? Q_OFF : G_OFF);
    const lds_f32* const rv_rows = (ROLE ? dsum_s : lse_s) + 4 * hh;
    lds_bf16* const pex = L + P_OFF + pair * (4 * 512) + lane * 8;

    bf16x8 bfrag[2][DK];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const __bf16* src = ROLE ? p.v : p.k;
      const int64_t grow = it.kv_row0 + min(64 * pair + 32 * kb + l32, it.kv_rows - 1);
      const int64_t off = grow * kv_stride + (int64_t)kvh * D + 8 * hh;
#pragma unroll
      for (int ks = 0; ks < DK; ++ks) bfrag[kb][ks] = *reinterpret_cast<const bf16x8*>(src + off + 16 * ks);
    }
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int ks = 0; ks < DK; ++ks) asm volatile("" : "+a"(bfrag[kb][ks]));  // loaded before the walk starts (see ktf)

    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 acc[2][DB];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int db = 0; db < DB; ++db) acc[kb][db] = zero16;

    const int jrel = it.j0 + 64 * pair + l32 - it.ctx;
    const int jrel_hi = it.j0 + 64 * pair + 63 - it.ctx;

    // role B's dS hand-over store address: key row 64 pair + 32 kb + l32, piece (2 ks + hh) ^ ((l32 / 4) % 4)
    unsigned ds_wr[2][2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
        ds_wr[kb][ks] = lds_addr(L + S_OFF) + (unsigned)((64 * pair + 32 * kb + l32) * 64 + (((2 * ks + hh) ^ ((l32 >> 2) & 3)) * 16));

#pragma unroll
    for (int s = 0; s < DIST; ++s) {
      dma_rows();
#pragma unroll
      for (int i = 0; i < PER; ++i) dma_piece(i);
      dma_advance();
    }
    __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
    wg_barrier();

    int sA = ROLE ? NS - 2 : 0;
    int s_qt = it.qt_first;
    int s_heads = G;
    f32x16 mask_c[2] = {zero16, zero16};
    bool mask_set = false;
    f32x16 x[2][2];
    bf16x8 f[2][2][2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) x[b][kb][i] = ROLE ? 0.f : -INFINITY;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
          for (int i = 0; i < 8; ++i) f[b][kb][ks][i] = (__bf16)0.0f;
      }
    bf16x8 fr[8];

    const unsigned t_lo0 = lds_addr(t_tile + t_off[0]), t_hi0 = lds_addr(t_tile + t_off[1]);
    const unsigned a_ev0 = lds_addr(a_tile + x_off[0]), a_od0 = lds_addr(a_tile + x_off[1]);
    const unsigned rv0 = lds_addr(rv_rows), pex0 = lds_addr(pex);
    constexpr unsigned SLOT = QT * 2;
    auto load_t = [&](unsigned lo_addr, unsigned hi_addr, auto m_c) __attribute__((always_inline)) {
      constexpr int m = decltype(m_c)::value;
      constexpr int off = ((m / DB) * (16 * 8) + (m % DB) * (4 * 32 * 8)) * 2;
      const s16x4 lo = lds_asm_read_tr<off>(lo_addr);
      const s16x4 hi = lds_asm_read_tr<off>(hi_addr);
      return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    auto load_a = [&](unsigned ev_addr, unsigned od_addr, auto ks_c) __attribute__((always_inline)) {
      constexpr int ks = decltype(ks_c)::value;
      constexpr int off = (ks >> 1) * (4 * 32 * 8) * 2;
      return lds_asm_read16<off>((ks & 1) ? od_addr : ev_addr);
    };
    // dS^T fragment of k-step ks (keys 16 ks .. 16 ks + 15): rows are 64 bytes
    auto load_q = [&](unsigned lo_addr, unsigned hi_addr, auto ks_c) __attribute__((always_inline)) {
      constexpr int ks = decltype(ks_c)::value;
      const s16x4 lo = lds_asm_read_tr<ks * 16 * 64>(lo_addr);
      const s16x4 hi = lds_asm_read_tr<ks * 16 * 64>(hi_addr);
      return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    {  // the first fragments of step 0 (zeros)
      const unsigned sT = prev_slot(prev_slot(sA)) * SLOT;
      static_for<0, MS_AHEAD>([&](auto m_c) __attribute__((always_inline)) {
        fr[decltype(m_c)::value] = load_t(t_lo0 + sT, t_hi0 + sT, m_c);
      });
    }

    // ---- dQ state ----
    // Every step issues the same 15 memory operations in the same order -- 4 tile stores, 4 tile loads, row values, 3
    // operand copies, progress store, progress fetch, the 4th operand copy -- so that "all but the last N operations have
    // completed" (s_waitcnt vmcnt(N); memory operations of a wave complete in order) names the same operations in every
    // step.  What a step has no use for (pipeline fill and drain, the chain's first block) goes to a scratch tile / scratch
    // word in the workspace, or reads a tile without using it.
    // A link of the chain costs about two steps: a block publishes a stage half a step after storing it (once the stores
    // are acknowledged), its successor fetches the progress half a step before it loads the stage's tile.
    f32x16 dq_acc;          // dQ^T of the stage in flight: [32 rows of the head dimension] x [32 queries]
    f32x4 dq_old[4];        // previous contents of the tile: loaded in step g, added at the start of step g + 1
    unsigned pf = 0u;       // predecessor's progress: fetched late in step g, looked at early in step g + 1
#pragma unroll
    for (int i = 0; i < 16; ++i) dq_acc[i] = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) dq_old[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    // running tile pointers (bytes into dq_acc) of the stage to load (ld_) and of the stage to store (st_), with the
    // heads left in their query tile (counting that one)
    const char* const acc_base = reinterpret_cast<const char*>(p.dq_acc);
    // scratch tiles: one of 64, by workgroup index (all workgroups fill their pipelines at the same time when the kernel starts)
    const char* const sink_tile = reinterpret_cast<const char*>(p.sink) + (slot & 63) * 16384 + wave * 4096;
    unsigned* const sink_word = p.status + 32;
    int64_t ld_off = acc_tile0, st_off = acc_tile0;
    int ld_left = G, st_left = G;                  // heads left in the tile of the stage to load / to store
    // predecessor's progress required before the next load: its walk begins delta_qt tiles (of G stages) before this one
    unsigned need = (unsigned)(it.delta_qt * G) + 1u;
    bool dead = !has_pred;                         // no more waiting: no predecessor, or a wait expired

    auto step = [&](int g, f32x16 (&cur)[2], f32x16 (&nxt)[2], bf16x8 (&f_old)[2][2],
                    bf16x8 (&f_new)[2][2]) __attribute__((always_inline)) {
      const int sR = prev_slot(sA), sT = prev_slot(sR);
      const unsigned oA = sA * SLOT, oR = sR * SLOT, oT = sT * SLOT;
      const unsigned t_lo = t_lo0 + oT, t_hi = t_hi0 + oT, a_ev = a_ev0 + oA, a_od = a_od0 + oA;
      const unsigned n_lo = t_lo0 + oR, n_hi = t_hi0 + oR;
      if (ROLE == 0) {
        const bool valid = g < n_iter;
        if (__builtin_expect(!valid || s_qt * BM < jrel_hi, 0)) {
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
      bf16x8 ph[2][2];
      f32x4 r4[4];
      const unsigned pa = pex0 + (ROLE == 0 ? (g & 1) : ((g & 1) ^ 1)) * (PS * 2);
      const unsigned ra = rv0 + sR * (RV * 4);
      const unsigned ds_w = (g & 1) * (DS * 2);         // role B writes dS(g - 4) here
      const unsigned ds_r = ((g & 1) ^ 1) * (DS * 2);   // everybody reads dS(g - 5), written in the step before
      const unsigned q_lo = ds_rd[0] + ds_r, q_hi = ds_rd[1] + ds_r;
      unsigned pw[2][8];
      float e_hold[2];
      // vector work of score h (0 .. 31): element i = h % 16 of key block kb = h / 16
      auto vec_half = [&](auto h_c) __attribute__((always_inline)) {
        constexpr int h = decltype(h_c)::value;
        constexpr int j = h >> 1, q = h & 1;
        constexpr int kb = j >> 3, dw = j & 7, i = 2 * dw + q;
        if (ROLE == 0) {
          if constexpr (j > 0 && q == 0) {
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
      // ---- dQ bookkeeping of this step (wave-uniform) ----
      // stage s: dQ^T and the load of its tile in step s + 5, added and stored at the start of step s + 6, published in the
      // middle of step s + 6 (progress s + 1)
      const int s_store = g - 6, s_pub = g - 5, s_load = g - 5;  // progress s_pub covers stages < s_pub
      const bool do_store = s_store >= 0 && s_store < n_iter;
      const bool do_pub = s_pub >= 1 && s_pub <= n_iter;
      const bool in_load = s_load >= 0 && s_load < n_iter;      // the tile exists: read it even if nothing is done with it
      const bool do_load = in_load && has_pred;
      // The step's 15 memory operations, one per mini-step (the waves of a workgroup run in step, and the CU's memory
      // pipeline takes 16 cycles per kilobyte: four waves issuing four kilobyte-sized operations each at once would hold up
      // whatever comes next).  Operation k is issued in mini-step vm_slot[k]; their order is what the waits count on.
      f32x4 st_v[4];
      const char* st_p = sink_tile;
      const char* ld_p = acc_base + acc_tile0;
      auto vm_op = [&](auto k_c) __attribute__((always_inline)) {
        constexpr int k = decltype(k_c)::value;
        if constexpr (k == 0) {
          // add dQ^T(g - 6): its last MFMA was issued a step ago; the tile's previous contents were requested in the step
          // before (since then: row values, 3 copies, progress store and fetch, a copy)
          asm volatile("s_waitcnt vmcnt(7)" : "+v"(dq_old[0]), "+v"(dq_old[1]), "+v"(dq_old[2]), "+v"(dq_old[3]) : : "memory");
          st_p = do_store ? acc_base + st_off : sink_tile;
          st_v[0] = f32x4{dq_acc[0], dq_acc[1], dq_acc[2], dq_acc[3]}; st_v[1] = f32x4{dq_acc[4], dq_acc[5], dq_acc[6], dq_acc[7]};
          st_v[2] = f32x4{dq_acc[8], dq_acc[9], dq_acc[10], dq_acc[11]}; st_v[3] = f32x4{dq_acc[12], dq_acc[13], dq_acc[14], dq_acc[15]};
          if (has_pred) {  // the chain's first block initialises every tile
            st_v[0] += dq_old[0]; st_v[1] += dq_old[1]; st_v[2] += dq_old[2]; st_v[3] += dq_old[3];
          }
          if (do_store) {
            if (st_left > 1) { --st_left; st_off += acc_head_bytes; }
            else { st_left = G; st_off += acc_tile_bytes; }
          }
        }
        if constexpr (k >= 0 && k < 4) {   // tile stores
          asm volatile("global_store_dwordx4 %0, %1, %2 offset:%3\n\ts_nop 1" : : "v"(lane16), "v"(st_v[k]), "s"(st_p), "n"(k * 1024) : "memory");
        }
        if constexpr (k == 4) {
          // the previous contents of the tile of stage g - 5, once the predecessor is done with it: its progress was fetched
          // late in the step before (since then: a copy, 4 tile stores); if it is not enough, ask again until it is
          asm volatile("s_waitcnt vmcnt(5)" : "+v"(pf) : : "memory");
          if (do_load) {
            const unsigned seen = __builtin_amdgcn_readfirstlane(pf);
            if (__builtin_expect(!dead && seen < need, 0)) {
              int spins = 0;
              for (;;) {
                unsigned v;
                asm volatile("global_load_dword %0, %1, off sc1\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(pred_prog) : "memory");
                if (__builtin_amdgcn_readfirstlane(v) >= need) break;
                if (++spins > p.spin_limit) {
                  if (lane == 0) atomicOr(p.status, 1u);
                  dead = true;
                  break;
                }
                __builtin_amdgcn_s_sleep(2);
              }
            }
          }
          ld_p = acc_base + (in_load ? ld_off : acc_tile0);
          if (in_load) {
            need += 1u;
            if (ld_left > 1) { --ld_left; ld_off += acc_head_bytes; }
            else { ld_left = G; ld_off += acc_tile_bytes; }
          }
        }
        if constexpr (k >= 4 && k < 8) {   // tile loads
          asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3 sc1" : "=&v"(dq_old[k - 4]) : "v"(lane16), "s"(ld_p), "n"((k - 4) * 1024) : "memory");
        }
        if constexpr (k == 8) dma_rows();
        if constexpr (k == 9 || k == 10 || k == 11) dma_piece(k - 9);
        if constexpr (k == 12) {
          // this step's tile stores (since then: 4 tile loads, row values, 3 copies) have been acknowledged: publish them
          asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
          const unsigned val = (unsigned)s_pub;
          unsigned* const dst = do_pub ? my_prog : sink_word;
          if (lane == 0) asm volatile("global_store_dword %0, %1, off sc0" : : "v"(dst), "v"(val) : "memory");
        }
        if constexpr (k == 13) asm volatile("global_load_dword %0, %1, off sc1" : "=v"(pf) : "v"(pred_prog) : "memory");  // for the next step
        if constexpr (k == 14) dma_piece(3);
      };
      asm volatile("s_nop 7" ::: "memory");
      __builtin_amdgcn_sched_barrier(0);
      static_for<0, NMS>([&](auto m_c) __attribute__((always_inline)) {
        constexpr int m = decltype(m_c)::value;
        constexpr int kind = kSeq[m].kind, idx = kSeq[m].idx;
        {  // wait for this mini-step's fragment (and, in VEC_START, for the hand-over and the row values)
          constexpr int lgkm = lgkm_wait(ROLE, m);
          if constexpr (m == VEC_START) {
            if (ROLE == 0)
              asm volatile("s_waitcnt lgkmcnt(%5)" : "+v"(fr[m & 7]), "+v"(r4[0]), "+v"(r4[1]), "+v"(r4[2]), "+v"(r4[3]) : "n"(lgkm));
            else
              asm volatile("s_waitcnt lgkmcnt(%9)" : "+v"(fr[m & 7]), "+v"(r4[0]), "+v"(r4[1]), "+v"(r4[2]), "+v"(r4[3]),
                           "+v"(ph[0][0]), "+v"(ph[0][1]), "+v"(ph[1][0]), "+v"(ph[1][1]) : "n"(lgkm));
          } else {
            asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(fr[m & 7]) : "n"(lgkm));
          }
        }
        {  // read the fragment of mini-step m + 4 (past the end: the next step's first transposed fragments)
          constexpr int mm = m + MS_AHEAD;
          if constexpr (mm >= NMS) {
            fr[mm & 7] = load_t(n_lo, n_hi, std::integral_constant<int, kSeq[mm % NMS].idx>{});
          } else if constexpr (kSeq[mm % NMS].kind == MS_T) {
            fr[mm & 7] = load_t(t_lo, t_hi, std::integral_constant<int, kSeq[mm % NMS].idx>{});
          } else if constexpr (kSeq[mm % NMS].kind == MS_R) {
            fr[mm & 7] = load_a(a_ev, a_od, std::integral_constant<int, kSeq[mm % NMS].idx>{});
          } else {
            fr[mm & 7] = load_q(q_lo, q_hi, std::integral_constant<int, kSeq[mm % NMS].idx>{});
          }
        }
        const bf16x8 fa = fr[m & 7];
        auto mma = [&](auto kb_c) __attribute__((always_inline)) {
          constexpr int kb = decltype(kb_c)::value;
          if constexpr (kind == MS_T) {
            constexpr int ks = idx / DB, db = idx % DB;
            acc[kb][db] = mfma32(fa, f_old[kb][ks], acc[kb][db]);
          } else if constexpr (kind == MS_R) {
            constexpr int ks = idx;
            if (ks == 0 && ROLE == 0)
              asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(nxt[kb]) : "v"(fa), "a"(bfrag[kb][ks]), "v"(mask_c[kb]));
            else if (ks == 0)
              asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(nxt[kb]) : "v"(fa), "a"(bfrag[kb][ks]));
            else
              asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(nxt[kb]) : "v"(fa), "a"(bfrag[kb][ks]));
          }
        };
        constexpr std::integral_constant<int, 0> c0{};
        constexpr std::integral_constant<int, 1> c1{};
        constexpr int hb = halves_before(m);
        if constexpr (kind == MS_Q) {
          // dQ^T(g - 5) += K^T[:, keys of k-step idx] dS^T
          const bf16x8& a_ = ktf[idx];
          if constexpr (idx == 0) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(dq_acc) : "a"(a_), "v"(fa));
          else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(dq_acc) : "a"(a_), "v"(fa));
          static_assert(vm_of(m) < 0, "memory operations sit in two-MFMA mini-steps");
          if constexpr (m >= VEC_START) vec_half(std::integral_constant<int, hb>{});
          __builtin_amdgcn_sched_barrier(0);
        } else {
        mma(c0);
        if constexpr (m == 0) {
          if (ROLE == 0) {
            lds_asm_write16<0>(pa, f_old[0][0]);
            lds_asm_write16<1024>(pa, f_old[0][1]);
            lds_asm_write16<2048>(pa, f_old[1][0]);
            lds_asm_write16<3072>(pa, f_old[1][1]);
          } else {
            ph[0][0] = lds_asm_read16<0>(pa);
            ph[0][1] = lds_asm_read16<1024>(pa);
            ph[1][0] = lds_asm_read16<2048>(pa);
            ph[1][1] = lds_asm_read16<3072>(pa);
          }
        }
        if constexpr (m == 1) {
          r4[0] = lds_asm_read16f<0>(ra);
          r4[1] = lds_asm_read16f<32>(ra);
          r4[2] = lds_asm_read16f<64>(ra);
          r4[3] = lds_asm_read16f<96>(ra);
        }
        if constexpr (m == 2) {
          if (ROLE == 1) {  // dS(g - 4), the operand of this step's dK^T products, for everybody's dQ^T in the next step
            lds_asm_write16<0>(ds_wr[0][0] + ds_w, f_old[0][0]);
            lds_asm_write16<0>(ds_wr[0][1] + ds_w, f_old[0][1]);
            lds_asm_write16<0>(ds_wr[1][0] + ds_w, f_old[1][0]);
            lds_asm_write16<0>(ds_wr[1][1] + ds_w, f_old[1][1]);
          }
        }
        // the two roles issue their memory operation in different halves of the mini-step: the CU's memory pipeline takes
        // 16 cycles per kilobyte, and waves that issue together wait for each other
        if constexpr (ROLE == 0) vm_op(std::integral_constant<int, vm_of(m)>{});
        if constexpr (m >= VEC_START) vec_half(std::integral_constant<int, hb>{});
        __builtin_amdgcn_sched_barrier(0);
        mma(c1);
        if constexpr (ROLE == 1) vm_op(std::integral_constant<int, vm_of(m)>{});
        if constexpr (m >= VEC_START) vec_half(std::integral_constant<int, hb + 1>{});
        if constexpr (m == 22) {  // after the step's last operand copy
          dma_advance();
          sA = sA == NS - 1 ? 0 : sA + 1;
          if (ROLE == 0 && --s_heads == 0) {
            s_heads = G;
            ++s_qt;
          }
        }
        __builtin_amdgcn_sched_barrier(0);
        }
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
      // Stage g + 1 must have landed: its last copy was the last operation of step g + 1 - DIST, so all but the operations of
      // the DIST - 1 steps since may be outstanding.
      asm volatile("s_waitcnt vmcnt(%5)" : "+v"(pf), "+v"(dq_old[0]), "+v"(dq_old[1]), "+v"(dq_old[2]), "+v"(dq_old[3])
                   : "n"((DIST - 1) * VM_OPS) : "memory");
      wg_barrier();
    };
    // stage n: S in step n, dV^T in n + 2 (role A), dK^T in n + 4 (role B), dQ^T and the load of its tile in n + 5, added,
    // stored and published in n + 6
    const int n_steps = n_iter + 7;
    for (int g = 0; g < n_steps; g += 2) {
      step(g, x[0], x[1], f[0], f[1]);
      step(g + 1, x[1], x[0], f[1], f[0]);
    }

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
}

// dQ tiles (float32, in the order the one-pass kernel keeps them) -> dq rows (bf16, scaled).  One workgroup per
// (32-row query tile, head); thread = (wave w, lane): element (register group g, r) of the tile's slice w is
// dQ^T[d = 32 w + 8 g + 4 hh + r][column l32], and column position 16 a + 8 h + 4 b + r' holds query 16 a + 8 b + 4 h + r'.
// The tile arrays of the sub-chains are added in a fixed order; array r holds the tile only if the r-th key block of
// the segment exists and sees the tile.
__global__ __launch_bounds__(256) void dq_convert_kernel(const float* __restrict__ dq_acc, const DqTileJob* __restrict__ jobs,
                                                         int64_t total_qt32, int64_t buf_floats, int num_bufs, int num_q_heads,
                                                         float scale, __bf16* __restrict__ dq) {
  constexpr int D = 128;
  const int head = blockIdx.x % num_q_heads;
  const DqTileJob job = jobs[blockIdx.x / num_q_heads];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63, l32 = lane & 31, hh = lane >> 5;
  const int qrow = 16 * (l32 >> 4) + 8 * ((l32 >> 2) & 1) + 4 * ((l32 >> 3) & 1) + (l32 & 3);
  if (qrow >= job.valid_rows) return;
  const float* tile = dq_acc + ((int64_t)head * total_qt32 + job.tile) * 4096 + w * 1024 + lane * 4;
  f32x4 acc[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) acc[g] = *reinterpret_cast<const f32x4*>(tile + g * 256);   // array 0 holds every tile
  for (int r = 1; r < num_bufs; ++r) {
    if (r >= job.n_blocks || job.qt < max(0, DKV_KEYS * r - job.ctx) / 32) break;  // later blocks see even less
#pragma unroll
    for (int g = 0; g < 4; ++g) acc[g] += *reinterpret_cast<const f32x4*>(tile + r * buf_floats + g * 256);
  }
  __bf16* out = dq + ((int64_t)(job.q_row0 + qrow) * num_q_heads + head) * D + 32 * w + 4 * hh;
#pragma unroll
  for (int g = 0; g < 4; ++g)
    *reinterpret_cast<bf16x4*>(out + 8 * g) = pack4(acc[g][0] * scale, acc[g][1] * scale, acc[g][2] * scale, acc[g][3] * scale);
}

__global__ __launch_bounds__(256) void zero_words_kernel(unsigned* __restrict__ p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0u;
}

}  // namespace

hipError_t launch_bwd_fused(const chunk_attn_desc* d, const BwdArgs& a, const BwdPlan& P, const float* lse2p, const float* dsp,
                            hipStream_t stream) {
  constexpr int D = 128;
  char* ws = a.workspace;
  hipError_t e;
  unsigned* progress = reinterpret_cast<unsigned*>(ws + P.fprog_off);
  const int64_t n_words = (int64_t)(P.fprog_bytes / sizeof(unsigned));
  unsigned* status = progress + n_words - (kFusedSinkBytes + 256) / 4;   // then 256 bytes of status, then the scratch tile
  hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)((n_words + 255) / 256)), dim3(256), 0, stream, progress, n_words);
  if ((e = hipGetLastError()) != hipSuccess) return e;

  FusedParams p;
  p.q = a.q; p.k = a.k; p.v = a.v; p.d_o = a.d_o; p.lse2p = lse2p; p.dsp = dsp;
  p.dk = a.dk; p.dv = a.dv;
  p.items = reinterpret_cast<const FusedItem*>(ws + P.fitems_off);
  p.order = reinterpret_cast<const int32_t*>(ws + P.forder_off);
  p.dq_acc = reinterpret_cast<float*>(ws + P.fdq_off);
  p.progress = progress;
  p.status = status;
  p.sink = reinterpret_cast<float*>(status + 64);
  p.total_q_tiles = P.q_tiles;
  p.total_qt32 = P.qt32_tiles;
  p.buf_bytes = (int64_t)d->num_q_heads * P.qt32_tiles * 16384;
  p.num_q_heads = d->num_q_heads; p.num_kv_heads = d->num_kv_heads; p.group = d->num_q_heads / d->num_kv_heads;
  p.scale = d->softmax_scale; p.scale_log2 = d->softmax_scale * 1.4426950408889634f;
  p.accumulate = a.accumulate ? 1 : 0;
  p.out_f32 = a.dkv_f32 ? 1 : 0;
  p.spin_limit = 1 << 20;
  const int64_t blocks = (int64_t)P.fplan.order.size();
  if (blocks > 0x7fffffff) return hipErrorInvalidValue;
  p.num_slots = (int32_t)blocks;
  constexpr int NS = FUSED_DIST + 5;
  const size_t smem = (size_t)2 * NS * 32 * D * 2 + 2 * 4096 * 2 + 2 * 4096 * 2 + 2 * NS * 64 * sizeof(float);
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_fused_pipe_kernel<D>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (attr != hipSuccess) return attr;
  ProfileEvents pe = profile_events();
  profile_events() = ProfileEvents{};
  if (pe.start && (e = hipEventRecord(pe.start, stream)) != hipSuccess) return e;
  hipLaunchKernelGGL((bwd_fused_pipe_kernel<D>), dim3((unsigned)blocks), dim3(256), smem, stream, p);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (pe.stop && (e = hipEventRecord(pe.stop, stream)) != hipSuccess) return e;

  // dQ tiles -> bf16 rows: the 32-row tiles of the query ranges are numbered like the plan's dq_tile0 + query tile
  const int64_t cblocks = P.qt32_tiles * d->num_q_heads;
  if (cblocks > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(dq_convert_kernel, dim3((unsigned)cblocks), dim3(256), 0, stream, p.dq_acc,
                     reinterpret_cast<const DqTileJob*>(ws + P.q32jobs_off), P.qt32_tiles, p.buf_bytes / 4, P.fplan.num_bufs,
                     d->num_q_heads, d->softmax_scale, a.dq);
  return hipGetLastError();
}

}  // namespace chunk_attn
