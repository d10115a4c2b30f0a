// Seeded random calls into the host-side planner and scheduler, meant to be built with -fsanitize=address,undefined:
// checks memory safety and the structural guarantees of the outputs (no reference values are needed for that).
#include <cstdio>
#include <algorithm>
#include <cstdint>
#include <cstdlib>
#include <random>
#include <vector>

#include "chunk_plan.h"
#include "chunk_sched.h"
#include "../../paper_2509_21275_amd/csrc/plan.hpp"  // the attention library's host-side validation and work-item planning

#define REQUIRE(c) do { if (!(c)) { std::printf("FAILED %s at line %d (seed %u)\n", #c, __LINE__, seed); return 1; } } while (0)

// The work items of the three attention kernels on a random segment table (contexts, gaps between key ranges, ragged
// lengths): the (query row, key row) pairs an item list implies must be exactly the unmasked pairs of the chunk
// (paper section 3.1: query i of a segment sees the keys j <= C + i of its own key range), each exactly once, no item
// and no scheduled (query tile, key tile) without a visible pair.
static int check_plan_cover(unsigned seed) {
  std::mt19937 rng(seed * 2654435761u + 17);
  auto uni = [&](int lo, int hi) { return (int)(rng() % (unsigned)(hi - lo + 1)) + lo; };
  const int n_seg = uni(1, 6);
  std::vector<chunk_attn_seg> segs(n_seg);
  int32_t tq = 0, tkv = uni(0, 1) ? uni(0, 70) : 0;  // key rows before the first segment that nobody sees
  for (auto& s : segs) {
    const int q_len = uni(0, 3) ? uni(1, 200) : uni(1, 33);
    const int ctx = uni(0, 2) ? 0 : uni(1, 300);
    s = chunk_attn_seg{tq, q_len, tkv, ctx + q_len};
    tq += q_len;
    tkv += ctx + q_len + (uni(0, 3) ? 0 : uni(1, 40));  // sometimes a gap
  }
  chunk_attn_desc d{8, 2, 128, tq, tkv, n_seg, segs.data(), 0.1f};
  REQUIRE(chunk_attn::validate(&d) == CHUNK_ATTN_OK);
  std::vector<uint8_t> want((size_t)tq * tkv, 0);
  int64_t n_pairs = 0;
  for (const auto& s : segs)
    for (int i = 0; i < s.q_len; ++i)
      for (int j = 0; j <= s.kv_len - s.q_len + i; ++j) { want[(size_t)(s.q_start + i) * tkv + s.kv_start + j] = 1; ++n_pairs; }
  REQUIRE(n_pairs == chunk_attn::pair_count(&d));
  // a query tile of rows [q0, q0 + rows), row r seeing the first n0 + r keys from key row kv0, walked in key tiles of `bn`
  auto cover_rows = [&](std::vector<uint8_t>& got, int q0, int rows, int kv0, int n0, int bn) -> bool {
    if (rows < 1 || n0 < 1) return false;
    const int n_last = n0 + rows - 1;
    for (int t = 0; t * bn < n_last; ++t) {  // every key tile the kernels walk holds a visible pair of the last row
      bool any = false;
      for (int r = 0; r < rows; ++r)
        for (int j = t * bn; j < std::min((t + 1) * bn, n0 + r); ++j) {
          if (q0 + r >= tq || kv0 + j >= tkv) return false;
          ++got[(size_t)(q0 + r) * tkv + kv0 + j];
          any = true;
        }
      if (!any) return false;
    }
    return true;
  };
  for (int tile_rows : {32, 64, 128, 256}) {
    std::vector<uint8_t> got((size_t)tq * tkv, 0);
    for (const auto& it : chunk_attn::plan_fwd(&d, tile_rows)) REQUIRE(cover_rows(got, it.q_row0, it.q_rows, it.kv_row0, it.n0, 32));
    REQUIRE(got == want);
    std::fill(got.begin(), got.end(), 0);
    for (const auto& it : chunk_attn::plan_dq(&d, tile_rows)) REQUIRE(cover_rows(got, it.q_row0, it.q_rows, it.kv_row0, it.n0, 32));
    REQUIRE(got == want);
  }
  // (the order and the walk directions chosen for key blocks that run side by side change neither the cover nor the
  // number of items; without them every block walks upwards)
  for (int variant = 0; variant < 5; ++variant) {
    const int keys = variant == 0 ? 32 : 128;
    const int side_by_side = variant < 2 ? 0 : variant == 2 ? 1 : variant == 3 ? 3 : 32;
    std::vector<uint8_t> got((size_t)tq * tkv, 0);
    const auto dkv_items = chunk_attn::plan_dkv(&d, keys, side_by_side);
    REQUIRE(dkv_items.size() == chunk_attn::plan_dkv(&d, keys).size());
    for (const auto& it : dkv_items) {
      REQUIRE(it.reverse == 0 || (it.reverse == 1 && side_by_side > 0));
      REQUIRE(it.in_step == 0 || (it.in_step == 1 && side_by_side > 0 && it.reverse == 0 && it.qt_first == 0));
      REQUIRE(it.kv_rows >= 1 && it.kv_rows <= keys && it.qt_first >= 0 && it.qt_first < it.n_qt);
      REQUIRE(it.n_qt == (it.q_len + 31) / 32);
      for (int qt = it.qt_first; qt < it.n_qt; ++qt) {  // the 32-row query tiles the kernel walks
        bool any = false;
        for (int i = 32 * qt; i < std::min(32 * qt + 32, it.q_len); ++i)
          for (int kk = 0; kk < it.kv_rows; ++kk)
            if (i >= it.j0 + kk - it.ctx) {  // query i of the segment sees key j0 + kk
              REQUIRE(it.q_row_seg + i < tq && it.kv_row0 + kk < tkv);
              ++got[(size_t)(it.q_row_seg + i) * tkv + it.kv_row0 + kk];
              any = true;
            }
        REQUIRE(any);
      }
    }
    REQUIRE(got == want);
  }
  // the one-pass backward's plan: the same cover, and chains in which every block follows a block that sees at least
  // the query tiles it sees, pinned to one XCD and handed out after its predecessor
  for (int bufs : {1, 2, 4}) {
    const chunk_attn::FusedPlan P = chunk_attn::plan_fused(&d, 128, 8, bufs);
    std::vector<uint8_t> got((size_t)tq * tkv, 0);
    std::vector<int> slot_of(P.items.size(), -1);
    REQUIRE(P.order.size() % 8 == 0);
    for (size_t b = 0; b < P.order.size(); ++b) {
      if (P.order[b] < 0) continue;
      REQUIRE(P.order[b] < (int)P.items.size() && slot_of[P.order[b]] < 0);
      slot_of[P.order[b]] = (int)b;
    }
    int n_tiles = 0;
    for (const auto& s : segs) n_tiles += (s.q_len + 31) / 32;
    REQUIRE(P.total_qt32 == n_tiles && (int)P.tiles.size() == n_tiles);
    for (size_t i = 0; i < P.items.size(); ++i) {
      const auto& it = P.items[i];
      REQUIRE(slot_of[i] >= 0);                                   // every item is run by exactly one workgroup
      REQUIRE(it.kvh >= 0 && it.kvh < d.num_kv_heads && it.buf >= 0 && it.buf < bufs);
      REQUIRE(it.kv_rows >= 1 && it.kv_rows <= 128 && it.qt_first >= 0 && it.qt_first < it.n_qt);
      REQUIRE(it.dq_tile0 >= 0 && it.dq_tile0 + it.n_qt <= n_tiles);
      if (it.pred >= 0) {
        const auto& pr = P.items[it.pred];
        REQUIRE(it.pred < (int)i && pr.kvh == it.kvh && pr.q_row_seg == it.q_row_seg && pr.buf == it.buf);
        REQUIRE(pr.kv_row0 + 128 * bufs == it.kv_row0);             // the block `bufs` before it
        REQUIRE(pr.qt_first <= it.qt_first && it.delta_qt == it.qt_first - pr.qt_first);
        REQUIRE(slot_of[it.pred] % 8 == slot_of[i] % 8);            // same XCD
        REQUIRE(slot_of[it.pred] < slot_of[i]);                     // handed out earlier
      } else {
        REQUIRE(it.j0 < 128 * bufs && it.delta_qt == 0);            // one of the first blocks of its segment
      }
      if (it.kvh != 0) continue;                                  // the pair cover, once per key/value head
      for (int qt = it.qt_first; qt < it.n_qt; ++qt) {
        bool any = false;
        for (int q = 32 * qt; q < std::min(32 * qt + 32, it.q_len); ++q)
          for (int kk = 0; kk < it.kv_rows; ++kk)
            if (q >= it.j0 + kk - it.ctx) {
              ++got[(size_t)(it.q_row_seg + q) * tkv + it.kv_row0 + kk];
              any = true;
            }
        REQUIRE(any);
      }
    }
    REQUIRE(got == want);
    // every dQ tile is initialised: the first block of sub-chain 0 sees every tile of its segment
    for (const auto& it : P.items)
      if (it.pred < 0 && it.buf == 0) REQUIRE(it.qt_first == 0);
  }
  return 0;
}

// The order and walk directions of key blocks that run side by side, worked out by hand for one slice of a split
// sequence: 1024 context tokens and 16384 own tokens, 128 keys per block, 32 blocks at a time.  Blocks 0 .. 7 lie in
// the context (every query sees them): first, upwards.  Of the 128 others the shortest quarter, 104 .. 135, is kept
// for the end.  Of 8 .. 103 the 32 longest (8 .. 39) walk down, then their partners from the short end (72 .. 103, the
// longest of them first) walk up; the 32 left over split in two: 40 .. 55 down, 56 .. 71 up.
static int check_side_by_side_example() {
  const unsigned seed = 0;  // (not a seeded case; REQUIRE prints it)
  chunk_attn_seg s{0, 16384, 0, 16384 + 1024};
  chunk_attn_desc d{64, 8, 128, 16384, 16384 + 1024, 1, &s, 0.1f};
  const auto items = chunk_attn::plan_dkv(&d, 128, 32);
  REQUIRE(items.size() == 136);
  std::vector<int> want_block, want_rev;
  auto put = [&](int lo, int hi, int rev) { for (int b = lo; b <= hi; ++b) { want_block.push_back(b); want_rev.push_back(rev); } };
  put(0, 7, 0); put(8, 39, 1); put(72, 103, 0); put(40, 55, 1); put(56, 71, 0); put(104, 135, 0);
  for (size_t i = 0; i < items.size(); ++i) {
    REQUIRE(items[i].j0 == 128 * want_block[i] && items[i].reverse == want_rev[i]);
    REQUIRE(items[i].in_step == (want_block[i] < 8 ? 1 : 0));  // the equal walks of the context start group by group
    // The shortest of the descending walks ends first and its workgroup takes the first (longest) ascending one, the
    // longest takes the last: every such pair covers the same number of query tiles (block b walks 512 - 4 (b - 8)).
    if (i >= 8 && i < 40) REQUIRE((items[i].n_qt - items[i].qt_first) + (items[79 - i].n_qt - items[79 - i].qt_first) == 644);
  }
  return 0;
}

int main(int argc, char** argv) {
  if (check_side_by_side_example()) return 1;
  const unsigned n_cases = argc > 1 ? (unsigned)std::atoi(argv[1]) : 200;
  int n_infeasible = 0, n_ckpt = 0;
  for (unsigned seed = 1; seed <= n_cases; ++seed) {
    std::mt19937 rng(seed);
    auto uni = [&](int lo, int hi) { return (int)(rng() % (unsigned)(hi - lo + 1)) + lo; };
    if (check_plan_cover(seed)) return 1;
    // ---- sequence processor ----
    chunk_cost_model cm{1e-6 * uni(1, 50), 1e-3 * uni(0, 50), 1.0 * uni(0, 5), 1e-4 * uni(0, 3), 0.1 * uni(0, 3), uni(1, 8), uni(1, 4)};
    const int n_seqs = uni(1, 40), K = uni(1, 9), align = 1 << uni(0, 7);
    std::vector<int32_t> lengths(n_seqs);
    for (auto& l : lengths) l = uni(1, uni(0, 3) ? 4000 : 60000);
    const int cap = n_seqs * (K + 1);
    std::vector<chunk_plan_chunk> chunks(cap);
    std::vector<chunk_plan_slice> slices(cap);
    int32_t nc = 0, ns = 0;
    double tt = 0;
    int64_t tm = 0;
    REQUIRE(chunk_plan_build(&cm, 1 << 20, lengths.data(), n_seqs, K, align, chunks.data(), cap, &nc, slices.data(), cap, &ns, &tt, &tm) == CHUNK_ATTN_OK);
    std::vector<int64_t> covered(n_seqs, 0);
    for (int c = 0; c < nc; ++c) {
      REQUIRE(chunks[c].num_slices >= 1 && chunks[c].first_slice >= 0 && chunks[c].first_slice + chunks[c].num_slices <= ns);
      int64_t tok = 0;
      for (int s = 0; s < chunks[c].num_slices; ++s) {
        const chunk_plan_slice& sl = slices[chunks[c].first_slice + s];
        REQUIRE(sl.seq >= 0 && sl.seq < n_seqs && sl.len >= 1 && sl.start >= 0 && sl.start + sl.len <= lengths[sl.seq]);
        covered[sl.seq] += sl.len;
        tok += sl.len;
      }
      REQUIRE(tok == chunks[c].tokens);
      std::vector<chunk_attn_seg> segs(chunks[c].num_slices);
      int32_t tq = 0, tkv = 0;
      REQUIRE(chunk_plan_segments(&chunks[c], slices.data(), segs.data(), &tq, &tkv) == CHUNK_ATTN_OK);
      REQUIRE(tq == chunks[c].tokens && tkv == chunks[c].tokens + chunks[c].context);
      chunk_attn_desc d{8, 2, 128, tq, tkv, chunks[c].num_slices, segs.data(), 0.1f};
      REQUIRE(chunk_attn::validate(&d) == CHUNK_ATTN_OK);
      REQUIRE(chunk_attn::pair_count(&d) > 0);
      REQUIRE(!chunk_attn::plan_fwd(&d, 64).empty() && !chunk_attn::plan_dq(&d, 64).empty() && !chunk_attn::plan_dkv(&d, 128).empty());
    }
    for (int s = 0; s < n_seqs; ++s) REQUIRE(covered[s] == lengths[s]);  // every token exactly once
    // ---- scheduler on the chunks just made: units = sequences (split chunks + the chunk with the tail), others alone ----
    const int d_p = uni(1, 6), lay = uni(1, 4);
    std::vector<double> m_ms(d_p, 1e8 * uni(0, 5));
    chunk_sched_mem_model mm{d_p, uni(1, 4), lay * d_p, 34.0 * 4096 * 2 * lay * d_p, 4.0 * 128256, 2.0, 4096.0, 1024.0, 1.0, m_ms.data()};
    std::vector<chunk_sched_chunk> sc;
    std::vector<int32_t> first{0};
    for (int s = 0; s < n_seqs && (int)sc.size() < 60; ++s) {  // units: one per sequence that owns split chunks, then the rest
      int owned = 0;
      for (int c = 0; c < nc; ++c)
        if (chunks[c].is_split && slices[chunks[c].first_slice].seq == s) { sc.push_back({chunks[c].tokens, 1}); ++owned; }
      for (int c = 0; c < nc; ++c)
        if (!chunks[c].is_split && slices[chunks[c].first_slice].seq == s) { sc.push_back({chunks[c].tokens, 0}); ++owned; }
      if (owned) first.push_back((int32_t)sc.size());
    }
    const int n_units = (int)first.size() - 1, n_ch = (int)sc.size();
    REQUIRE(n_units >= 1);
    double peak = 0;
    for (const auto& c : sc) peak = std::max(peak, chunk_sched_act_bytes(&mm, d_p, c.tokens, c.is_split, 0));
    REQUIRE(peak > 0);
    mm.capacity = m_ms[0] + peak * (0.3 + 0.1 * uni(0, 40));  // from 'nothing fits' to 'no checkpointing needed'
    std::vector<int32_t> gou(n_units), order(n_ch), of(n_units + 1), cf(n_units + 1), C(n_ch + n_units * (d_p - 1) + 1);
    int32_t ng = 0, feasible = 0;
    double cost = 0;
    REQUIRE(chunk_sched_group(&mm, sc.data(), first.data(), n_units, 0.01, 1.0 * uni(0, 3), 0.05, gou.data(), &ng, &cost, order.data(),
                              of.data(), C.data(), cf.data(), &feasible) == CHUNK_ATTN_OK);
    if (!feasible) { ++n_infeasible; continue; }
    int64_t csum = 0;
    for (int i = 0; i < cf[ng]; ++i) csum += C[i];
    n_ckpt += csum > 0;
    REQUIRE(ng >= 1 && ng <= n_units && of[ng] == n_ch);
    std::vector<char> seen(n_ch, 0);
    for (int g = 0; g < ng; ++g) {
      const int n = of[g + 1] - of[g];
      REQUIRE(n >= 1 && cf[g + 1] - cf[g] == n + d_p - 1);
      std::vector<int32_t> unit_of(n), f2b(n);
      int n_split = 1;
      for (int k = 0; k < n; ++k) {
        const int ch = order[of[g] + k];
        REQUIRE(ch >= 0 && ch < n_ch && !seen[ch]);
        seen[ch] = 1;
        int u = 0;
        while (first[u + 1] <= ch) ++u;
        REQUIRE(gou[u] == g);
        unit_of[k] = u;
        n_split = std::max(n_split, first[u + 1] - first[u]);
      }
      REQUIRE(chunk_sched_f2b(unit_of.data(), n, f2b.data()) == CHUNK_ATTN_OK);
      // the plan fits: run it through the timeline with the footprints its C implies
      std::vector<double> tf(n, 1.0), tb(n, 2.0), mem((size_t)d_p * n), peak_mem(d_p);
      for (int p = 1; p <= d_p; ++p)
        for (int k = 0; k < n; ++k) {
          const int c = C[cf[g] + f2b[k] + d_p - p];
          REQUIRE(c >= 0 && c <= lay);
          mem[(size_t)(p - 1) * n + k] = chunk_sched_act_bytes(&mm, p, sc[order[of[g] + k]].tokens, sc[order[of[g] + k]].is_split, c);
        }
      double makespan = 0;
      REQUIRE(chunk_sched_simulate(d_p, n, n_split, f2b.data(), tf.data(), tb.data(), nullptr, mem.data(), 0.0, &makespan, nullptr,
                                   peak_mem.data(), nullptr) == CHUNK_ATTN_OK);
      for (int p = 0; p < d_p; ++p) REQUIRE(m_ms[p] + peak_mem[p] <= mm.capacity * (1 + 1e-9));
      REQUIRE(makespan > 0);
    }
    for (int k = 0; k < n_ch; ++k) REQUIRE(seen[k]);
    // ---- the whole solve on the same batch ----
    {
      const int k_max = 1 + uni(0, 3), capb = n_seqs * (k_max + 1);
      std::vector<chunk_plan_chunk> bc(capb);
      std::vector<chunk_plan_slice> bs(capb);
      std::vector<int32_t> pipe(capb), pos(capb), cfb(capb + 1), Cb((size_t)capb * d_p);
      int32_t bk = 0, bnc = 0, bns = 0, bnp = 0, bok = 0;
      double bt = 0;
      REQUIRE(chunk_sched_plan_batch(&cm, &mm, 1 << 20, lengths.data(), n_seqs, 1, k_max, align, 1.0 / 3.0, 0.05, &bk, &bt, bc.data(), capb,
                                     &bnc, bs.data(), capb, &bns, pipe.data(), pos.data(), &bnp, Cb.data(), cfb.data(), &bok) == CHUNK_ATTN_OK);
      if (bok) {
        REQUIRE(bk >= 1 && bk <= k_max && bt > 0 && bnc >= 1 && bnp >= 1);
        std::vector<int> per_pipe(bnp, 0);
        for (int c = 0; c < bnc; ++c) {
          REQUIRE(pipe[c] >= 0 && pipe[c] < bnp && pos[c] >= 0);
          ++per_pipe[pipe[c]];
        }
        for (int g = 0; g < bnp; ++g) REQUIRE(cfb[g + 1] - cfb[g] == per_pipe[g] + d_p - 1);
      }
    }
  }
  std::printf("ok %u cases (%d did not fit, %d needed checkpointing)\n", n_cases, n_infeasible, n_ckpt);
  return 0;
}
