// Seeded random calls into the host-side planner and scheduler, meant to be built with -fsanitize=address,undefined:
// checks memory safety and the structural guarantees of the outputs (no reference values are needed for that).
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "chunk_plan.h"
#include "chunk_sched.h"
#include "../../paper_2509_21275_amd/csrc/plan.hpp"  // the attention library's host-side validation and work-item planning

#define REQUIRE(c) do { if (!(c)) { std::printf("FAILED %s at line %d (seed %u)\n", #c, __LINE__, seed); return 1; } } while (0)

int main(int argc, char** argv) {
  const unsigned n_cases = argc > 1 ? (unsigned)std::atoi(argv[1]) : 200;
  int n_infeasible = 0, n_ckpt = 0;
  for (unsigned seed = 1; seed <= n_cases; ++seed) {
    std::mt19937 rng(seed);
    auto uni = [&](int lo, int hi) { return (int)(rng() % (unsigned)(hi - lo + 1)) + lo; };
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
