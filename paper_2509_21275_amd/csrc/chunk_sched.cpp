// Host-side chunk scheduler: sequence grouping, stage-aware chunk-level checkpointing and a 1F1B timeline
// (paper section 3.4; memory model of sections 3.2.2 and 3.2.3).  See include/chunk_sched.h for the interface and
// for the readings of the points the paper leaves open.
#include "../../include/chunk_sched.h"

#include <algorithm>
#include <cmath>
#include <limits>
#include <numeric>
#include <vector>

namespace {

// branch-and-bound nodes per checkpointing problem: about kNodeWork / (rows * variables), within [kNodeMin, kNodeMax]
constexpr int64_t kNodeMin = 20, kNodeMax = 4000;
constexpr double kNodeWork = 2e7;
constexpr double kEps = 1e-9;

bool model_ok(const chunk_sched_mem_model* m) {
  if (!m || !m->m_ms) return false;
  if (m->d_p < 1 || m->d_p > CHUNK_SCHED_MAX_STAGES || m->d_s < 1 || m->layers < m->d_p || m->layers % m->d_p != 0)
    return false;
  if (!(m->m_token > 0.0) || !(m->m_logits >= 0.0) || !(m->e > 0.0) || !(m->hidden > 0.0) || !(m->kv_hidden >= 0.0) ||
      !(m->capacity > 0.0))
    return false;
  for (int p = 0; p < m->d_p; ++p)
    if (!(m->m_ms[p] >= 0.0)) return false;
  return true;
}

// Coefficients of Algorithm 2 for one chunk: M_act(p, S_k) = I_p[k] - F[k] * ckpt(p, k).
struct Coeff {
  double i_any;   // I[k]
  double i_last;  // I_p[k] on the last stage (adds the logits)
  double f;       // F[k]
};

Coeff coeff(const chunk_sched_mem_model& m, const chunk_sched_chunk& c) {
  const double n_dev = (double)m.d_p * m.d_s, t = (double)c.tokens, split = c.is_split ? 1.0 : 0.0;
  Coeff r;
  r.i_any = (m.m_token / n_dev + split * 2.0 * m.e * m.layers * m.kv_hidden / n_dev) * t;
  r.i_last = r.i_any + m.m_logits / m.d_s * t;
  r.f = (m.m_token / ((double)m.layers * m.d_s) - m.e * (m.hidden + 2.0 * split * m.kv_hidden) / m.d_s) * t;
  return r;
}

bool units_ok(const int32_t* unit_of_chunk, int32_t n) {
  // the chunks of a unit must be adjacent: a unit id never comes back after another one has started
  std::vector<int32_t> seen;
  for (int k = 0; k < n; ++k) {
    if (k > 0 && unit_of_chunk[k] == unit_of_chunk[k - 1]) continue;
    if (std::find(seen.begin(), seen.end(), unit_of_chunk[k]) != seen.end()) return false;
    seen.push_back(unit_of_chunk[k]);
  }
  return true;
}

void f2b_of(const int32_t* unit_of_chunk, int32_t n, int32_t* f2b) {
  for (int start = 0; start < n;) {
    int end = start;
    while (end < n && unit_of_chunk[end] == unit_of_chunk[start]) ++end;
    for (int k = start; k < end; ++k) f2b[k] = start + (end - 1 - k);
    start = end;
  }
}

bool is_permutation(const int32_t* f2b, int32_t n) {
  std::vector<char> hit(n, 0);
  for (int k = 0; k < n; ++k) {
    if (f2b[k] < 0 || f2b[k] >= n || hit[f2b[k]]) return false;
    hit[f2b[k]] = 1;
  }
  return true;
}

// Passes of one stage in order: +k + 1 for the forward pass of chunk k, -(k + 1) for its backward pass.
std::vector<int32_t> stage_passes(int d_p, int p, int n, int n_split, const std::vector<int32_t>& b2f) {
  const int w = std::min(n, d_p - p + n_split);
  std::vector<int32_t> ops;
  ops.reserve(2 * n);
  for (int k = 0; k < w; ++k) ops.push_back(k + 1);
  for (int nf = w, nb = 0; nb < n; ++nb) {
    ops.push_back(-(b2f[nb] + 1));
    if (nf < n) ops.push_back(++nf);
  }
  return ops;
}

std::vector<int32_t> inverse(const int32_t* f2b, int n) {
  std::vector<int32_t> b2f(n);
  for (int k = 0; k < n; ++k) b2f[f2b[k]] = k;
  return b2f;
}

// ---- linear programme  max sum(y)  s.t.  A y <= r, 0 <= y <= ub,  A >= 0, r >= 0  (dictionary simplex) ----
struct Row {
  std::vector<int> idx;
  std::vector<double> a;
  double r;
};

struct Lp {
  int nv = 0;
  std::vector<Row> rows;
};

// Solves the programme with extra bounds lo <= y <= hi.  Returns false if lo alone violates a row.
bool solve_lp(const Lp& lp, const std::vector<int>& lo, const std::vector<int>& hi, std::vector<double>* y, double* z) {
  const int nv = lp.nv, m = (int)lp.rows.size(), rows = m + nv;
  // y = lo + t, 0 <= t <= hi - lo.  Dictionary: basic_i = b[i] - sum_j d[i][j] * nonbasic_j
  std::vector<double> d((size_t)rows * nv, 0.0), b(rows), c(nv, 1.0);
  for (int i = 0; i < m; ++i) {
    double rr = lp.rows[i].r;
    for (size_t q = 0; q < lp.rows[i].idx.size(); ++q) {
      d[(size_t)i * nv + lp.rows[i].idx[q]] = lp.rows[i].a[q];
      rr -= lp.rows[i].a[q] * lo[lp.rows[i].idx[q]];
    }
    if (rr < -kEps) return false;
    b[i] = std::max(rr, 0.0);
  }
  for (int j = 0; j < nv; ++j) {
    d[(size_t)(m + j) * nv + j] = 1.0;
    b[m + j] = hi[j] - lo[j];
    if (b[m + j] < 0) return false;
  }
  std::vector<int> nonbasic(nv), basic(rows);
  for (int j = 0; j < nv; ++j) nonbasic[j] = j;             // structural t_j
  for (int i = 0; i < rows; ++i) basic[i] = nv + i;         // slacks
  double z0 = 0.0;
  const int64_t max_iter = 50LL * (rows + nv) + 1000;
  for (int64_t it = 0; it < max_iter; ++it) {
    const bool bland = it > 4LL * (rows + nv);
    int e = -1;
    for (int j = 0; j < nv; ++j) {
      if (c[j] <= kEps) continue;
      if (e < 0 || (bland ? nonbasic[j] < nonbasic[e] : c[j] > c[e])) e = j;
    }
    if (e < 0) break;
    int l = -1;
    double best = 0.0;
    for (int i = 0; i < rows; ++i) {
      const double a = d[(size_t)i * nv + e];
      if (a <= kEps) continue;
      const double ratio = b[i] / a;
      if (l < 0 || ratio < best - 1e-12 || (ratio <= best + 1e-12 && basic[i] < basic[l])) {
        l = i;
        best = ratio;
      }
    }
    if (l < 0) return false;  // unbounded: cannot happen, every variable has an upper-bound row
    // pivot: entering nonbasic e, leaving basic l
    double* rl = &d[(size_t)l * nv];
    const double piv = rl[e];
    const double inv = 1.0 / piv;
    for (int j = 0; j < nv; ++j) rl[j] *= inv;
    rl[e] = inv;
    b[l] *= inv;
    for (int i = 0; i < rows; ++i) {
      if (i == l) continue;
      double* ri = &d[(size_t)i * nv];
      const double f = ri[e];
      if (f == 0.0) continue;
      for (int j = 0; j < nv; ++j) ri[j] -= f * rl[j];
      ri[e] = -f * inv;
      b[i] -= f * b[l];
      if (b[i] < 0.0) b[i] = 0.0;
    }
    const double ce = c[e];
    for (int j = 0; j < nv; ++j) c[j] -= ce * rl[j];
    c[e] = -ce * inv;
    z0 += ce * b[l];
    std::swap(nonbasic[e], basic[l]);
  }
  y->assign(nv, 0.0);
  for (int i = 0; i < rows; ++i)
    if (basic[i] < nv) (*y)[basic[i]] = b[i];
  double zz = 0.0;
  for (int j = 0; j < nv; ++j) {
    (*y)[j] += lo[j];
    zz += (*y)[j];
  }
  *z = zz;
  (void)z0;
  return true;
}

// Integer programme by best-first branch and bound.  Keeps the best integer y (largest sum) and the largest value
// any unexplored part of the search can still reach.
struct Bnb {
  Lp lp;       // the rows, plus the rounding cuts added at the root
  int ub;
  double gap;  // stop once (best bound - incumbent) <= gap * incumbent, measured on sum(C) = nv * ub - sum(y)
  std::vector<int> best;
  int64_t best_sum = -1;
  int64_t nodes = 0;
  int64_t reach = -1;  // proven: no integer y sums to more than this
  bool cut_short = false;

  struct Node {
    double z;
    std::vector<double> y;
    std::vector<int> lo, hi;
  };

  void offer(const std::vector<double>& ylp, const std::vector<int>& lo, const std::vector<int>& hi) {
    // rounding down keeps a packing problem feasible; then raise variables while the rows hold, those the
    // relaxation had closest to the next integer first
    const int nv = lp.nv;
    std::vector<int> y(nv), by_frac(nv);
    std::vector<double> frac(nv);
    for (int j = 0; j < nv; ++j) {
      const double fl = std::floor(ylp[j] + 1e-7);
      y[j] = std::min(hi[j], std::max(lo[j], (int)fl));
      frac[j] = ylp[j] - fl;
      by_frac[j] = j;
    }
    std::stable_sort(by_frac.begin(), by_frac.end(), [&](int a, int b) { return frac[a] > frac[b]; });
    std::vector<double> lhs(lp.rows.size(), 0.0);
    for (size_t i = 0; i < lp.rows.size(); ++i)
      for (size_t q = 0; q < lp.rows[i].idx.size(); ++q) lhs[i] += lp.rows[i].a[q] * y[lp.rows[i].idx[q]];
    // rows that contain a variable
    std::vector<std::vector<std::pair<int, double>>> of_var(nv);
    for (size_t i = 0; i < lp.rows.size(); ++i)
      for (size_t q = 0; q < lp.rows[i].idx.size(); ++q) of_var[lp.rows[i].idx[q]].push_back({(int)i, lp.rows[i].a[q]});
    bool grew = true;
    while (grew) {
      grew = false;
      for (int j : by_frac) {
        if (y[j] >= ub) continue;
        bool fits = true;
        for (const auto& ra : of_var[j])
          if (lhs[ra.first] + ra.second > lp.rows[ra.first].r * (1.0 + 1e-12) + 1e-12) {
            fits = false;
            break;
          }
        if (!fits) continue;
        ++y[j];
        for (const auto& ra : of_var[j]) lhs[ra.first] += ra.second;
        grew = true;
      }
    }
    int64_t s = std::accumulate(y.begin(), y.end(), (int64_t)0);
    if (s + 1 >= best_sum) {
      // exchange: lower one variable and raise two that share a row with it (net + 1), until nothing is gained
      auto fits = [&](int j) {
        if (y[j] >= ub) return false;
        for (const auto& ra : of_var[j])
          if (lhs[ra.first] + ra.second > lp.rows[ra.first].r * (1.0 + 1e-12) + 1e-12) return false;
        return true;
      };
      auto bump = [&](int j, int by) {
        y[j] += by;
        for (const auto& ra : of_var[j]) lhs[ra.first] += by * ra.second;
      };
      std::vector<std::vector<int>> near(nv);
      for (int j = 0; j < nv; ++j) {
        std::vector<char> hit(nv, 0);
        for (const auto& ra : of_var[j])
          for (int q : lp.rows[ra.first].idx) hit[q] = 1;
        for (int q = 0; q < nv; ++q)
          if (hit[q] && q != j) near[j].push_back(q);
      }
      bool gained = true;
      while (gained) {
        gained = false;
        for (int a0 = 0; a0 < nv && !gained; ++a0) {
          if (y[a0] <= 0) continue;
          bump(a0, -1);
          for (size_t bi = 0; bi < near[a0].size() && !gained; ++bi) {
            const int b0 = near[a0][bi];
            if (!fits(b0)) continue;
            bump(b0, 1);
            for (size_t ci = bi; ci < near[a0].size(); ++ci)
              if (fits(near[a0][ci])) {
                bump(near[a0][ci], 1);
                gained = true;
                break;
              }
            if (!gained) bump(b0, -1);
          }
          if (!gained) bump(a0, 1);
        }
        if (gained) ++s;
      }
    }
    if (s > best_sum) {
      best_sum = s;
      best = y;
    }
  }

  // Rounding cuts from the rows the relaxation's solution sits on: a row  sum a_j c_j >= need  over integers c gives
  // sum ceil(a_j / d) c_j >= ceil(need / d)  for any d > 0; with c = ub - y that is again a packing row.
  int add_cuts(const std::vector<double>& y, size_t n_orig) {
    int added = 0;
    for (size_t i = 0; i < n_orig; ++i) {
      const Row row = lp.rows[i];  // a copy: the cuts appended below may move the rows
      double asum = 0.0;
      for (double a : row.a) asum += a;
      const double need = ub * asum - row.r;
      if (need <= 0.0) continue;
      std::vector<double> ds = row.a;
      std::sort(ds.begin(), ds.end());
      ds.erase(std::unique(ds.begin(), ds.end()), ds.end());
      for (double dv : ds) {
        Row cut;
        double gsum = 0.0, at_y = 0.0;
        for (size_t q = 0; q < row.idx.size(); ++q) {
          const double g = std::ceil(row.a[q] / dv);
          cut.idx.push_back(row.idx[q]);
          cut.a.push_back(g);
          gsum += g;
          at_y += g * y[row.idx[q]];
        }
        cut.r = ub * gsum - std::ceil(need / dv - 1e-9);
        if (cut.r < 0.0) cut.r = 0.0;
        if (at_y > cut.r + 1e-6) {
          lp.rows.push_back(std::move(cut));
          ++added;
        }
      }
    }
    return added;
  }

  void run() {
    const int nv = lp.nv;
    const int64_t total = (int64_t)nv * ub;
    Node root;
    root.lo.assign(nv, 0);
    root.hi.assign(nv, ub);
    if (!solve_lp(lp, root.lo, root.hi, &root.y, &root.z)) return;
    const size_t n_orig = lp.rows.size();
    for (int round = 0; round < 20; ++round) {
      if (add_cuts(root.y, n_orig) == 0) break;
      if (!solve_lp(lp, root.lo, root.hi, &root.y, &root.z)) return;
    }
    ++nodes;
    offer(root.y, root.lo, root.hi);
    const int64_t node_limit = std::max(
        kNodeMin, std::min(kNodeMax, (int64_t)(kNodeWork / ((double)(lp.rows.size() + nv) * nv))));
    auto worse = [](const Node& a, const Node& b) { return a.z < b.z; };
    std::vector<Node> heap;
    heap.push_back(std::move(root));
    while (!heap.empty()) {
      std::pop_heap(heap.begin(), heap.end(), worse);
      Node nd = std::move(heap.back());
      heap.pop_back();
      const int64_t bound = (int64_t)std::floor(nd.z + 1e-6);  // no unexplored node can do better
      if (bound <= best_sum) break;
      reach = bound;
      if ((double)(bound - best_sum) <= gap * (double)(total - best_sum)) break;
      if (nodes >= node_limit) {
        cut_short = true;
        break;
      }
      reach = -1;
      int branch = -1;
      double frac_best = 0.0;
      for (int j = 0; j < nv; ++j) {
        const double fr = nd.y[j] - std::floor(nd.y[j] + 1e-7);
        const double dist = std::min(fr, 1.0 - fr);
        if (fr > 1e-7 && fr < 1.0 - 1e-7 && dist > frac_best) {
          frac_best = dist;
          branch = j;
        }
      }
      if (branch < 0) continue;  // integral: offer() recorded it when the node was made
      const int fl = (int)std::floor(nd.y[branch] + 1e-7);
      for (int side = 0; side < 2; ++side) {
        Node ch;
        ch.lo = nd.lo;
        ch.hi = nd.hi;
        if (side == 0) ch.lo[branch] = fl + 1;
        else ch.hi[branch] = fl;
        if (ch.lo[branch] > ch.hi[branch]) continue;
        ++nodes;
        if (!solve_lp(lp, ch.lo, ch.hi, &ch.y, &ch.z)) continue;
        offer(ch.y, ch.lo, ch.hi);
        if ((int64_t)std::floor(ch.z + 1e-6) <= best_sum) continue;
        heap.push_back(std::move(ch));
        std::push_heap(heap.begin(), heap.end(), worse);
      }
    }
    if (reach < best_sum) reach = best_sum;  // the search ran out: the incumbent is the best there is
  }
};

// Checkpointing of one pipeline.  Returns 1 feasible, 0 infeasible, negative error.
int solve_pipeline(const chunk_sched_mem_model& m, const std::vector<chunk_sched_chunk>& chunks,
                   const std::vector<int32_t>& unit_of, int n_split, double gap, std::vector<int32_t>* C, int64_t* sum,
                   int64_t* nodes, int64_t* lower_bound) {
  const int n = (int)chunks.size(), d_p = m.d_p, nv = n + d_p - 1, u = m.layers / d_p;
  std::vector<int32_t> f2b(n);
  f2b_of(unit_of.data(), n, f2b.data());
  const std::vector<int32_t> b2f = inverse(f2b.data(), n);
  std::vector<Coeff> co(n);
  for (int k = 0; k < n; ++k) {
    co[k] = coeff(m, chunks[k]);
    if (!(co[k].f > 0.0)) return CHUNK_ATTN_INVALID_ARG;  // a checkpointed layer must free memory
  }
  Lp lp;
  lp.nv = nv;
  for (int p = 1; p <= d_p; ++p) {
    const double cap = m.capacity - m.m_ms[p - 1];
    const std::vector<int32_t> ops = stage_passes(d_p, p, n, n_split, b2f);
    const int w = std::min(n, d_p - p + n_split);
    std::vector<int> live;
    int n_fwd = 0;
    for (int32_t op : ops) {
      if (op < 0) {
        live.erase(std::find(live.begin(), live.end(), -op - 1));
        continue;
      }
      live.push_back(op - 1);
      if (++n_fwd < w) continue;
      // window: sum_k (I_p[k] - F[k] c_k) <= cap, with c = u - y:  sum_k F[k] y_k <= cap - sum_k (I_p[k] - F[k] u)
      Row row;
      double need = -cap, fsum = 0.0, amax = 0.0;
      for (int k : live) {
        need += p == d_p ? co[k].i_last : co[k].i_any;
        fsum += co[k].f;
        amax = std::max(amax, co[k].f);
        row.idx.push_back(f2b[k] + d_p - p);
        row.a.push_back(co[k].f);
      }
      if (need <= 0.0) continue;  // fits without any checkpointing
      row.r = u * fsum - need;
      if (row.r < -1e-9 * std::abs(need)) return 0;  // does not fit with every layer checkpointed
      row.r = std::max(row.r, 0.0);
      for (double& a : row.a) a /= amax;
      row.r /= amax;
      lp.rows.push_back(std::move(row));
    }
  }
  Bnb bnb;
  bnb.ub = u;
  bnb.gap = gap;
  if (lp.rows.empty()) {
    bnb.best.assign(nv, u);
    bnb.best_sum = bnb.reach = (int64_t)nv * u;
  } else {
    bnb.lp = std::move(lp);
    bnb.run();
  }
  if (bnb.best_sum < 0) return CHUNK_ATTN_INVALID_ARG;  // cannot happen: y = 0 is feasible here
  C->resize(nv);
  int64_t s = 0;
  for (int j = 0; j < nv; ++j) {
    (*C)[j] = u - bnb.best[j];
    s += (*C)[j];
  }
  *sum = s;
  if (nodes) *nodes = bnb.cut_short ? -bnb.nodes : bnb.nodes;
  if (lower_bound) *lower_bound = (int64_t)nv * u - bnb.reach;
  return 1;
}

}  // namespace

extern "C" {

double chunk_sched_act_bytes(const chunk_sched_mem_model* model, int32_t p, int32_t tokens, int32_t is_split,
                             int32_t l_ckpt) {
  if (!model_ok(model) || p < 1 || p > model->d_p || tokens < 0 || l_ckpt < 0 || l_ckpt > model->layers / model->d_p)
    return -1.0;
  const Coeff c = coeff(*model, chunk_sched_chunk{tokens, is_split});
  return (p == model->d_p ? c.i_last : c.i_any) - c.f * l_ckpt;
}

int chunk_sched_f2b(const int32_t* unit_of_chunk, int32_t n, int32_t* f2b) {
  if (!unit_of_chunk || !f2b || n < 1 || !units_ok(unit_of_chunk, n)) return CHUNK_ATTN_INVALID_ARG;
  f2b_of(unit_of_chunk, n, f2b);
  return CHUNK_ATTN_OK;
}

int chunk_sched_windows(int32_t d_p, int32_t p, int32_t n, int32_t n_split, const int32_t* f2b, int32_t* windows,
                        int32_t* n_windows, int32_t* width) {
  if (!f2b || !windows || !n_windows || !width || d_p < 1 || d_p > CHUNK_SCHED_MAX_STAGES || p < 1 || p > d_p || n < 1 ||
      n_split < 1 || n_split > n || !is_permutation(f2b, n))
    return CHUNK_ATTN_INVALID_ARG;
  const std::vector<int32_t> b2f = inverse(f2b, n);
  const int w = std::min(n, d_p - p + n_split);
  std::vector<int32_t> live;
  int n_fwd = 0, out = 0;
  for (int32_t op : stage_passes(d_p, p, n, n_split, b2f)) {
    if (op < 0) {
      auto it = std::find(live.begin(), live.end(), -op - 1);
      if (it == live.end()) return CHUNK_ATTN_INVALID_ARG;  // a backward pass before its forward pass
      live.erase(it);
      continue;
    }
    live.push_back(op - 1);
    if (++n_fwd < w) continue;
    std::vector<int32_t> sorted = live;
    std::sort(sorted.begin(), sorted.end());
    for (int32_t k : sorted) windows[out++] = k;
  }
  *width = w;
  *n_windows = n - w + 1;
  return CHUNK_ATTN_OK;
}

int chunk_sched_solve_ckpt(const chunk_sched_mem_model* model, const chunk_sched_chunk* chunks,
                           const int32_t* unit_of_chunk, int32_t n, int32_t n_split, double gap, int32_t* C,
                           int64_t* sum, int32_t* feasible, int64_t* nodes, int64_t* lower_bound) {
  if (!model_ok(model) || !chunks || !unit_of_chunk || !C || !sum || !feasible || n < 1 || n > CHUNK_SCHED_MAX_CHUNKS ||
      n_split < 1 || n_split > n || !(gap >= 0.0) || !units_ok(unit_of_chunk, n))
    return CHUNK_ATTN_INVALID_ARG;
  for (int k = 0; k < n; ++k)
    if (chunks[k].tokens < 1) return CHUNK_ATTN_INVALID_ARG;
  std::vector<chunk_sched_chunk> cs(chunks, chunks + n);
  std::vector<int32_t> unit_of(unit_of_chunk, unit_of_chunk + n), sol;
  int64_t s = 0;
  if (nodes) *nodes = 0;
  const int rc = solve_pipeline(*model, cs, unit_of, n_split, gap, &sol, &s, nodes, lower_bound);
  if (rc < 0) return rc;
  *feasible = rc;
  if (rc == 1) {
    std::copy(sol.begin(), sol.end(), C);
    *sum = s;
  }
  return CHUNK_ATTN_OK;
}

int chunk_sched_group(const chunk_sched_mem_model* model, const chunk_sched_chunk* chunks, const int32_t* unit_first,
                      int32_t n_units, double layer_fwd_time, double delta, double gap, int32_t* group_of_unit,
                      int32_t* n_groups, double* cost, int32_t* order, int32_t* order_first, int32_t* C, int32_t* c_first,
                      int32_t* feasible) {
  if (!model_ok(model) || !chunks || !unit_first || !group_of_unit || !n_groups || !cost || !order || !order_first || !C ||
      !c_first || !feasible || n_units < 1 || !(layer_fwd_time >= 0.0) || !(delta >= 0.0) || !(gap >= 0.0) ||
      unit_first[0] != 0)
    return CHUNK_ATTN_INVALID_ARG;
  for (int u = 0; u < n_units; ++u)
    if (unit_first[u + 1] <= unit_first[u]) return CHUNK_ATTN_INVALID_ARG;
  const int n_chunks = unit_first[n_units];
  for (int k = 0; k < n_chunks; ++k)
    if (chunks[k].tokens < 1) return CHUNK_ATTN_INVALID_ARG;
  auto count_of = [&](int u) { return unit_first[u + 1] - unit_first[u]; };
  auto tokens_of = [&](int u) {
    int64_t t = 0;
    for (int k = unit_first[u]; k < unit_first[u + 1]; ++k) t += chunks[k].tokens;
    return t;
  };
  std::vector<int> counts;
  for (int u = 0; u < n_units; ++u) counts.push_back(count_of(u));
  std::sort(counts.begin(), counts.end());
  counts.erase(std::unique(counts.begin(), counts.end()), counts.end());
  const int m = (int)counts.size();

  struct Plan {
    bool ok = false;
    double cost = 0.0;
    std::vector<int> units;       // in pipeline order
    std::vector<int32_t> C;
  };
  // pipeline of the units whose chunk count lies in counts[a .. b)
  auto plan_range = [&](int a, int b, Plan* out) -> int {
    std::vector<int> us;
    for (int u = 0; u < n_units; ++u)
      if (count_of(u) >= counts[a] && count_of(u) <= counts[b - 1]) us.push_back(u);
    std::stable_sort(us.begin(), us.end(), [&](int x, int y) {
      if (count_of(x) != count_of(y)) return count_of(x) > count_of(y);
      return tokens_of(x) > tokens_of(y);
    });
    std::vector<chunk_sched_chunk> cs;
    std::vector<int32_t> unit_of;
    for (size_t j = 0; j < us.size(); ++j)
      for (int k = unit_first[us[j]]; k < unit_first[us[j] + 1]; ++k) {
        cs.push_back(chunks[k]);
        unit_of.push_back((int32_t)j);
      }
    if ((int)cs.size() > CHUNK_SCHED_MAX_CHUNKS) return CHUNK_ATTN_INVALID_ARG;
    int64_t s = 0;
    const int rc = solve_pipeline(*model, cs, unit_of, counts[b - 1], gap, &out->C, &s, nullptr, nullptr);
    if (rc < 0) return rc;
    out->ok = rc == 1;
    out->cost = delta + layer_fwd_time * (double)s;
    out->units = us;
    return CHUNK_ATTN_OK;
  };

  const double inf = std::numeric_limits<double>::infinity();
  std::vector<double> dp(m + 1, inf);
  std::vector<int> from(m + 1, -1);
  std::vector<std::vector<Plan>> plans(m + 1, std::vector<Plan>(m + 1));
  dp[0] = 0.0;
  for (int i = 1; i <= m; ++i)
    for (int k = 0; k < i; ++k) {
      if (dp[k] == inf) continue;
      const int rc = plan_range(k, i, &plans[k][i]);
      if (rc != CHUNK_ATTN_OK) return rc;
      if (!plans[k][i].ok) continue;
      const double c = dp[k] + plans[k][i].cost;
      if (c < dp[i] - 1e-12 * std::max(1.0, std::abs(c))) {
        dp[i] = c;
        from[i] = k;
      }
    }
  if (dp[m] == inf) {
    *feasible = 0;
    return CHUNK_ATTN_OK;
  }
  std::vector<std::pair<int, int>> ranges;
  for (int i = m; i > 0; i = from[i]) ranges.push_back({from[i], i});
  std::reverse(ranges.begin(), ranges.end());
  int no = 0, nc = 0;
  for (size_t g = 0; g < ranges.size(); ++g) {
    const Plan& pl = plans[ranges[g].first][ranges[g].second];
    order_first[g] = no;
    c_first[g] = nc;
    for (int u : pl.units) {
      group_of_unit[u] = (int32_t)g;
      for (int k = unit_first[u]; k < unit_first[u + 1]; ++k) order[no++] = k;
    }
    for (int32_t c : pl.C) C[nc++] = c;
  }
  order_first[ranges.size()] = no;
  c_first[ranges.size()] = nc;
  *n_groups = (int32_t)ranges.size();
  *cost = dp[m];
  *feasible = 1;
  return CHUNK_ATTN_OK;
}

int chunk_sched_simulate(int32_t d_p, int32_t n, int32_t n_split, const int32_t* f2b, const double* t_fwd,
                         const double* t_bwd, const double* t_recomp, const double* mem, double p2p, double* makespan,
                         double* busy, double* peak_mem, int32_t* peak_held) {
  if (!f2b || !t_fwd || !t_bwd || d_p < 1 || d_p > CHUNK_SCHED_MAX_STAGES || n < 1 || n_split < 1 || n_split > n ||
      !(p2p >= 0.0) || !is_permutation(f2b, n))
    return CHUNK_ATTN_INVALID_ARG;
  const std::vector<int32_t> b2f = inverse(f2b, n);
  std::vector<std::vector<int32_t>> ops(d_p);
  for (int p = 1; p <= d_p; ++p) ops[p - 1] = stage_passes(d_p, p, n, n_split, b2f);
  const double unset = -1.0;
  std::vector<double> f_end((size_t)d_p * n, unset), b_end((size_t)d_p * n, unset), free_at(d_p, 0.0), work(d_p, 0.0);
  std::vector<size_t> next(d_p, 0);
  std::vector<double> cur_mem(d_p, 0.0), top_mem(d_p, 0.0);
  std::vector<int32_t> cur_held(d_p, 0), top_held(d_p, 0);
  size_t left = (size_t)d_p * 2 * n;
  while (left > 0) {
    bool moved = false;
    for (int s = 0; s < d_p; ++s) {
      while (next[s] < ops[s].size()) {
        const int32_t op = ops[s][next[s]];
        const int k = (op > 0 ? op : -op) - 1;
        double ready = free_at[s], dur;
        if (op > 0) {
          if (s > 0) {
            if (f_end[(size_t)(s - 1) * n + k] == unset) break;
            ready = std::max(ready, f_end[(size_t)(s - 1) * n + k] + p2p);
          }
          dur = t_fwd[k];
        } else {
          if (f_end[(size_t)s * n + k] == unset) return CHUNK_ATTN_INVALID_ARG;  // backward before forward
          if (s + 1 < d_p) {
            if (b_end[(size_t)(s + 1) * n + k] == unset) break;
            ready = std::max(ready, b_end[(size_t)(s + 1) * n + k] + p2p);
          }
          dur = t_bwd[k] + (t_recomp ? t_recomp[(size_t)s * n + k] : 0.0);
        }
        if (!(dur >= 0.0)) return CHUNK_ATTN_INVALID_ARG;
        const double done = ready + dur;
        if (op > 0) {
          f_end[(size_t)s * n + k] = done;
          cur_mem[s] += mem ? mem[(size_t)s * n + k] : 0.0;
          top_mem[s] = std::max(top_mem[s], cur_mem[s]);
          top_held[s] = std::max(top_held[s], ++cur_held[s]);
        } else {
          b_end[(size_t)s * n + k] = done;
          cur_mem[s] -= mem ? mem[(size_t)s * n + k] : 0.0;
          --cur_held[s];
        }
        free_at[s] = done;
        work[s] += dur;
        ++next[s];
        --left;
        moved = true;
      }
    }
    if (!moved) return CHUNK_ATTN_INVALID_ARG;  // the orders wait for each other
  }
  if (makespan) *makespan = *std::max_element(free_at.begin(), free_at.end());
  for (int s = 0; s < d_p; ++s) {
    if (busy) busy[s] = work[s];
    if (peak_mem) peak_mem[s] = top_mem[s];
    if (peak_held) peak_held[s] = top_held[s];
  }
  return CHUNK_ATTN_OK;
}

int chunk_sched_plan_batch(const chunk_cost_model* cost, const chunk_sched_mem_model* mem, int64_t token_capacity,
                           const int32_t* lengths, int32_t n_seqs, int32_t k_min, int32_t k_max, int32_t align,
                           double fwd_fraction, double gap, int32_t* best_k, double* est_time, chunk_plan_chunk* chunks,
                           int32_t max_chunks, int32_t* n_chunks, chunk_plan_slice* slices, int32_t max_slices,
                           int32_t* n_slices, int32_t* pipeline_of_chunk, int32_t* fwd_pos_of_chunk,
                           int32_t* n_pipelines, int32_t* C, int32_t* c_first, int32_t* feasible) {
  if (!cost || !model_ok(mem) || !lengths || !best_k || !est_time || !chunks || !n_chunks || !slices || !n_slices ||
      !pipeline_of_chunk || !fwd_pos_of_chunk || !n_pipelines || !C || !c_first || !feasible || n_seqs < 1 || k_min < 1 ||
      k_max < k_min || align < 1 || token_capacity < 1 || !(fwd_fraction > 0.0) || !(fwd_fraction < 1.0) || !(gap >= 0.0))
    return CHUNK_ATTN_INVALID_ARG;
  const int d_p = mem->d_p;
  const double per_stage = (double)mem->layers / d_p;
  struct Best {
    bool ok = false;
    int k = 0;
    double time = 0.0;
    std::vector<chunk_plan_chunk> chunks;
    std::vector<chunk_plan_slice> slices;
    std::vector<int32_t> pipe, pos, C, c_first;
    int n_pipes = 0;
  } best;
  for (int K = k_min; K <= k_max; ++K) {
    const int cap = n_seqs * (K + 1);
    std::vector<chunk_plan_chunk> ch(cap);
    std::vector<chunk_plan_slice> sl(cap);
    int32_t nc = 0, ns = 0;
    int rc = chunk_plan_build(cost, token_capacity, lengths, n_seqs, K, align, ch.data(), cap, &nc, sl.data(), cap, &ns,
                              nullptr, nullptr);
    if (rc != CHUNK_ATTN_OK) return rc;
    ch.resize(nc);
    sl.resize(ns);
    // sequences as the scheduler sees them
    std::vector<std::vector<int>> units;
    {
      std::vector<std::vector<int>> split_of(n_seqs);
      for (int c = 0; c < nc; ++c)
        if (ch[c].is_split) split_of[sl[ch[c].first_slice].seq].push_back(c);
      for (auto& v : split_of)
        std::sort(v.begin(), v.end(), [&](int a, int b) { return ch[a].context < ch[b].context; });
      for (int c = 0; c < nc; ++c) {
        if (ch[c].is_split) continue;
        std::vector<int> u;
        if (ch[c].context > 0) {
          std::vector<int>& head = split_of[sl[ch[c].first_slice].seq];
          u = head;
          head.clear();
        }
        u.push_back(c);
        units.push_back(u);
      }
      for (const auto& v : split_of)
        if (!v.empty()) return CHUNK_ATTN_INVALID_ARG;  // a split chunk without its tail: cannot happen
    }
    std::vector<chunk_sched_chunk> sc;
    std::vector<int32_t> first{0}, chunk_of;  // chunk_of[i]: planner chunk behind scheduler chunk i
    double sum_t = 0.0;
    for (const auto& u : units) {
      for (int c : u) {
        sc.push_back(chunk_sched_chunk{ch[c].tokens, ch[c].is_split});
        chunk_of.push_back(c);
        sum_t += ch[c].time;
      }
      first.push_back((int32_t)sc.size());
    }
    const int n_units = (int)units.size();
    const double mean_t = sum_t / nc;
    const double delta = (d_p - 1) * mean_t * per_stage, f_hat = fwd_fraction * mean_t;
    std::vector<int32_t> gou(n_units), order(nc), of(n_units + 1), cf(n_units + 1), Cv((size_t)nc + (size_t)n_units * (d_p - 1) + 1);
    int32_t ng = 0, ok = 0;
    double cost_g = 0.0;
    rc = chunk_sched_group(mem, sc.data(), first.data(), n_units, f_hat, delta, gap, gou.data(), &ng, &cost_g, order.data(),
                           of.data(), Cv.data(), cf.data(), &ok);
    if (rc != CHUNK_ATTN_OK) return rc;
    if (!ok) continue;
    const double total = sum_t * per_stage + cost_g;
    if (best.ok && !(total < best.time * (1.0 - 1e-12))) continue;
    best.ok = true;
    best.k = K;
    best.time = total;
    best.chunks = ch;
    best.slices = sl;
    best.n_pipes = ng;
    best.pipe.assign(nc, -1);
    best.pos.assign(nc, -1);
    for (int g = 0; g < ng; ++g)
      for (int i = of[g]; i < of[g + 1]; ++i) {
        best.pipe[chunk_of[order[i]]] = g;
        best.pos[chunk_of[order[i]]] = i - of[g];
      }
    best.C.assign(Cv.begin(), Cv.begin() + cf[ng]);
    best.c_first.assign(cf.begin(), cf.begin() + ng + 1);
  }
  if (!best.ok) {
    *feasible = 0;
    return CHUNK_ATTN_OK;
  }
  if ((int)best.chunks.size() > max_chunks || (int)best.slices.size() > max_slices) return CHUNK_ATTN_INVALID_ARG;
  std::copy(best.chunks.begin(), best.chunks.end(), chunks);
  std::copy(best.slices.begin(), best.slices.end(), slices);
  std::copy(best.pipe.begin(), best.pipe.end(), pipeline_of_chunk);
  std::copy(best.pos.begin(), best.pos.end(), fwd_pos_of_chunk);
  std::copy(best.C.begin(), best.C.end(), C);
  std::copy(best.c_first.begin(), best.c_first.end(), c_first);
  *n_chunks = (int32_t)best.chunks.size();
  *n_slices = (int32_t)best.slices.size();
  *n_pipelines = best.n_pipes;
  *best_k = best.k;
  *est_time = best.time;
  *feasible = 1;
  return CHUNK_ATTN_OK;
}

}  // extern "C"
