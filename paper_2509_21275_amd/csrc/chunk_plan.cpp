// Host-side sequence processor (include/chunk_plan.h): the paper's Algorithm 1 with its cost model.
// Pure C++, no HIP.
#include "../../include/chunk_plan.h"

#include <algorithm>
#include <cmath>
#include <vector>

namespace {

bool model_ok(const chunk_cost_model* m) {
  return m && m->alpha1 > 0.0 && m->alpha2 >= 0.0 && m->beta1 >= 0.0 && m->a2a_per_token >= 0.0 && m->a2a_const >= 0.0 &&
         m->n_devices >= 1 && m->dp >= 1;
}

// cost of one slice of length s behind a context of C tokens, without the per-chunk constants
double slice_cost(const chunk_cost_model& m, double C, double s) {
  return (m.alpha1 * ((C + s) * (C + s) - C * C) + m.alpha2 * s) / m.n_devices + m.a2a_per_token * s;
}
double chunk_const(const chunk_cost_model& m) { return m.beta1 / m.dp + m.a2a_const; }

// largest real s with slice_cost(C, s) <= budget (the cost is a quadratic a s^2 + b s in s)
double slice_for_budget(const chunk_cost_model& m, double C, double budget) {
  const double a = m.alpha1 / m.n_devices;
  const double b = (2.0 * m.alpha1 * C + m.alpha2) / m.n_devices + m.a2a_per_token;
  if (budget <= 0.0) return 0.0;
  return (-b + std::sqrt(b * b + 4.0 * a * budget)) / (2.0 * a);
}

struct Bucket {
  int64_t context = 0;
  int tail = -1;            // index into `items` of the tail slice, or -1
  std::vector<int> shorts;  // indices into `items`
  double cost = 0.0;        // sum of slice costs (no constants)
  int64_t tokens = 0;
  int order = 0;            // creation order (tie break)
  double metric(double constant) const { return (cost + constant) / (double)tokens; }  // tot_time / tot_tokens
};

struct Item {  // a tail slice or a short sequence
  int seq, start, len;
  int64_t context;
  double cost;
};

}  // namespace

extern "C" {

double chunk_plan_time(const chunk_cost_model* model, int64_t context, const int32_t* slice_lens, int32_t n) {
  if (!model_ok(model) || !slice_lens || n < 1 || context < 0) return -1.0;
  double t = slice_cost(*model, (double)context, (double)slice_lens[0]);
  for (int i = 1; i < n; ++i) t += slice_cost(*model, 0.0, (double)slice_lens[i]);
  return t + chunk_const(*model);
}

int chunk_plan_mesh(const chunk_cost_model* model, int32_t max_len, int32_t K, int32_t align, int64_t capacity,
                    int32_t* mesh, int32_t* k_out, double* time_threshold, int64_t* token_threshold) {
  if (!model_ok(model) || !mesh || !k_out || max_len < 1 || K < 1 || align < 1 || capacity < 1)
    return CHUNK_ATTN_INVALID_ARG;
  const chunk_cost_model& m = *model;
  K = std::max(1, std::min<int32_t>(K, max_len / align));
  // Find the slice budget for which K - 1 aligned slices leave a last slice that costs no more than they do:
  // bisection on the budget (the total length covered grows with it).
  auto lay_out = [&](double budget, std::vector<int32_t>& out) {
    out.clear();
    int64_t pos = 0;
    for (int k = 0; k + 1 < K; ++k) {
      int64_t s = (int64_t)std::floor(slice_for_budget(m, (double)pos, budget));
      s = s / align * align;
      s = std::max<int64_t>(s, align);
      s = std::min<int64_t>(s, max_len - pos - (int64_t)(K - 1 - k) * align);  // leave room for the slices behind
      out.push_back((int32_t)s);
      pos += s;
    }
    out.push_back((int32_t)(max_len - pos));
    return slice_cost(m, (double)pos, (double)(max_len - pos));  // cost of the last slice
  };
  std::vector<int32_t> cur;
  double lo = 0.0, hi = slice_cost(m, 0.0, (double)max_len);
  for (int it = 0; it < 100; ++it) {
    const double mid = 0.5 * (lo + hi);
    const double last = lay_out(mid, cur);
    if (last > mid) lo = mid; else hi = mid;  // last slice too expensive: the others must take more
  }
  lay_out(hi, cur);
  double tmax = 0.0;
  int64_t pos = 0;
  for (int k = 0; k < K; ++k) {
    mesh[k] = cur[k];
    tmax = std::max(tmax, slice_cost(m, (double)pos, (double)cur[k]) + chunk_const(m));
    pos += cur[k];
  }
  *k_out = K;
  if (time_threshold) *time_threshold = tmax;
  if (token_threshold) *token_threshold = std::min<int64_t>(capacity, mesh[0]);
  return CHUNK_ATTN_OK;
}

int chunk_plan_build(const chunk_cost_model* model, int64_t capacity, const int32_t* lengths, int32_t n_seqs, int32_t K,
                     int32_t align, chunk_plan_chunk* chunks, int32_t max_chunks, int32_t* n_chunks,
                     chunk_plan_slice* slices, int32_t max_slices, int32_t* n_slices, double* time_threshold,
                     int64_t* token_threshold) {
  if (!model_ok(model) || !lengths || !chunks || !n_chunks || !slices || !n_slices || n_seqs < 1 || K < 1 ||
      align < 1 || capacity < 1)
    return CHUNK_ATTN_INVALID_ARG;
  const chunk_cost_model& m = *model;
  int32_t max_len = 0;
  for (int i = 0; i < n_seqs; ++i) {
    if (lengths[i] < 1) return CHUNK_ATTN_INVALID_ARG;
    max_len = std::max(max_len, lengths[i]);
  }
  // mesh and thresholds
  std::vector<int32_t> mesh(K);
  int32_t k_eff = 0;
  double T_t = 0.0;
  int64_t T_m = 0;
  int rc = chunk_plan_mesh(model, max_len, K, align, capacity, mesh.data(), &k_eff, &T_t, &T_m);
  if (rc != CHUNK_ATTN_OK) return rc;
  mesh.resize(k_eff);

  int nc = 0, ns = 0;
  auto push_chunk = [&](int64_t ctx, int first, int count, int is_split, int64_t tokens, double time) {
    if (nc >= max_chunks) return false;
    chunks[nc++] = chunk_plan_chunk{ctx, first, count, is_split, (int32_t)tokens, time};
    return true;
  };
  auto push_slice = [&](int seq, int start, int len) {
    if (ns >= max_slices) return false;
    slices[ns++] = chunk_plan_slice{seq, start, len};
    return true;
  };

  // splitting: a sequence longer than the first j mesh slices together gives j split chunks and a tail slice;
  // a sequence no longer than mesh[0] is "short"
  std::vector<Item> items;
  std::vector<int> tails, shorts;
  for (int i = 0; i < n_seqs; ++i) {
    int64_t pos = 0;
    int k = 0;
    while (k < k_eff && pos + mesh[k] < lengths[i]) {
      if (!push_slice(i, (int)pos, mesh[k])) return CHUNK_ATTN_INVALID_ARG;
      if (!push_chunk(pos, ns - 1, 1, 1, mesh[k], slice_cost(m, (double)pos, (double)mesh[k]) + chunk_const(m)))
        return CHUNK_ATTN_INVALID_ARG;
      pos += mesh[k];
      ++k;
    }
    Item it{i, (int)pos, (int)(lengths[i] - pos), pos, slice_cost(m, (double)pos, (double)(lengths[i] - pos))};
    items.push_back(it);
    (pos > 0 ? tails : shorts).push_back((int)items.size() - 1);
  }

  // one bucket per tail slice (two tail slices never share a chunk); short sequences by decreasing time
  std::vector<Bucket> buckets;
  for (int t : tails) {
    Bucket b;
    b.context = items[t].context; b.tail = t; b.cost = items[t].cost; b.tokens = items[t].len; b.order = (int)buckets.size();
    buckets.push_back(b);
  }
  std::stable_sort(shorts.begin(), shorts.end(), [&](int a, int b) { return items[a].cost > items[b].cost; });

  // packing loop: best-fit-decreasing over buckets ordered by time per token
  for (int sidx : shorts) {
    const Item& s = items[sidx];
    int64_t min_tokens = -1;
    for (const Bucket& b : buckets) min_tokens = min_tokens < 0 ? b.tokens : std::min(min_tokens, b.tokens);
    if (buckets.empty() || min_tokens + s.len > T_m) {  // no bucket has room for it
      Bucket b;
      b.shorts.push_back(sidx); b.cost = s.cost; b.tokens = s.len; b.order = (int)buckets.size();
      buckets.push_back(b);
      continue;
    }
    std::vector<int> order(buckets.size());
    for (size_t i = 0; i < order.size(); ++i) order[i] = (int)i;
    const double cc = chunk_const(m);
    std::stable_sort(order.begin(), order.end(),
                     [&](int a, int b) { return buckets[a].metric(cc) < buckets[b].metric(cc); });
    for (;;) {
      bool placed = false;
      for (int bi : order) {  // first bucket, in that order, that stays within both thresholds
        Bucket& b = buckets[bi];
        if (b.cost + s.cost + chunk_const(m) <= T_t && b.tokens + s.len <= T_m) {
          b.shorts.push_back(sidx); b.cost += s.cost; b.tokens += s.len;
          placed = true;
          break;
        }
      }
      if (placed) break;
      // nothing fits: relax the time threshold to the cheapest bucket that has room for the tokens, then retry
      double best = -1.0;
      for (const Bucket& b : buckets)
        if (b.tokens + s.len <= T_m) {
          const double t = b.cost + s.cost + chunk_const(m);
          best = best < 0.0 ? t : std::min(best, t);
        }
      T_t = best;
    }
  }

  // buckets -> hybrid chunks (tail slice first) and batched chunks
  for (const Bucket& b : buckets) {
    const int first = ns;
    if (b.tail >= 0 && !push_slice(items[b.tail].seq, items[b.tail].start, items[b.tail].len)) return CHUNK_ATTN_INVALID_ARG;
    for (int sidx : b.shorts)
      if (!push_slice(items[sidx].seq, items[sidx].start, items[sidx].len)) return CHUNK_ATTN_INVALID_ARG;
    if (!push_chunk(b.context, first, ns - first, 0, b.tokens, b.cost + chunk_const(m))) return CHUNK_ATTN_INVALID_ARG;
  }
  *n_chunks = nc;
  *n_slices = ns;
  if (time_threshold) *time_threshold = T_t;
  if (token_threshold) *token_threshold = T_m;
  return CHUNK_ATTN_OK;
}

int chunk_plan_segments(const chunk_plan_chunk* chunk, const chunk_plan_slice* slices, chunk_attn_seg* segs,
                        int32_t* total_q, int32_t* total_kv) {
  if (!chunk || !slices || !segs || !total_q || !total_kv || chunk->num_slices < 1 || chunk->context < 0)
    return CHUNK_ATTN_INVALID_ARG;
  int64_t q = 0, kv = 0;
  for (int i = 0; i < chunk->num_slices; ++i) {
    const chunk_plan_slice& s = slices[chunk->first_slice + i];
    const int64_t ctx = i == 0 ? chunk->context : 0;
    if (s.len < 1 || q + s.len > 0x7fffffff || kv + ctx + s.len > 0x7fffffff) return CHUNK_ATTN_INVALID_ARG;
    segs[i] = chunk_attn_seg{(int32_t)q, s.len, (int32_t)kv, (int32_t)(ctx + s.len)};
    q += s.len;
    kv += ctx + s.len;
  }
  *total_q = (int32_t)q;
  *total_kv = (int32_t)kv;
  return CHUNK_ATTN_OK;
}

}  // extern "C"
