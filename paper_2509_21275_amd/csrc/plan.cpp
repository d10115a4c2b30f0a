#include "plan.hpp"

#include <algorithm>
#include <cmath>

namespace chunk_attn {

int validate(const chunk_attn_desc* d) {
  if (!d || !d->segments) return CHUNK_ATTN_INVALID_ARG;
  if (d->num_q_heads <= 0 || d->num_kv_heads <= 0 || d->head_dim <= 0 || d->total_q <= 0 || d->total_kv <= 0 ||
      d->num_segments <= 0)
    return CHUNK_ATTN_INVALID_ARG;
  if (!(d->softmax_scale > 0.0f) || !std::isfinite(d->softmax_scale)) return CHUNK_ATTN_INVALID_ARG;
  if (d->head_dim != 64 && d->head_dim != 96 && d->head_dim != 128 && d->head_dim != 256) return CHUNK_ATTN_UNSUPPORTED;
  if (d->num_q_heads % d->num_kv_heads != 0) return CHUNK_ATTN_UNSUPPORTED;
  int64_t q_next = 0, kv_next = 0;
  for (int t = 0; t < d->num_segments; ++t) {
    const chunk_attn_seg& s = d->segments[t];
    if (s.q_len < 1 || s.kv_len < s.q_len) return CHUNK_ATTN_BAD_SEGMENT;
    if (s.q_start != q_next) return CHUNK_ATTN_BAD_SEGMENT;  // in order, back to back, from row 0
    if (s.kv_start < kv_next) return CHUNK_ATTN_BAD_SEGMENT; // in order, no overlap
    q_next = (int64_t)s.q_start + s.q_len;
    kv_next = (int64_t)s.kv_start + s.kv_len;
    if (q_next > d->total_q || kv_next > d->total_kv) return CHUNK_ATTN_BAD_SEGMENT;
  }
  if (q_next != d->total_q) return CHUNK_ATTN_BAD_SEGMENT;
  return CHUNK_ATTN_OK;
}

int64_t pair_count(const chunk_attn_desc* d) {
  int64_t n = 0;
  for (int t = 0; t < d->num_segments; ++t) {
    const int64_t s = d->segments[t].q_len, C = (int64_t)d->segments[t].kv_len - s;
    n += s * C + s * (s + 1) / 2;
  }
  return n;
}

int64_t count_tiles(const chunk_attn_desc* d, bool kv, int width) {
  int64_t n = 0;
  for (int t = 0; t < d->num_segments; ++t)
    n += ((kv ? d->segments[t].kv_len : d->segments[t].q_len) + width - 1) / width;
  return n;
}

std::vector<TileJob> tile_jobs(const chunk_attn_desc* d, bool kv, int width, std::vector<int32_t>* seg_tile0) {
  std::vector<TileJob> jobs;
  if (seg_tile0) seg_tile0->clear();
  for (int t = 0; t < d->num_segments; ++t) {
    const chunk_attn_seg& s = d->segments[t];
    const int32_t start = kv ? s.kv_start : s.q_start, len = kv ? s.kv_len : s.q_len;
    if (seg_tile0) seg_tile0->push_back((int32_t)jobs.size());
    for (int32_t r = 0; r < len; r += width) {
      TileJob j;
      j.src_row0 = start + r;
      j.valid_rows = std::min<int32_t>(width, len - r);
      j.image = (int32_t)jobs.size();
      j.pad = 0;
      jobs.push_back(j);
    }
  }
  return jobs;
}

// Order of the query-stationary work items: sequence by sequence, the sequence with the most keys first, and inside a
// sequence the query tile that walks the most keys first.  The workgroups of an XCD then work on neighbouring tiles of
// one sequence and share its K / V stream in the L2, the long sequences still start first, and every sequence ends in
// short items that fill the tail (the workgroups balance the rest by taking blocks from each other's queues).
// Measured against "longest walk first over the whole chunk": +1.7 % on the packed 64K chunk, nothing on the others.
template <class Item>
static void by_sequence_then_walk(const chunk_attn_desc* d, std::vector<Item>& items) {
  std::vector<int32_t> keys_of(d->total_kv + 1, 0);  // by the first key row of a segment: its number of keys
  for (int t = 0; t < d->num_segments; ++t) keys_of[d->segments[t].kv_start] = d->segments[t].kv_len;
  std::stable_sort(items.begin(), items.end(), [&](const Item& a, const Item& b) {
    const int32_t ka = keys_of[a.kv_row0], kb = keys_of[b.kv_row0];
    if (ka != kb) return ka > kb;
    if (a.kv_row0 != b.kv_row0) return a.kv_row0 < b.kv_row0;
    return (int64_t)a.n0 + a.q_rows > (int64_t)b.n0 + b.q_rows;
  });
}

std::vector<FwdItem> plan_fwd(const chunk_attn_desc* d, int tile_rows) {
  std::vector<FwdItem> items;
  int32_t kv_tile0 = 0;
  for (int t = 0; t < d->num_segments; ++t) {
    const chunk_attn_seg& s = d->segments[t];
    const int32_t C = s.kv_len - s.q_len;
    for (int32_t i0 = 0; i0 < s.q_len; i0 += tile_rows) {
      FwdItem it{};
      it.kv_tile0 = kv_tile0;
      it.q_row0 = s.q_start + i0;
      it.q_rows = std::min<int32_t>(tile_rows, s.q_len - i0);
      it.kv_row0 = s.kv_start;
      it.n0 = C + i0 + 1;
      items.push_back(it);
    }
    kv_tile0 += (s.kv_len + 63) / 64;
  }
  by_sequence_then_walk(d, items);
  return items;
}

std::vector<DqItem> plan_dq(const chunk_attn_desc* d, int tile_rows) {
  std::vector<DqItem> items;
  int32_t kv_tile0 = 0, q_tile0 = 0;
  for (int t = 0; t < d->num_segments; ++t) {
    const chunk_attn_seg& s = d->segments[t];
    const int32_t C = s.kv_len - s.q_len;
    for (int32_t i0 = 0; i0 < s.q_len; i0 += tile_rows) {
      DqItem it{};
      it.q_row0 = s.q_start + i0;
      it.q_rows = std::min<int32_t>(tile_rows, s.q_len - i0);
      it.kv_row0 = s.kv_start;
      it.n0 = C + i0 + 1;
      it.kv_tile0 = kv_tile0;
      it.q_slot0 = q_tile0 * 64 + i0;
      items.push_back(it);
    }
    kv_tile0 += (s.kv_len + 31) / 32;
    q_tile0 += (s.q_len + 63) / 64;
  }
  by_sequence_then_walk(d, items);
  return items;
}

// Order and walk directions of one sequence's key blocks, given in key order (= longest walk first), when `width` of
// them run side by side and read the same stream of query rows through one L2.  Blocks that start together stay
// together only if they start at the same row; blocks of unequal length end at different times.  So:
//   * blocks that every query sees come first, walking upwards: equal walks, started together at the first row;
//   * of the others (walks that begin at the block's diagonal and all end at the last row) the longest `width` walk
//     DOWN from the last row, started together; as each ends, at its diagonal, its workgroup takes the partner that
//     makes the pair's length the same for all -- the shortest remaining walks, longest of them first, walking UP:
//     a block that ends its descent at row r after time T - r is followed by one that starts its ascent near the row
//     where the others are by then; all of them arrive at the last row together, and the next `width` longest descend;
//   * the shortest quarter is kept for the end, longest first, walking upwards: small items for the workgroups to
//     even out what their unequal speeds have left.
// The result holds indices into the input order; reverse[i] is the direction of input block i.
// in_step[i]: block i is one of the equal walks at the front.  The workgroups that run them drift apart over many blocks
// (left alone their speeds differ by up to 2 %), until they no longer find each other's rows in the L2; the kernel
// therefore starts such a block only when the blocks of the groups of `width` before it have ended.
void side_by_side_order(const std::vector<DkvItem>& blocks, int width, std::vector<int>& order, std::vector<char>& reverse,
                        std::vector<char>& in_step) {
  const int n = (int)blocks.size();
  order.clear();
  reverse.assign(n, 0);
  in_step.assign(n, 0);
  int lo = 0;
  while (lo < n && blocks[lo].qt_first == 0 && blocks[lo].j0 + blocks[lo].kv_rows <= blocks[lo].ctx) {
    in_step[lo] = 1;
    order.push_back(lo++);
  }
  int hi = n - (n - lo) / 4;
  const int tail = hi;
  while (lo < hi) {
    const int m = hi - lo;
    const int down = m >= 2 * width ? width : (m + 1) / 2, up = std::min(down, m - down);
    for (int i = 0; i < down; ++i) {
      order.push_back(lo + i);
      reverse[lo + i] = 1;
    }
    for (int i = 0; i < up; ++i) order.push_back(hi - up + i);
    lo += down;
    hi -= up;
  }
  for (int i = tail; i < n; ++i) order.push_back(i);
}

std::vector<DkvItem> plan_dkv(const chunk_attn_desc* d, int keys, int side_by_side) {
  std::vector<DkvItem> items;
  int32_t q_tile0 = 0;
  for (int t = 0; t < d->num_segments; ++t) {
    const chunk_attn_seg& s = d->segments[t];
    const int32_t C = s.kv_len - s.q_len;
    const int32_t n_qt = (s.q_len + 31) / 32;
    for (int32_t j0 = 0; j0 < s.kv_len; j0 += keys) {
      DkvItem it{};
      it.kv_row0 = s.kv_start + j0;
      it.kv_rows = std::min<int32_t>(keys, s.kv_len - j0);
      it.j0 = j0;
      it.ctx = C;
      it.q_row_seg = s.q_start;
      it.q_len = s.q_len;
      it.qt_first = std::max<int32_t>(0, j0 - C) / 32;  // query i sees key j0 iff i >= j0 - C
      it.n_qt = n_qt;
      it.q_tile0 = q_tile0;
      items.push_back(it);
    }
    q_tile0 += (s.q_len + 63) / 64;
  }
  // sequence by sequence, longest first; the key blocks of a sequence in key order, which is longest walk first (see
  // by_sequence_then_walk)
  std::stable_sort(items.begin(), items.end(), [](const DkvItem& a, const DkvItem& b) { return a.n_qt > b.n_qt; });
  if (side_by_side <= 0) return items;
  std::vector<DkvItem> out;
  out.reserve(items.size());
  std::vector<DkvItem> seq;
  std::vector<int> order;
  std::vector<char> reverse, in_step;
  for (size_t i = 0; i < items.size();) {
    size_t e = i;
    while (e < items.size() && items[e].q_row_seg == items[i].q_row_seg && items[e].kv_row0 - items[e].j0 == items[i].kv_row0 - items[i].j0) ++e;
    seq.assign(items.begin() + i, items.begin() + e);
    side_by_side_order(seq, side_by_side, order, reverse, in_step);
    for (int k : order) {
      out.push_back(seq[k]);
      out.back().reverse = reverse[k];
      out.back().in_step = in_step[k];
    }
    i = e;
  }
  return out;
}

int fused_num_bufs(const chunk_attn_desc* d, int keys) {
  int most = 0;
  for (int t = 0; t < d->num_segments; ++t) most = std::max(most, (d->segments[t].kv_len + keys - 1) / keys);
  return most >= 64 ? 4 : most >= 16 ? 2 : 1;
}

FusedPlan plan_fused(const chunk_attn_desc* d, int keys, int num_xcd, int num_bufs) {
  FusedPlan P;
  P.num_bufs = num_bufs;
  struct Chain { int first_item, n_items; int64_t work; };
  std::vector<Chain> chains;
  int32_t q_tile0 = 0, dq_tile0 = 0;
  for (int t = 0; t < d->num_segments; ++t) {
    const chunk_attn_seg& s = d->segments[t];
    const int32_t C = s.kv_len - s.q_len;
    const int32_t n_qt = (s.q_len + 31) / 32;
    for (int kvh = 0; kvh < d->num_kv_heads; ++kvh) {
      Chain ch{(int)P.items.size(), 0, 0};
      int32_t b = 0;
      for (int32_t j0 = 0; j0 < s.kv_len; j0 += keys, ++b) {
        FusedItem it{};
        it.kv_row0 = s.kv_start + j0;
        it.kv_rows = std::min<int32_t>(keys, s.kv_len - j0);
        it.j0 = j0;
        it.ctx = C;
        it.q_row_seg = s.q_start;
        it.q_len = s.q_len;
        it.qt_first = std::max<int32_t>(0, j0 - C) / 32;
        it.n_qt = n_qt;
        it.q_tile0 = q_tile0;
        it.kvh = kvh;
        it.buf = b % num_bufs;
        it.pred = b < num_bufs ? -1 : (int32_t)P.items.size() - num_bufs;   // the block num_bufs before it: same sub-chain
        it.delta_qt = b < num_bufs ? 0 : it.qt_first - P.items[it.pred].qt_first;
        it.dq_tile0 = dq_tile0;
        ch.work += n_qt - it.qt_first;
        ++ch.n_items;
        P.items.push_back(it);
      }
      chains.push_back(ch);
    }
    for (int32_t qt = 0; qt < n_qt; ++qt)
      P.tiles.push_back(DqTileJob{s.q_start + 32 * qt, std::min<int32_t>(32, s.q_len - 32 * qt), dq_tile0 + qt, qt, C,
                                  (s.kv_len + keys - 1) / keys, 0, 0});
    q_tile0 += (s.q_len + 63) / 64;
    dq_tile0 += n_qt;
  }
  P.total_qt32 = dq_tile0;
  // chains to XCDs: most work first, each to the XCD with the least work so far
  std::vector<int> by_work(chains.size());
  for (size_t i = 0; i < chains.size(); ++i) by_work[i] = (int)i;
  std::stable_sort(by_work.begin(), by_work.end(), [&](int a, int b) { return chains[a].work > chains[b].work; });
  std::vector<int64_t> load(num_xcd, 0);
  std::vector<std::vector<int32_t>> lists(num_xcd);
  for (int c : by_work) {
    int x = 0;
    for (int i = 1; i < num_xcd; ++i)
      if (load[i] < load[x]) x = i;
    load[x] += chains[c].work;
    for (int i = 0; i < chains[c].n_items; ++i) lists[x].push_back(chains[c].first_item + i);
  }
  // inside an XCD: longest walk first; the walks of a chain do not grow along it, and the sort is stable, so a block
  // always comes after its predecessor
  size_t longest = 0;
  for (auto& l : lists) {
    std::stable_sort(l.begin(), l.end(), [&](int32_t a, int32_t b) {
      return P.items[a].n_qt - P.items[a].qt_first > P.items[b].n_qt - P.items[b].qt_first;
    });
    longest = std::max(longest, l.size());
  }
  P.order.assign(longest * num_xcd, -1);
  for (int x = 0; x < num_xcd; ++x)
    for (size_t i = 0; i < lists[x].size(); ++i) P.order[i * num_xcd + x] = lists[x][i];
  return P;
}

std::vector<std::pair<int32_t, int32_t>> uncovered_kv_ranges(const chunk_attn_desc* d) {
  std::vector<std::pair<int32_t, int32_t>> gaps;
  int32_t next = 0;
  for (int t = 0; t < d->num_segments; ++t) {
    const chunk_attn_seg& s = d->segments[t];
    if (s.kv_start > next) gaps.push_back({next, s.kv_start});
    next = s.kv_start + s.kv_len;
  }
  if (next < d->total_kv) gaps.push_back({next, d->total_kv});
  return gaps;
}

}  // namespace chunk_attn
