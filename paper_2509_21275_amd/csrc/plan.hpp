// Host-side planning for chunk attention: descriptor checks and the tile schedules that
// the kernels walk.  Pure C++ (no HIP), so it can be exercised without a GPU.
//
// A chunk {C, S} (paper section 3.1) arrives as a segment table; the schedule turns it into
// independent work items.  Only tiles that contain at least one unmasked (query, key) pair
// are ever scheduled: the causal mask and the block-diagonal structure of a packed chunk
// are exploited by construction, not by testing tiles on the device.
#pragma once
#include <cstdint>
#include <vector>

#include "../../include/chunk_attn.h"

namespace chunk_attn {

// A tile (64 or 32 rows) of a tensor to be transposed by the pre-pass: rows [src_row0, src_row0 + valid_rows).
struct TileJob {
  int32_t src_row0, valid_rows;
  int32_t image;  // index of the output image (per head)
  int32_t pad;
};

// Forward work item: a tile of consecutive query rows of one segment.
struct FwdItem {
  int32_t q_row0;    // first query row (global)
  int32_t q_rows;    // valid rows in the tile (>= 1)
  int32_t kv_row0;   // first key row of the segment (global)
  int32_t n0;        // keys visible to the tile's first row: C + i0 + 1; row r sees n0 + r
  int32_t kv_tile0;  // index of the transposed image of the segment's first 64-key tile
  int32_t pad0, pad1, pad2;
};

// Work item of the dQ kernel: a tile of consecutive query rows of one segment (as in the forward).
struct DqItem {
  int32_t q_row0;    // first query row (global)
  int32_t q_rows;    // valid rows in the tile (>= 1)
  int32_t kv_row0;   // first key row of the segment (global)
  int32_t n0;        // keys visible to the tile's first row
  int32_t kv_tile0;  // index of the transposed image of the segment's first 32-key tile
  int32_t q_slot0;   // slot of the tile's first row in the padded per-row arrays (LSE, D)
  int32_t pad0, pad1;
};

// Work item of the dK/dV kernel: up to 128 consecutive key rows of one segment and the 32-row query tiles
// (aligned to the segment's first query) that contain at least one query seeing them.
struct DkvItem {
  int32_t kv_row0;    // first key row of the tile (global)
  int32_t kv_rows;    // valid key rows
  int32_t j0;         // index of the tile's first key inside the segment
  int32_t ctx;        // context length C of the segment
  int32_t q_row_seg;  // first query row of the segment (global)
  int32_t q_len;      // queries in the segment
  int32_t qt_first;   // first 32-row query tile (inside the segment) that sees a key of this tile
  int32_t n_qt;       // number of 32-row query tiles of the segment
  int32_t q_tile0;    // index of the segment's first 64-row tile in the padded per-row arrays (LSE, D)
  int32_t reverse;    // 1: the kernel walks the query tiles from the segment's last one down to qt_first (plan_dkv)
  int32_t in_step;    // 1: started only when the blocks of the groups before it (of `side_by_side` blocks) have ended (plan_dkv)
  int32_t pad1;
};

// Work item of the one-pass backward kernel (head_dim 128): a DkvItem plus what the kernel needs to add its share of dQ
// into the float32 dQ tiles in a fixed order.  All key blocks of one (segment, key/value head) form a chain, in
// order of their first key; a block adds to a dQ tile after its predecessor in the chain has (every query tile a block
// sees is also seen by its predecessor, so the first block of a chain initialises every tile).
struct FusedItem {
  int32_t kv_row0, kv_rows, j0, ctx, q_row_seg, q_len, qt_first, n_qt, q_tile0;  // as in DkvItem
  int32_t kvh;        // key/value head
  int32_t pred;       // item index of the predecessor in the chain, -1 for the chain's first block
  int32_t delta_qt;   // qt_first - predecessor's qt_first (>= 0)
  int32_t dq_tile0;   // index of the segment's first 32-row query tile in the dQ tile array (per head)
  int32_t buf;        // which dQ tile array the block's sub-chain adds into
  int32_t pad1, pad2;
};
// A 32-row tile of dQ for the conversion to bf16 rows.
struct DqTileJob {
  int32_t q_row0, valid_rows;  // first query row (global) and rows in the tile
  int32_t tile;                // index of the tile in a dQ tile array (per head)
  int32_t qt;                  // index of the tile inside its segment
  int32_t ctx, n_blocks;       // context length and number of key blocks of the segment
  int32_t pad0, pad1;
};
struct FusedPlan {
  std::vector<FusedItem> items;
  std::vector<int32_t> order;   // workgroup b runs item order[b] (-1: nothing); b % 8 is the XCD the chain is pinned to
  std::vector<DqTileJob> tiles;
  int64_t total_qt32 = 0;       // 32-row query tiles of all segments
  int num_bufs = 1;
};
// Sub-chains per (segment, key/value head): the blocks of a chain are dealt round robin to `num_bufs` sub-chains, each
// adding into a dQ tile array of its own (summed by the conversion), which shortens the wait along a chain.
int fused_num_bufs(const chunk_attn_desc* d, int keys);
FusedPlan plan_fused(const chunk_attn_desc* d, int keys, int num_xcd, int num_bufs);

int validate(const chunk_attn_desc* d);
int64_t pair_count(const chunk_attn_desc* d);

// Tiles of `tile_rows` query rows per segment, most work first.
std::vector<FwdItem> plan_fwd(const chunk_attn_desc* d, int tile_rows);
std::vector<DqItem> plan_dq(const chunk_attn_desc* d, int tile_rows);
// `keys` consecutive key rows per item.  `side_by_side` = 0: every item walks its query tiles upwards.  > 0: the number
// of items of one key/value head that run at the same time; the items of a sequence are then ordered, and given a walk
// direction each, so that those items read the same query rows at about the same time (see plan.cpp).
std::vector<DkvItem> plan_dkv(const chunk_attn_desc* d, int keys, int side_by_side = 0);
// `width`-row tiles of every segment's key range (kv = true) or query range (kv = false), in segment order;
// seg_tile0[t] receives the image index of segment t's first tile.
std::vector<TileJob> tile_jobs(const chunk_attn_desc* d, bool kv, int width, std::vector<int32_t>* seg_tile0);
int64_t count_tiles(const chunk_attn_desc* d, bool kv, int width);
// Key-row ranges [begin, end) not covered by any segment (to be zero-filled when not accumulating).
std::vector<std::pair<int32_t, int32_t>> uncovered_kv_ranges(const chunk_attn_desc* d);

}  // namespace chunk_attn
