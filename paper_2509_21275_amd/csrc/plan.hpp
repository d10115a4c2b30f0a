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

// A 64-row tile of a tensor to be transposed by the pre-pass: rows [src_row0, src_row0 + valid_rows).
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

// Backward work item: a tile of consecutive key rows of one segment and the queries that see it.
struct BwdItem {
  int32_t kv_row0;  // first key row of the tile (global)
  int32_t kv_rows;  // valid key rows in the tile (>= 1)
  int32_t q_row0;   // first query row (global) that sees any key of the tile
  int32_t q_rows;   // queries from q_row0 to the end of the segment (>= 1)
  int32_t n0;       // keys of the segment visible to query q_row0, counted from the segment's first key
  int32_t j0;       // index of the tile's first key inside the segment
  int32_t pad0, pad1;
};

int validate(const chunk_attn_desc* d);
int64_t pair_count(const chunk_attn_desc* d);

// Tiles of `tile_rows` query rows per segment, most work first.
std::vector<FwdItem> plan_fwd(const chunk_attn_desc* d, int tile_rows);
// Tiles of `tile_rows` key rows per segment, most work first.
std::vector<BwdItem> plan_bwd(const chunk_attn_desc* d, int tile_rows);
// 64-row tiles of every segment's key range (kv = true) or query range (kv = false), in segment order;
// seg_tile0[t] receives the image index of segment t's first tile.
std::vector<TileJob> tile_jobs(const chunk_attn_desc* d, bool kv, std::vector<int32_t>* seg_tile0);
int64_t count_tiles(const chunk_attn_desc* d, bool kv);
// Key-row ranges [begin, end) not covered by any segment (to be zero-filled when not accumulating).
std::vector<std::pair<int32_t, int32_t>> uncovered_kv_ranges(const chunk_attn_desc* d);

}  // namespace chunk_attn
