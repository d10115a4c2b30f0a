// Kernel parameter blocks and launchers (internal to the library).
#pragma once
#include <hip/hip_runtime.h>

#include "device_common.hpp"
#include "plan.hpp"

namespace chunk_attn {

struct FwdParams {
  const __bf16* q;
  const __bf16* k;
  const __bf16* v;
  __bf16* o;
  float* lse;
  const __bf16* vt;         // transposed V images [Hkv][total_kv_tiles][D][64]
  const FwdItem* items;
  int64_t total_kv_tiles;
  int32_t num_q_heads, num_kv_heads, group;  // group = Hq / Hkv
  int32_t heads_per_wg;                      // query heads of one group handled by one workgroup (1, 2 or 4)
  int32_t head_splits;                       // group / heads_per_wg
  int32_t total_q;
  float scale_log2;                          // softmax scale * log2(e)
};

// rows of query tile per forward work item for a given head layout
inline int fwd_heads_per_wg(int group) { return group % 4 == 0 ? 4 : (group % 2 == 0 ? 2 : 1); }
inline int fwd_tile_rows(int group) { return 32 * (4 / fwd_heads_per_wg(group)); }

// Events armed by chunk_attn_profile_events for the calling thread (null when disarmed).
struct ProfileEvents {
  hipEvent_t start = nullptr, stop = nullptr;
};
ProfileEvents& profile_events();

struct BwdParams {
  const __bf16* q;
  const __bf16* k;
  const __bf16* v;
  const __bf16* d_o;
  const float* lse;
  const float* dsum;  // D_i = <dO_i, O_i>, [Hq][total_q]
  float* dq_acc;      // float32 [total_q][Hq][D], unscaled
  __bf16* dk;
  __bf16* dv;
  const BwdItem* items;
  int32_t num_q_heads, num_kv_heads, group, total_q;
  float scale, scale_log2;
  int32_t accumulate;
};

// Pointers of one backward call (device memory, caller-owned).
struct BwdArgs {
  const __bf16 *q, *k, *v, *o, *d_o;
  const float* lse;
  __bf16 *dq, *dk, *dv;
  bool accumulate;
  char* workspace;
};

size_t bwd_workspace_bytes(const chunk_attn_desc* d);
// Builds the backward schedule and reports where in the workspace it has to be uploaded.
void bwd_prepare(const chunk_attn_desc* d, std::vector<BwdItem>& items, size_t* items_off);
// Enqueues the backward kernels; the schedule must already be on its way to the workspace on `stream`.
hipError_t launch_bwd(const chunk_attn_desc* d, const BwdArgs& a, const std::vector<BwdItem>& items,
                      hipStream_t stream);

hipError_t launch_fwd(const FwdParams& p, int head_dim, int num_blocks, hipStream_t stream);

// Transposed 64-row tile images of x[rows][num_heads][head_dim]: out[num_heads][total_tiles][head_dim][64].
hipError_t launch_transpose(const __bf16* x, int num_heads, int head_dim, const TileJob* jobs, int num_jobs,
                            int64_t total_tiles, __bf16* out, hipStream_t stream);

}  // namespace chunk_attn
