// Kernel parameter blocks and launchers (internal to the library).
#pragma once
#include <hip/hip_runtime.h>

#include <algorithm>

#include "device_common.hpp"
#include "plan.hpp"

#ifndef DKV_KEYS
#define DKV_KEYS 128
#endif

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
  int32_t heads_per_wg;                      // query heads of one group handled by one workgroup (a power of two)
  int32_t head_splits;                       // group / heads_per_wg
  int32_t total_q;
  float scale_log2;                          // softmax scale * log2(e)
  int32_t* redo;                             // per-workgroup redo flags of the pipelined forward (null: run every item)
  int32_t* any_redo;                         // raised together with any redo flag (gates the second pass's preparation)
  float ref_limit;                           // log2 growth of the row maximum past the first tile's that raises the flag
  int32_t* taken;                            // 8 block-queue counters of the pipelined forward (zero before the launch)
  unsigned long long* clock_log;             // null, or where the pipelined forward's workgroups log their clocks
};

// rows of query tile per forward work item for a given head layout
// Shape of a query-stationary workgroup (forward and dQ kernels): `waves` waves of 32 query rows each, spread
// over as many query heads of one group as divide both (so that the key/value tiles they stream are shared).
// forward: 4 waves; for head_dim 128 each wave owns two 32-row query blocks (fwd_pipe_kernel; its second pass,
// fwd_kernel with 8 waves of one block, covers the same rows per workgroup)
inline int fwd_waves(int) { return 4; }
inline int fwd_qblocks(int head_dim) { return head_dim == 128 ? 2 : 1; }
inline int dq_waves(int head_dim) { return head_dim == 128 ? 8 : 4; }
inline int heads_per_wg(int group, int waves) {
  int h = 1;
  while (h * 2 <= waves && group % (h * 2) == 0) h *= 2;
  return h;
}
// key rows per work item of the dK/dV kernel (32 per pair of waves); head_dim 256 leaves room for two pairs only
inline int dkv_keys(int head_dim) { return head_dim > 128 ? 64 : DKV_KEYS; }
inline int tile_rows(int group, int waves) { return 32 * (waves / heads_per_wg(group, waves)); }

// Workgroups launched by a kernel whose workgroups claim their blocks themselves (device_common.hpp): one per CU of the
// current device, and never more than there are blocks.
inline int persistent_grid(int64_t blocks) {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      cus <= 0)
    cus = 256;
  return (int)std::max<int64_t>(1, std::min<int64_t>(blocks, cus));
}
constexpr int kBlockQueues = 8;  // counters per kernel that claims its blocks

// Events armed by chunk_attn_profile_events for the calling thread (null when disarmed).
struct ProfileEvents {
  hipEvent_t start = nullptr, stop = nullptr;
};
ProfileEvents& profile_events();

// Pointers of one backward call (device memory, caller-owned).
struct BwdArgs {
  const __bf16 *q, *k, *v, *o, *d_o;
  const float* lse;
  __bf16 *dq, *dk, *dv;
  bool accumulate;
  bool dkv_f32;  // dk / dv are fp32 arrays
  char* workspace;
};

// Host-side plan of one backward call and the layout of its workspace:
// [dQ items | dK/dV items | 64-row query-tile jobs | 32-row key-tile jobs] (one uploaded blob), then the
// LSE and D arrays padded to 64-row tiles and the transposed images of K (32-row tiles).
struct BwdPlan {
  std::vector<DqItem> dq_items;
  std::vector<DkvItem> dkv_items;
  std::vector<TileJob> qjobs, kjobs;
  int64_t q_tiles = 0, kv32_tiles = 0;
  size_t dq_items_off = 0, dkv_items_off = 0, qjobs_off = 0, kjobs_off = 0, queues_off = 0, blob_bytes = 0;
  size_t lse2p_off = 0, dsp_off = 0, kt_off = 0, total = 0;
  // one-pass backward (head_dim 128): its items and workgroup order travel at the end of the blob; then the per-wave
  // progress counters and the status word (cleared by a kernel on every call) and the float32 dQ tiles
  bool fused = false;
  FusedPlan fplan;
  int64_t qt32_tiles = 0;
  size_t fitems_off = 0, forder_off = 0, q32jobs_off = 0, fprog_off = 0, fprog_bytes = 0, fdq_off = 0;
};
constexpr size_t kFusedSinkBytes = 64 * 16384;  // scratch dQ tiles of the one-pass backward, behind its status word
constexpr int kNumXcd = 8;  // XCDs of an MI355X: workgroup b runs on XCD b % 8

// 0: the library's choice, 1: the two-kernel backward, 2: the one-pass backward (head_dim 128 only)
int bwd_mode();
// Device memory the caller has set aside for the clock logs of the three pipelined kernels (null: none), and the section
// of kernel `which` in it (0 forward, 1 dQ, 2 dK/dV), kClockLogEntries values of 8 bytes each.
constexpr size_t kClockLogEntries = 4 * 1024;
unsigned long long* clock_log(int which);
hipError_t launch_bwd_fused(const chunk_attn_desc* d, const BwdArgs& a, const BwdPlan& plan, const float* lse2p, const float* dsp,
                            hipStream_t stream);
// Fills the offsets (and, if with_plan, the schedules) for a validated descriptor.
void bwd_layout(const chunk_attn_desc* d, BwdPlan& plan, bool with_plan);
// The host image of the blob at the start of the workspace.
std::vector<char> bwd_blob(const BwdPlan& plan);
// Enqueues the backward kernels; the blob must already be on its way to the workspace on `stream`.
hipError_t launch_bwd(const chunk_attn_desc* d, const BwdArgs& a, const BwdPlan& plan, hipStream_t stream);

// The forward kernels of one call.  `vjobs` (device) lists the 64-row tiles of V whose transposed images p.vt receives:
// before the kernel for head_dim 64, after the pipelined kernel and only if it raised a redo flag for head_dim 128.
hipError_t launch_fwd(const FwdParams& p, int head_dim, int num_blocks, const TileJob* vjobs, int num_vjobs, hipStream_t stream);

// Transposed tile images (width 64 or 32 rows) of x[rows][num_heads][head_dim]:
// out[num_heads][total_tiles][head_dim][width].  With a non-null `gate` (device) the kernel does nothing unless *gate != 0.
hipError_t launch_transpose(const __bf16* x, int num_heads, int head_dim, int width, const TileJob* jobs, int num_jobs,
                            int64_t total_tiles, __bf16* out, hipStream_t stream, const int32_t* gate = nullptr);

}  // namespace chunk_attn
