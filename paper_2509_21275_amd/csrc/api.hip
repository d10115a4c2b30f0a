// C ABI of the chunk-attention library (include/chunk_attn.h): argument checks, workspace carving,
// schedule upload and kernel launches.  No device memory is allocated here; the only memory the
// library owns is a small ring of pinned host buffers through which tile schedules are uploaded
// (released by chunk_attn_shutdown).
#include <algorithm>
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>

#include "kernels.hpp"

using namespace chunk_attn;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

thread_local std::string g_last_hip_error;

int hip_fail(hipError_t e, const char* what) {
  g_last_hip_error = std::string(what) + ": " + hipGetErrorString(e);
  return CHUNK_ATTN_HIP_ERROR;
}

// Pinned staging buffers for the schedule uploads.  A buffer is reused only after the copy that read it has
// completed; while the GPU is still busy with earlier calls the pool grows (up to kMaxBytes) instead of making the
// caller wait, so that the host can plan and enqueue ahead of the GPU.  Buffers come in power-of-two sizes and are
// never freed on the way (freeing pinned memory waits for the device): a buffer that is too small is simply skipped.
struct StagingRing {
  static constexpr size_t kMaxBytes = (size_t)256 << 20;
  static constexpr size_t kMinSlot = (size_t)256 << 10;
  struct Slot {
    void* host = nullptr;
    size_t cap = 0;
    hipEvent_t ev = nullptr;
    bool in_flight = false;
  };
  std::vector<Slot> slots;
  size_t next = 0, total = 0;
  std::mutex mu;

  // Copies `bytes` from src into pinned memory and enqueues the upload to `dst` on `stream`.
  hipError_t upload(void* dst, const void* src, size_t bytes, hipStream_t stream) {
    std::lock_guard<std::mutex> lock(mu);
    hipError_t e;
    size_t want = kMinSlot;
    while (want < bytes) want *= 2;
    // a completed buffer that is large enough, oldest first (copies on one stream complete in order, so after a few
    // pending ones the rest are pending too)
    Slot* s = nullptr;
    int pending_seen = 0;
    for (size_t i = 0; i < slots.size() && !s && pending_seen < 4; ++i) {
      const size_t idx = (next + i) % slots.size();
      Slot& c = slots[idx];
      if (c.cap < bytes) continue;
      if (c.in_flight) {
        e = hipEventQuery(c.ev);
        if (e == hipSuccess) c.in_flight = false;
        else if (e != hipErrorNotReady) return e;
        else ++pending_seen;
      }
      if (!c.in_flight) {
        s = &c;
        next = (idx + 1) % slots.size();
      }
    }
    if (!s && total + want <= kMaxBytes) {  // grow
      Slot n;
      if ((e = hipHostMalloc(&n.host, want, hipHostMallocDefault)) != hipSuccess) return e;
      n.cap = want;
      if ((e = hipEventCreateWithFlags(&n.ev, hipEventDisableTiming)) != hipSuccess) return e;
      total += want;
      slots.push_back(n);
      s = &slots.back();
    }
    if (!s) {  // the pool is at its limit: wait for the oldest buffer that is large enough
      for (size_t i = 0; i < slots.size() && !s; ++i) {
        Slot& c = slots[(next + i) % slots.size()];
        if (c.cap >= bytes) s = &c;
      }
      if (s) {
        if (s->in_flight && (e = hipEventSynchronize(s->ev)) != hipSuccess) return e;
        s->in_flight = false;
      } else {  // none is: replace the oldest one (this waits for the device)
        s = &slots[next % slots.size()];
        if (s->in_flight && (e = hipEventSynchronize(s->ev)) != hipSuccess) return e;
        s->in_flight = false;
        if ((e = hipHostFree(s->host)) != hipSuccess) return e;
        total -= s->cap;
        s->host = nullptr;
        s->cap = 0;
        if ((e = hipHostMalloc(&s->host, want, hipHostMallocDefault)) != hipSuccess) return e;
        s->cap = want;
        total += want;
      }
    }
    std::memcpy(s->host, src, bytes);
    if ((e = hipMemcpyAsync(dst, s->host, bytes, hipMemcpyHostToDevice, stream)) != hipSuccess) return e;
    if ((e = hipEventRecord(s->ev, stream)) != hipSuccess) return e;
    s->in_flight = true;
    return hipSuccess;
  }

  // Waits for the uploads still reading the buffers and frees them all; the ring starts again from nothing.
  hipError_t release() {
    std::lock_guard<std::mutex> lock(mu);
    hipError_t first = hipSuccess;
    for (Slot& c : slots) {
      hipError_t e = hipSuccess;
      if (c.in_flight) e = hipEventSynchronize(c.ev);
      if (e == hipSuccess && c.ev) e = hipEventDestroy(c.ev);
      if (e == hipSuccess && c.host) e = hipHostFree(c.host);
      if (e != hipSuccess && first == hipSuccess) first = e;
    }
    slots.clear();
    next = total = 0;
    return first;
  }
};
StagingRing g_ring;

// log2 growth of a row's maximum past the first key tile's at which the head_dim 128 forward hands the row to its
// rescaling second pass: bf16 probabilities and fp32 sums hold 2^60 with room to spare
std::atomic<float> g_fwd_rescale_limit{60.0f};

std::atomic<int> g_bwd_mode{0};
std::atomic<unsigned long long*> g_clock_log{nullptr};

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// Forward workspace: [work items | transpose jobs | redo flags (zero)] (uploaded as one blob) then the
// transposed V images.
struct FwdLayout {
  int tile_rows;
  size_t items_bytes, jobs_off, flags_off, blob_bytes, vt_off, total;
  int64_t blocks;
  int64_t kv_tiles;
  std::vector<FwdItem> items;
  std::vector<TileJob> jobs;
};

void layout_fwd(const chunk_attn_desc* d, FwdLayout& L, bool with_plan) {
  const int group = d->num_q_heads / d->num_kv_heads;
  L.tile_rows = tile_rows(group, fwd_waves(d->head_dim)) * fwd_qblocks(d->head_dim);
  size_t n_items = 0;
  if (with_plan) {
    L.items = plan_fwd(d, L.tile_rows);
    L.jobs = tile_jobs(d, true, 64, nullptr);
    n_items = L.items.size();
  } else {
    for (int t = 0; t < d->num_segments; ++t) n_items += (d->segments[t].q_len + L.tile_rows - 1) / L.tile_rows;
  }
  L.kv_tiles = count_tiles(d, true, 64);
  L.items_bytes = n_items * sizeof(FwdItem);
  L.jobs_off = align_up(L.items_bytes);
  L.blocks = (int64_t)n_items * d->num_kv_heads * (group / heads_per_wg(group, fwd_waves(d->head_dim)));
  L.flags_off = align_up(L.jobs_off + (size_t)L.kv_tiles * sizeof(TileJob));
  // one flag per block, then "any flag raised", then the block-queue counters of the pipelined kernel (all zero)
  L.blob_bytes = L.flags_off + ((size_t)L.blocks + 1 + kBlockQueues) * sizeof(int32_t);
  L.vt_off = align_up(L.blob_bytes);
  L.total = L.vt_off + align_up((size_t)L.kv_tiles * d->num_kv_heads * d->head_dim * 64 * sizeof(__bf16));
}

// ---- the forward that allocates nothing (chunk_attn_fwd_static) ----
// Its scratch memory is this array instead of a caller's workspace: every GPU the library runs on holds its own copy, at
// its own address, until the process ends.  Host code never uses the array's name as an address: static_scratch() asks
// the runtime for the device address once per device and hands that out.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
constexpr int kStaticMaxSegments = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

std::mutex g_scratch_mu;
void* g_scratch_ptr[64] = {};  // per device

hipError_t static_scratch(char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if ((e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch))) != hipSuccess) return e;
    g_scratch_ptr[dev] = ptr;
  }
  *out = static_cast<char*>(g_scratch_ptr[dev]);
  return hipSuccess;
}

// The forward's schedule made on the device from a segment table passed by value: work items in segment order (their
// order does not change any result), the 64-row tiles of V, and the redo flags cleared.
struct StaticSegs {
  chunk_attn_seg seg[kStaticMaxSegments];
};
__global__ __launch_bounds__(256) void plan_fwd_static_kernel(StaticSegs segs, int n_seg, int tile_rows, FwdItem* items,
                                                              int n_items, TileJob* jobs, int n_jobs, int32_t* flags,
                                                              int n_flags) {
  __shared__ int item0[kStaticMaxSegments + 1], job0[kStaticMaxSegments + 1];
  if (threadIdx.x == 0) {
    int ni = 0, nj = 0;
    for (int t = 0; t < n_seg; ++t) {
      item0[t] = ni;
      job0[t] = nj;
      ni += (segs.seg[t].q_len + tile_rows - 1) / tile_rows;
      nj += (segs.seg[t].kv_len + 63) / 64;
    }
    item0[n_seg] = ni;
    job0[n_seg] = nj;
  }
  __syncthreads();
  for (int x = threadIdx.x; x < n_items; x += 256) {
    int t = 0;
    while (t + 1 < n_seg && item0[t + 1] <= x) ++t;
    const chunk_attn_seg s = segs.seg[t];
    const int i0 = (x - item0[t]) * tile_rows;
    FwdItem it{};
    it.q_row0 = s.q_start + i0;
    it.q_rows = min(tile_rows, s.q_len - i0);
    it.kv_row0 = s.kv_start;
    it.n0 = s.kv_len - s.q_len + i0 + 1;
    it.kv_tile0 = job0[t];
    items[x] = it;
  }
  for (int x = threadIdx.x; x < n_jobs; x += 256) {
    int t = 0;
    while (t + 1 < n_seg && job0[t + 1] <= x) ++t;
    const chunk_attn_seg s = segs.seg[t];
    const int r = (x - job0[t]) * 64;
    jobs[x] = TileJob{s.kv_start + r, min(64, s.kv_len - r), x, 0};
  }
  for (int x = threadIdx.x; x < n_flags; x += 256) flags[x] = 0;
}

// ---- head_dim 96 ----
// The kernels tile the head dimension in powers of two.  A head of 96 is run as a head of 128 whose last 32 columns
// are zero: zero columns of Q and K add nothing to a score, zero columns of V and dO give zero columns of O, dV and (through
// dS K, dS^T Q) of dQ and dK, and D_i = <dO_i, O_i> is unchanged, so every result is the 96-wide one exactly, with the
// softmax scale the caller gave.  The padded copies live at the head of the workspace; rows move in 16-byte chunks.
constexpr int kNarrowDim = 96, kPaddedDim = 128;

inline bool is_narrow(const chunk_attn_desc* d) { return d->head_dim == kNarrowDim; }
inline chunk_attn_desc widened(const chunk_attn_desc* d) {
  chunk_attn_desc w = *d;
  w.head_dim = kPaddedDim;
  return w;
}
inline size_t padded_bytes(int64_t rows, int heads, size_t elem) { return align_up((size_t)rows * heads * kPaddedDim * elem); }

// dst[row][0 .. out_chunks) = src[row][0 .. in_chunks) followed by zero chunks
__global__ __launch_bounds__(256) void pad_rows_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n_out,
                                                       int in_chunks, int out_chunks) {
  for (int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x; x < n_out; x += (int64_t)gridDim.x * 256) {
    const int64_t row = x / out_chunks;
    const int c = (int)(x - row * out_chunks);
    dst[x] = c < in_chunks ? src[row * in_chunks + c] : make_uint4(0, 0, 0, 0);
  }
}
// dst[row][0 .. in_chunks) = src[row][0 .. in_chunks) of rows that are out_chunks wide
__global__ __launch_bounds__(256) void unpad_rows_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n_in,
                                                         int in_chunks, int out_chunks) {
  for (int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x; x < n_in; x += (int64_t)gridDim.x * 256) {
    const int64_t row = x / in_chunks;
    const int c = (int)(x - row * in_chunks);
    dst[x] = src[row * out_chunks + c];
  }
}
inline int copy_grid(int64_t n) { return (int)std::min<int64_t>((n + 255) / 256, 256 * 16); }
// rows = tensor rows * heads; elem = bytes per element
hipError_t pad_rows(const void* src, void* dst, int64_t rows, size_t elem, hipStream_t stream) {
  const int in_chunks = kNarrowDim * (int)elem / 16, out_chunks = kPaddedDim * (int)elem / 16;
  const int64_t n = rows * out_chunks;
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(pad_rows_kernel, dim3(copy_grid(n)), dim3(256), 0, stream, static_cast<const uint4*>(src),
                     static_cast<uint4*>(dst), n, in_chunks, out_chunks);
  return hipGetLastError();
}
hipError_t unpad_rows(const void* src, void* dst, int64_t rows, size_t elem, hipStream_t stream) {
  const int in_chunks = kNarrowDim * (int)elem / 16, out_chunks = kPaddedDim * (int)elem / 16;
  const int64_t n = rows * in_chunks;
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(unpad_rows_kernel, dim3(copy_grid(n)), dim3(256), 0, stream, static_cast<const uint4*>(src),
                     static_cast<uint4*>(dst), n, in_chunks, out_chunks);
  return hipGetLastError();
}

// Padded copies at the head of a workspace, the widened call's own workspace behind them.
struct NarrowFwdLayout {
  size_t q_off, k_off, v_off, o_off, inner_off, total;
};
NarrowFwdLayout narrow_fwd_layout(const chunk_attn_desc* d, size_t inner_bytes) {
  const size_t qb = padded_bytes(d->total_q, d->num_q_heads, 2), kb = padded_bytes(d->total_kv, d->num_kv_heads, 2);
  NarrowFwdLayout N;
  N.q_off = 0;
  N.k_off = qb;
  N.v_off = N.k_off + kb;
  N.o_off = N.v_off + kb;
  N.inner_off = N.o_off + qb;
  N.total = N.inner_off + inner_bytes;
  return N;
}
struct NarrowBwdLayout {
  size_t q_off, k_off, v_off, o_off, do_off, dq_off, dk_off, dv_off, inner_off, total;
};
// dk / dv copies are sized for float32, whichever entry point is called later
NarrowBwdLayout narrow_bwd_layout(const chunk_attn_desc* d, size_t inner_bytes) {
  const size_t qb = padded_bytes(d->total_q, d->num_q_heads, 2), kb = padded_bytes(d->total_kv, d->num_kv_heads, 2);
  const size_t gb = padded_bytes(d->total_kv, d->num_kv_heads, 4);
  NarrowBwdLayout N;
  N.q_off = 0;
  N.k_off = qb;
  N.v_off = N.k_off + kb;
  N.o_off = N.v_off + kb;
  N.do_off = N.o_off + qb;
  N.dq_off = N.do_off + qb;
  N.dk_off = N.dq_off + qb;
  N.dv_off = N.dk_off + gb;
  N.inner_off = N.dv_off + gb;
  N.total = N.inner_off + inner_bytes;
  return N;
}

}  // namespace

namespace chunk_attn {
int bwd_mode() { return g_bwd_mode.load(); }
unsigned long long* clock_log(int which) {
  unsigned long long* base = g_clock_log.load();
  return base ? base + (size_t)which * kClockLogEntries : nullptr;
}
ProfileEvents& profile_events() {
  static thread_local ProfileEvents ev;
  return ev;
}
}  // namespace chunk_attn

extern "C" {

int chunk_attn_profile_events(void* start_event, void* stop_event) {
  profile_events().start = static_cast<hipEvent_t>(start_event);
  profile_events().stop = static_cast<hipEvent_t>(stop_event);
  return CHUNK_ATTN_OK;
}

int chunk_attn_validate(const chunk_attn_desc* desc) { return validate(desc); }

int chunk_attn_shutdown(void) {
  const hipError_t e = g_ring.release();
  return e == hipSuccess ? CHUNK_ATTN_OK : hip_fail(e, "releasing the staging buffers");
}

int chunk_attn_test_set_bwd_mode(int mode) {
  if (mode < 0 || mode > 2) return CHUNK_ATTN_INVALID_ARG;
  g_bwd_mode.store(mode);
  return CHUNK_ATTN_OK;
}

int chunk_attn_measure_set_clock_log(void* device_buffer, size_t bytes) {
  if (device_buffer == nullptr) {
    g_clock_log.store(nullptr);
    return CHUNK_ATTN_OK;
  }
  if ((reinterpret_cast<uintptr_t>(device_buffer) & 7) != 0) return CHUNK_ATTN_INVALID_ARG;
  if (bytes < 3 * kClockLogEntries * sizeof(unsigned long long)) return CHUNK_ATTN_WORKSPACE_TOO_SMALL;
  g_clock_log.store(static_cast<unsigned long long*>(device_buffer));
  return CHUNK_ATTN_OK;
}

int chunk_attn_test_bwd_status_offset(const chunk_attn_desc* desc, size_t* offset) {
  const int rc = validate(desc);
  if (rc != CHUNK_ATTN_OK) return rc;
  if (!offset) return CHUNK_ATTN_INVALID_ARG;
  const chunk_attn_desc w = is_narrow(desc) ? widened(desc) : *desc;
  BwdPlan P;
  bwd_layout(&w, P, false);
  *offset = P.fprog_off + P.fprog_bytes - kFusedSinkBytes - 256;
  if (is_narrow(desc)) *offset += narrow_bwd_layout(desc, P.total).inner_off;
  return CHUNK_ATTN_OK;
}

int chunk_attn_test_set_fwd_rescale_limit(float log2_growth) {
  g_fwd_rescale_limit.store(log2_growth);
  return CHUNK_ATTN_OK;
}

int64_t chunk_attn_pair_count(const chunk_attn_desc* desc) {
  const int rc = validate(desc);
  if (rc != CHUNK_ATTN_OK) return rc;
  return pair_count(desc);
}

const char* chunk_attn_strerror(int code) {
  switch (code) {
    case CHUNK_ATTN_OK: return "ok";
    case CHUNK_ATTN_INVALID_ARG: return "invalid argument (null pointer, non-positive size or bad scale)";
    case CHUNK_ATTN_UNSUPPORTED: return "unsupported shape (head_dim must be 64, 96, 128 or 256; num_kv_heads must divide num_q_heads)";
    case CHUNK_ATTN_BAD_SEGMENT: return "bad segment table";
    case CHUNK_ATTN_WORKSPACE_TOO_SMALL: return "workspace too small (see chunk_attn_workspace_bytes)";
    case CHUNK_ATTN_TOO_LARGE:
      return "chunk too large for chunk_attn_fwd_static (at most 64 segments and 16 MiB of forward scratch, see "
             "chunk_attn_workspace_bytes); use chunk_attn_fwd with a workspace";
    case CHUNK_ATTN_HIP_ERROR: {
      static thread_local std::string msg;
      msg = "HIP error: " + g_last_hip_error;
      return msg.c_str();
    }
    default: return "unknown error code";
  }
}

int chunk_attn_workspace_bytes(const chunk_attn_desc* desc, size_t* fwd_bytes, size_t* bwd_bytes) {
  const int rc = validate(desc);
  if (rc != CHUNK_ATTN_OK) return rc;
  const chunk_attn_desc w = is_narrow(desc) ? widened(desc) : *desc;
  if (fwd_bytes) {
    FwdLayout L;
    layout_fwd(&w, L, false);
    *fwd_bytes = is_narrow(desc) ? narrow_fwd_layout(desc, L.total).total : L.total;
  }
  if (bwd_bytes) {
    BwdPlan P;
    bwd_layout(&w, P, false);
    *bwd_bytes = is_narrow(desc) ? narrow_bwd_layout(desc, P.total).total : P.total;
  }
  return CHUNK_ATTN_OK;
}

int chunk_attn_fwd(const chunk_attn_desc* desc, const void* q, const void* k, const void* v, void* o, float* lse,
                   void* workspace, size_t workspace_bytes, void* stream_v) {
  const int rc = validate(desc);
  if (rc != CHUNK_ATTN_OK) return rc;
  if (!q || !k || !v || !o || !lse || !workspace) return CHUNK_ATTN_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) != 0) return CHUNK_ATTN_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || (reinterpret_cast<uintptr_t>(lse) & 3) != 0)
    return CHUNK_ATTN_INVALID_ARG;  // the kernels move rows in 16-byte pieces
  if (is_narrow(desc)) {  // run as head_dim 128 on zero-padded copies
    const chunk_attn_desc w = widened(desc);
    FwdLayout Lw;
    layout_fwd(&w, Lw, false);
    const NarrowFwdLayout N = narrow_fwd_layout(desc, Lw.total);
    if (workspace_bytes < N.total) return CHUNK_ATTN_WORKSPACE_TOO_SMALL;
    hipStream_t st = static_cast<hipStream_t>(stream_v);
    char* base = static_cast<char*>(workspace);
    const int64_t qr = (int64_t)desc->total_q * desc->num_q_heads, kr = (int64_t)desc->total_kv * desc->num_kv_heads;
    hipError_t pe;
    if ((pe = pad_rows(q, base + N.q_off, qr, 2, st)) != hipSuccess || (pe = pad_rows(k, base + N.k_off, kr, 2, st)) != hipSuccess ||
        (pe = pad_rows(v, base + N.v_off, kr, 2, st)) != hipSuccess)
      return hip_fail(pe, "padding launch");
    const int r = chunk_attn_fwd(&w, base + N.q_off, base + N.k_off, base + N.v_off, base + N.o_off, lse, base + N.inner_off,
                                 workspace_bytes - N.inner_off, stream_v);
    if (r != CHUNK_ATTN_OK) return r;
    if ((pe = unpad_rows(base + N.o_off, o, qr, 2, st)) != hipSuccess) return hip_fail(pe, "unpadding launch");
    return CHUNK_ATTN_OK;
  }
  FwdLayout L;
  layout_fwd(desc, L, true);
  if (workspace_bytes < L.total) return CHUNK_ATTN_WORKSPACE_TOO_SMALL;
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  char* ws = static_cast<char*>(workspace);

  std::vector<char> blob(L.blob_bytes, 0);
  std::memcpy(blob.data(), L.items.data(), L.items_bytes);
  std::memcpy(blob.data() + L.jobs_off, L.jobs.data(), L.jobs.size() * sizeof(TileJob));
  hipError_t e = g_ring.upload(ws, blob.data(), blob.size(), stream);
  if (e != hipSuccess) return hip_fail(e, "schedule upload");
  __bf16* vt = reinterpret_cast<__bf16*>(ws + L.vt_off);

  FwdParams p;
  p.q = static_cast<const __bf16*>(q);
  p.k = static_cast<const __bf16*>(k);
  p.v = static_cast<const __bf16*>(v);
  p.o = static_cast<__bf16*>(o);
  p.lse = lse;
  p.vt = vt;
  p.items = reinterpret_cast<const FwdItem*>(ws);
  p.total_kv_tiles = L.kv_tiles;
  p.num_q_heads = desc->num_q_heads;
  p.num_kv_heads = desc->num_kv_heads;
  p.group = desc->num_q_heads / desc->num_kv_heads;
  p.heads_per_wg = heads_per_wg(p.group, fwd_waves(desc->head_dim));
  p.head_splits = p.group / p.heads_per_wg;
  p.total_q = desc->total_q;
  p.scale_log2 = desc->softmax_scale * 1.4426950408889634f;
  p.redo = desc->head_dim == 128 ? reinterpret_cast<int32_t*>(ws + L.flags_off) : nullptr;
  p.any_redo = reinterpret_cast<int32_t*>(ws + L.flags_off) + L.blocks;
  p.taken = p.any_redo + 1;
  p.clock_log = clock_log(0);
  p.ref_limit = g_fwd_rescale_limit.load();
  const int64_t blocks = L.blocks;
  if (blocks > 0x7fffffff) return CHUNK_ATTN_UNSUPPORTED;
  ProfileEvents pe = profile_events();
  profile_events() = ProfileEvents{};
  if (pe.start && (e = hipEventRecord(pe.start, stream)) != hipSuccess) return hip_fail(e, "event record");
  e = launch_fwd(p, desc->head_dim, (int)blocks, reinterpret_cast<const TileJob*>(ws + L.jobs_off), (int)L.jobs.size(), stream);
  if (e != hipSuccess) return hip_fail(e, "forward launch");
  if (pe.stop && (e = hipEventRecord(pe.stop, stream)) != hipSuccess) return hip_fail(e, "event record");
  return CHUNK_ATTN_OK;
}

int chunk_attn_fwd_static(const chunk_attn_desc* desc, const void* q, const void* k, const void* v, void* o, float* lse,
                          void* stream_v) {
  const int rc = validate(desc);
  if (rc != CHUNK_ATTN_OK) return rc;
  if (!q || !k || !v || !o || !lse) return CHUNK_ATTN_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || (reinterpret_cast<uintptr_t>(lse) & 3) != 0)
    return CHUNK_ATTN_INVALID_ARG;
  const chunk_attn_desc wide = is_narrow(desc) ? widened(desc) : *desc;
  FwdLayout L;
  layout_fwd(&wide, L, false);
  const NarrowFwdLayout N = is_narrow(desc) ? narrow_fwd_layout(desc, L.total) : NarrowFwdLayout{0, 0, 0, 0, 0, L.total};
  if (desc->num_segments > kStaticMaxSegments || N.total > kStaticScratchBytes || L.blocks > 0x7fffffff)
    return CHUNK_ATTN_TOO_LARGE;
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  char* ws = nullptr;
  hipError_t e = static_scratch(&ws);
  if (e != hipSuccess) return hip_fail(e, "address of the static scratch buffer");
  void* o_user = o;
  const int64_t qr = (int64_t)desc->total_q * desc->num_q_heads, kr = (int64_t)desc->total_kv * desc->num_kv_heads;
  if (is_narrow(desc)) {  // zero-padded copies at the head of the scratch array, the head_dim 128 forward behind them
    if ((e = pad_rows(q, ws + N.q_off, qr, 2, stream)) != hipSuccess || (e = pad_rows(k, ws + N.k_off, kr, 2, stream)) != hipSuccess ||
        (e = pad_rows(v, ws + N.v_off, kr, 2, stream)) != hipSuccess)
      return hip_fail(e, "padding launch");
    q = ws + N.q_off;
    k = ws + N.k_off;
    v = ws + N.v_off;
    o = ws + N.o_off;
    ws += N.inner_off;
    desc = &wide;
  }

  StaticSegs segs;
  for (int t = 0; t < desc->num_segments; ++t) segs.seg[t] = desc->segments[t];
  const int n_items = (int)(L.items_bytes / sizeof(FwdItem));
  hipLaunchKernelGGL(plan_fwd_static_kernel, dim3(1), dim3(256), 0, stream, segs, desc->num_segments, L.tile_rows,
                     reinterpret_cast<FwdItem*>(ws), n_items, reinterpret_cast<TileJob*>(ws + L.jobs_off), (int)L.kv_tiles,
                     reinterpret_cast<int32_t*>(ws + L.flags_off), (int)L.blocks + 1 + kBlockQueues);
  if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e, "schedule kernel launch");

  FwdParams p;
  p.q = static_cast<const __bf16*>(q);
  p.k = static_cast<const __bf16*>(k);
  p.v = static_cast<const __bf16*>(v);
  p.o = static_cast<__bf16*>(o);
  p.lse = lse;
  p.vt = reinterpret_cast<__bf16*>(ws + L.vt_off);
  p.items = reinterpret_cast<const FwdItem*>(ws);
  p.total_kv_tiles = L.kv_tiles;
  p.num_q_heads = desc->num_q_heads;
  p.num_kv_heads = desc->num_kv_heads;
  p.group = desc->num_q_heads / desc->num_kv_heads;
  p.heads_per_wg = heads_per_wg(p.group, fwd_waves(desc->head_dim));
  p.head_splits = p.group / p.heads_per_wg;
  p.total_q = desc->total_q;
  p.scale_log2 = desc->softmax_scale * 1.4426950408889634f;
  p.redo = desc->head_dim == 128 ? reinterpret_cast<int32_t*>(ws + L.flags_off) : nullptr;
  p.any_redo = reinterpret_cast<int32_t*>(ws + L.flags_off) + L.blocks;
  p.taken = p.any_redo + 1;
  p.clock_log = clock_log(0);
  p.ref_limit = g_fwd_rescale_limit.load();
  e = launch_fwd(p, desc->head_dim, (int)L.blocks, reinterpret_cast<const TileJob*>(ws + L.jobs_off), (int)L.kv_tiles, stream);
  if (e != hipSuccess) return hip_fail(e, "forward launch");
  if (o != o_user && (e = unpad_rows(o, o_user, qr, 2, stream)) != hipSuccess) return hip_fail(e, "unpadding launch");
  return CHUNK_ATTN_OK;
}

namespace {
int bwd_any(const chunk_attn_desc* desc, const void* q, const void* k, const void* v, const void* o, const void* d_o,
            const float* lse, void* dq, void* dk, void* dv, bool dkv_f32, int accumulate_dkv, void* workspace,
            size_t workspace_bytes, void* stream_v) {
  const int rc = validate(desc);
  if (rc != CHUNK_ATTN_OK) return rc;
  if (!q || !k || !v || !o || !d_o || !lse || !dq || !dk || !dv || !workspace) return CHUNK_ATTN_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) != 0) return CHUNK_ATTN_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(d_o) || !aligned16(dq) || !aligned16(dk) ||
      !aligned16(dv) || (reinterpret_cast<uintptr_t>(lse) & 3) != 0)
    return CHUNK_ATTN_INVALID_ARG;  // the kernels move rows in 16-byte pieces
  if (is_narrow(desc)) {  // run as head_dim 128 on zero-padded copies
    const chunk_attn_desc w = widened(desc);
    BwdPlan Pw;
    bwd_layout(&w, Pw, false);
    const NarrowBwdLayout N = narrow_bwd_layout(desc, Pw.total);
    if (workspace_bytes < N.total) return CHUNK_ATTN_WORKSPACE_TOO_SMALL;
    hipStream_t st = static_cast<hipStream_t>(stream_v);
    char* base = static_cast<char*>(workspace);
    const int64_t qr = (int64_t)desc->total_q * desc->num_q_heads, kr = (int64_t)desc->total_kv * desc->num_kv_heads;
    const size_t ge = dkv_f32 ? 4 : 2;
    hipError_t pe;
    if ((pe = pad_rows(q, base + N.q_off, qr, 2, st)) != hipSuccess || (pe = pad_rows(k, base + N.k_off, kr, 2, st)) != hipSuccess ||
        (pe = pad_rows(v, base + N.v_off, kr, 2, st)) != hipSuccess || (pe = pad_rows(o, base + N.o_off, qr, 2, st)) != hipSuccess ||
        (pe = pad_rows(d_o, base + N.do_off, qr, 2, st)) != hipSuccess)
      return hip_fail(pe, "padding launch");
    // accumulating calls add to what dk / dv hold and leave the rows outside every key range as they are
    if (accumulate_dkv && ((pe = pad_rows(dk, base + N.dk_off, kr, ge, st)) != hipSuccess ||
                           (pe = pad_rows(dv, base + N.dv_off, kr, ge, st)) != hipSuccess))
      return hip_fail(pe, "padding launch");
    const int r = bwd_any(&w, base + N.q_off, base + N.k_off, base + N.v_off, base + N.o_off, base + N.do_off, lse,
                          base + N.dq_off, base + N.dk_off, base + N.dv_off, dkv_f32, accumulate_dkv, base + N.inner_off,
                          workspace_bytes - N.inner_off, stream_v);
    if (r != CHUNK_ATTN_OK) return r;
    if ((pe = unpad_rows(base + N.dq_off, dq, qr, 2, st)) != hipSuccess || (pe = unpad_rows(base + N.dk_off, dk, kr, ge, st)) != hipSuccess ||
        (pe = unpad_rows(base + N.dv_off, dv, kr, ge, st)) != hipSuccess)
      return hip_fail(pe, "unpadding launch");
    return CHUNK_ATTN_OK;
  }
  BwdPlan P;
  bwd_layout(desc, P, true);
  if (workspace_bytes < P.total) return CHUNK_ATTN_WORKSPACE_TOO_SMALL;
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  BwdArgs a;
  a.q = static_cast<const __bf16*>(q);
  a.k = static_cast<const __bf16*>(k);
  a.v = static_cast<const __bf16*>(v);
  a.o = static_cast<const __bf16*>(o);
  a.d_o = static_cast<const __bf16*>(d_o);
  a.lse = lse;
  a.dq = static_cast<__bf16*>(dq);
  a.dk = static_cast<__bf16*>(dk);
  a.dv = static_cast<__bf16*>(dv);
  a.accumulate = accumulate_dkv != 0;
  a.dkv_f32 = dkv_f32;
  a.workspace = static_cast<char*>(workspace);
  const std::vector<char> blob = bwd_blob(P);
  hipError_t e = g_ring.upload(a.workspace, blob.data(), blob.size(), stream);
  if (e != hipSuccess) return hip_fail(e, "schedule upload");
  e = launch_bwd(desc, a, P, stream);
  if (e != hipSuccess) return hip_fail(e, "backward launch");
  return CHUNK_ATTN_OK;
}
}  // namespace

int chunk_attn_bwd(const chunk_attn_desc* desc, const void* q, const void* k, const void* v, const void* o,
                   const void* d_o, const float* lse, void* dq, void* dk, void* dv, int accumulate_dkv,
                   void* workspace, size_t workspace_bytes, void* stream_v) {
  return bwd_any(desc, q, k, v, o, d_o, lse, dq, dk, dv, false, accumulate_dkv, workspace, workspace_bytes, stream_v);
}

int chunk_attn_bwd_f32kv(const chunk_attn_desc* desc, const void* q, const void* k, const void* v, const void* o,
                         const void* d_o, const float* lse, void* dq, float* dk, float* dv, int accumulate_dkv,
                         void* workspace, size_t workspace_bytes, void* stream_v) {
  return bwd_any(desc, q, k, v, o, d_o, lse, dq, dk, dv, true, accumulate_dkv, workspace, workspace_bytes, stream_v);
}

}  // extern "C"
