// C-ABI layer of the GPU entry points: argument checks, plan object, pointer-table staging.
// (The entry points that need no GPU are in bcp_host.cpp.)
#include <algorithm>
#include <chrono>
#include <cstring>
#include <mutex>
#include <new>
#include <unordered_map>
#include <vector>

#include "bcp_internal.h"

namespace bcp {

namespace {
PlanConfig g_config;
std::mutex g_config_mu;
}  // namespace

bcp_status hip_fail(hipError_t e, const char* what) {
  set_error(std::string(what) + ": " + hipGetErrorString(e));
  if (e == hipErrorOutOfMemory) return BCP_ERR_OOM;
  if (e == hipErrorNoDevice || e == hipErrorInvalidDevice) return BCP_ERR_NO_DEVICE;
  return BCP_ERR_HIP;
}

PlanConfig config() {
  std::lock_guard<std::mutex> g(g_config_mu);
  return g_config;
}

}  // namespace bcp

using namespace bcp;

// Buffer pointers normally travel as kernel arguments.  Only a table too big for that
// (more than kMaxKernargPtrs buffers) goes host -> device through a small ring of pinned staging
// slots, set up at the first such call, so an asynchronous call never reads a slot a later call
// already rewrote.
constexpr int kSlots = 8;

struct bcp_plan_s {
  PlanDevice dev;
  bcp_stats stats{};
  int device = 0;
  void* table_dev = nullptr;   // [src pointers | dst pointers]
  char* table_host = nullptr;  // pinned, kSlots slots
  size_t table_bytes = 0;
  int32_t n_src = 0, n_dst = 0;
  std::vector<int64_t> src_extent, dst_extent;  // per buffer: one past the highest byte the plan touches
  hipEvent_t slot_done[kSlots]{};
  bool slot_used[kSlots]{};
  int next_slot = 0;
  std::mutex mu;
  std::vector<hipEvent_t> chunk_events;  // bcp_reshard_from_host: one per chunk in flight, reused
  std::mutex chunk_mu;
  bool used = false;                 // a copy kernel was launched on this plan,
  hipStream_t last_stream = nullptr; // most recently on this stream
};

extern "C" {

bcp_status bcp_release_workspace(int64_t* freed_bytes) { return release_workspace(freed_bytes); }

bcp_status bcp_configure(int64_t tile_bytes, int32_t persistent, int32_t wg_per_cu, int32_t threads) try {
  std::lock_guard<std::mutex> g(g_config_mu);
  if (tile_bytes > 0) {
    if (tile_bytes < 4096 || tile_bytes > (4 << 20) || (tile_bytes & (tile_bytes - 1))) {
      set_error("tile_bytes must be a power of two in [4 KiB, 4 MiB]");
      return BCP_ERR_INVALID_ARG;
    }
    g_config.tile_bytes = tile_bytes;
  }
  if (persistent >= 0) g_config.persistent = persistent ? 1 : 0;
  if (wg_per_cu > 0) {
    if (wg_per_cu > 64) {
      set_error("wg_per_cu must be <= 64");
      return BCP_ERR_INVALID_ARG;
    }
    g_config.wg_per_cu = wg_per_cu;
  }
  if (threads > 0) {
    if (threads != 256 && threads != 512 && threads != 1024) {
      set_error("threads must be 256, 512 or 1024");
      return BCP_ERR_INVALID_ARG;
    }
    g_config.threads = threads;
  }
  return BCP_OK;
} catch (...) {
  return on_exception("bcp_configure");
}

// ---- plan ------------------------------------------------------------------------------------
bcp_status bcp_plan(const bcp_shard_meta* saved, int64_t n_saved, const bcp_shard_meta* target, int64_t n_target,
                    uint32_t flags, void* stream, bcp_plan_t* out_plan) try {
  const auto t0 = std::chrono::steady_clock::now();
  if (!out_plan) {
    set_error("bcp_plan: out_plan is null");
    return BCP_ERR_INVALID_ARG;
  }
  *out_plan = nullptr;
  if (n_saved < 0 || n_target < 0 || (n_saved > 0 && !saved) || (n_target > 0 && !target)) {
    set_error("bcp_plan: null metadata array or negative count");
    return BCP_ERR_INVALID_ARG;
  }
  if (flags & ~(BCP_ALLOW_UNCOVERED | BCP_SKIP_OVERLAP_CHECK | BCP_ORDER_BY_SOURCE | BCP_META_ON_DEVICE |
                BCP_CONVERT_F32_TO_BF16)) {
    set_error("bcp_plan: unknown flag");
    return BCP_ERR_INVALID_ARG;
  }
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) {
    set_error("bcp_plan: no HIP device available");
    return BCP_ERR_NO_DEVICE;
  }
  bcp_plan_s* plan = new (std::nothrow) bcp_plan_s();
  if (!plan) {
    set_error("bcp_plan: host allocation failed");
    return BCP_ERR_OOM;
  }
  struct Guard {  // an exception on the way must not leak the plan
    bcp_plan_s* p;
    ~Guard() {
      if (p) bcp_plan_destroy(p);
    }
  } guard{plan};
  bcp_status s = BCP_OK;
  PlannerResult res;
  do {
    if (hipGetDevice(&plan->device) != hipSuccess) {
      set_error("bcp_plan: hipGetDevice failed");
      s = BCP_ERR_NO_DEVICE;
      break;
    }
    s = run_planner(saved, n_saved, target, n_target, flags, (hipStream_t)stream, &res);
    if (s != BCP_OK) break;
    plan->dev = res.dev;
    bcp_stats& st = plan->stats;
    st.n_saved_boxes = res.n_saved_boxes;
    st.n_target_boxes = res.n_target_boxes;
    st.n_pairs = (int64_t)res.ctl.n_pairs;
    st.n_regions = (int64_t)res.ctl.n_regions;
    st.n_tiles = (int64_t)res.ctl.n_tiles;
    st.payload_bytes = (int64_t)res.ctl.payload_bytes;
    st.n_transposed = (int64_t)res.ctl.n_transposed;
    st.max_src_buf = res.ctl.max_src_buf;
    st.max_dst_buf = res.ctl.max_dst_buf;
    for (int k = 0; k <= BCP_MAX_DIMS; ++k) st.region_dims_hist[k] = (int64_t)res.ctl.dims_hist[k];
    st.plan_device_ms = res.device_ms;
    st.n_batches = res.dev.n_batches;
    st.src_bytes = (int64_t)res.ctl.src_bytes;
    plan->src_extent = std::move(res.src_extent);
    plan->dst_extent = std::move(res.dst_extent);
    plan->n_src = (int32_t)(st.max_src_buf + 1);
    plan->n_dst = (int32_t)(st.max_dst_buf + 1);
    plan->table_bytes = sizeof(void*) * (size_t)(plan->n_src + plan->n_dst);
  } while (0);
  if (s != BCP_OK) return s;  // the guard destroys the plan; destroying sets no error text
  plan->stats.plan_wall_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
  guard.p = nullptr;
  *out_plan = plan;
  return BCP_OK;
} catch (...) {
  return on_exception("bcp_plan");
}

bcp_status bcp_plan_destroy(bcp_plan_t plan) try {
  if (!plan) return BCP_OK;
  // back to the block pool, ordered behind the last launch that reads them
  block_free(plan->dev.regions, plan->dev.regions_bytes, plan->used, plan->last_stream);
  block_free(plan->dev.heads, plan->dev.desc_bytes, plan->used, plan->last_stream);  // heads | tiles | queue
  if (plan->table_dev) (void)hipFree(plan->table_dev);
  if (plan->table_host) (void)hipHostFree(plan->table_host);
  for (int i = 0; i < kSlots; ++i)
    if (plan->slot_done[i]) (void)hipEventDestroy(plan->slot_done[i]);
  for (hipEvent_t e : plan->chunk_events) (void)hipEventDestroy(e);
  delete plan;
  return BCP_OK;
} catch (...) {
  return on_exception("bcp_plan_destroy");
}

bcp_status bcp_plan_stats(bcp_plan_t plan, bcp_stats* out) try {
  if (!plan || !out) {
    set_error("bcp_plan_stats: null argument");
    return BCP_ERR_INVALID_ARG;
  }
  *out = plan->stats;
  return BCP_OK;
} catch (...) {
  return on_exception("bcp_plan_stats");
}

bcp_status bcp_plan_regions(bcp_plan_t plan, bcp_region_info* out, int64_t capacity, int64_t* n_regions) try {
  if (!plan || !n_regions || capacity < 0 || (capacity > 0 && !out)) {
    set_error("bcp_plan_regions: bad argument");
    return BCP_ERR_INVALID_ARG;
  }
  *n_regions = plan->dev.n_regions;
  const int64_t n = std::min(capacity, plan->dev.n_regions);
  if (n == 0) return BCP_OK;
  std::vector<Region> tmp((size_t)n);
  BCP_HIP(hipMemcpy(tmp.data(), plan->dev.regions, sizeof(Region) * (size_t)n, hipMemcpyDeviceToHost));
  for (int64_t i = 0; i < n; ++i) {
    const Region& r = tmp[(size_t)i];
    bcp_region_info& o = out[i];
    std::memset(&o, 0, sizeof(o));
    o.src_base = r.src_base;
    o.dst_base = r.dst_base;
    o.run_bytes = r.run_bytes;
    for (int k = 0; k < BCP_MAX_DIMS; ++k) {
      o.len[k] = r.len[k];
      o.src_pitch[k] = r.spitch[k];
      o.dst_pitch[k] = r.dpitch[k];
    }
    o.ndim = r.ndim;
    o.src_buf = r.src_buf;
    o.dst_buf = r.dst_buf;
    o.kind = r.kind;
    o.target_index = r.trec;
    o.saved_index = r.srec;
  }
  return BCP_OK;
} catch (...) {
  return on_exception("bcp_plan_regions");
}

bcp_status bcp_plan_buffer_extents(bcp_plan_t plan, int64_t* src_extent, int32_t n_src, int64_t* dst_extent,
                                   int32_t n_dst) try {
  if (!plan || n_src < plan->n_src || n_dst < plan->n_dst || (n_src > 0 && !src_extent) || (n_dst > 0 && !dst_extent)) {
    set_error("bcp_plan_buffer_extents: bad argument");
    return BCP_ERR_INVALID_ARG;
  }
  for (int32_t i = 0; i < n_src; ++i) src_extent[i] = (size_t)i < plan->src_extent.size() ? plan->src_extent[(size_t)i] : 0;
  for (int32_t i = 0; i < n_dst; ++i) dst_extent[i] = (size_t)i < plan->dst_extent.size() ? plan->dst_extent[(size_t)i] : 0;
  return BCP_OK;
} catch (...) {
  return on_exception("bcp_plan_buffer_extents");
}

// ---- reshard ---------------------------------------------------------------------------------
// argument checks shared by the reshard entry points (a plan without tiles accepts anything)
static bcp_status check_reshard_args(bcp_plan_t plan, const void* const* src_blobs, int32_t n_src,
                                     void* const* dst_buffers, int32_t n_dst, const char* who) {
  if (!plan) {
    set_error(std::string(who) + ": plan is null");
    return BCP_ERR_INVALID_ARG;
  }
  if (plan->dev.n_tiles == 0) return BCP_OK;
  if (!src_blobs || !dst_buffers || n_src < plan->n_src || n_dst < plan->n_dst) {
    set_error(std::string(who) + ": need at least " + std::to_string(plan->n_src) + " source and " +
              std::to_string(plan->n_dst) + " destination buffers");
    return BCP_ERR_INVALID_ARG;
  }
  for (int32_t i = 0; i < plan->n_src; ++i)
    if (!src_blobs[i]) {
      set_error(std::string(who) + ": src_blobs[" + std::to_string(i) + "] is null");
      return BCP_ERR_INVALID_ARG;
    }
  for (int32_t i = 0; i < plan->n_dst; ++i)
    if (!dst_buffers[i]) {
      set_error(std::string(who) + ": dst_buffers[" + std::to_string(i) + "] is null");
      return BCP_ERR_INVALID_ARG;
    }
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != plan->device) {
    set_error(std::string(who) + ": the plan belongs to another device");
    return BCP_ERR_INVALID_ARG;
  }
  return BCP_OK;
}

static bcp_status reshard_impl(bcp_plan_t plan, const void* const* src_blobs, int32_t n_src, void* const* dst_buffers,
                               int32_t n_dst, void* stream, const uint64_t* key_range, const char* who) {
  if (bcp_status s = check_reshard_args(plan, src_blobs, n_src, dst_buffers, n_dst, who)) return s;
  if (plan->dev.n_tiles == 0) return BCP_OK;
  hipStream_t st = (hipStream_t)stream;
  plan->used = true;
  plan->last_stream = st;
  if (plan->n_src + plan->n_dst <= kMaxKernargPtrs)
    return launch_reshard(plan->dev, src_blobs, plan->n_src, dst_buffers, plan->n_dst, nullptr, st, key_range);
  std::lock_guard<std::mutex> g(plan->mu);
  if (!plan->table_dev) {
    hipError_t e = hipMalloc(&plan->table_dev, plan->table_bytes);
    if (e == hipSuccess) e = hipHostMalloc((void**)&plan->table_host, plan->table_bytes * kSlots, hipHostMallocDefault);
    for (int i = 0; i < kSlots && e == hipSuccess; ++i) e = hipEventCreateWithFlags(&plan->slot_done[i], hipEventDisableTiming);
    if (e != hipSuccess) return hip_fail(e, "pointer table allocation");
  }
  const int slot = plan->next_slot;
  plan->next_slot = (slot + 1) % kSlots;
  if (plan->slot_used[slot]) BCP_HIP(hipEventSynchronize(plan->slot_done[slot]));
  char* h = plan->table_host + plan->table_bytes * (size_t)slot;
  std::memcpy(h, src_blobs, sizeof(void*) * (size_t)plan->n_src);
  std::memcpy(h + sizeof(void*) * (size_t)plan->n_src, dst_buffers, sizeof(void*) * (size_t)plan->n_dst);
  BCP_HIP(hipMemcpyAsync(plan->table_dev, h, plan->table_bytes, hipMemcpyHostToDevice, st));
  BCP_HIP(hipEventRecord(plan->slot_done[slot], st));
  plan->slot_used[slot] = true;
  return launch_reshard(plan->dev, nullptr, plan->n_src, nullptr, plan->n_dst, plan->table_dev, st, key_range);
}

bcp_status bcp_reshard(bcp_plan_t plan, const void* const* src_blobs, int32_t n_src, void* const* dst_buffers,
                       int32_t n_dst, void* stream) try {
  return reshard_impl(plan, src_blobs, n_src, dst_buffers, n_dst, stream, nullptr, "bcp_reshard");
} catch (...) {
  return on_exception("bcp_reshard");
}

bcp_status bcp_reshard_checked(bcp_plan_t plan, const void* const* src_blobs, const int64_t* src_bytes, int32_t n_src,
                               void* const* dst_buffers, const int64_t* dst_bytes, int32_t n_dst, void* stream) try {
  if (bcp_status s = check_reshard_args(plan, src_blobs, n_src, dst_buffers, n_dst, "bcp_reshard_checked")) return s;
  if (plan->dev.n_tiles == 0) return BCP_OK;
  if (!src_bytes || !dst_bytes) {
    set_error("bcp_reshard_checked: null size array");
    return BCP_ERR_INVALID_ARG;
  }
  for (int side = 0; side < 2; ++side) {
    const std::vector<int64_t>& need = side ? plan->dst_extent : plan->src_extent;
    const int64_t* have = side ? dst_bytes : src_bytes;
    for (size_t i = 0; i < need.size(); ++i)
      if (have[i] < need[i]) {
        set_error(std::string("bcp_reshard_checked: ") + (side ? "dst_buffers[" : "src_blobs[") + std::to_string(i) + "] holds " +
                  std::to_string(have[i]) + " bytes, the plan touches " + std::to_string(need[i]));
        return BCP_ERR_OUT_OF_BOUNDS;
      }
  }
  return reshard_impl(plan, src_blobs, n_src, dst_buffers, n_dst, stream, nullptr, "bcp_reshard_checked");
} catch (...) {
  return on_exception("bcp_reshard_checked");
}

bcp_status bcp_reshard_noalloc(bcp_plan_t plan, const void* const* src_blobs, int32_t n_src, void* const* dst_buffers,
                               int32_t n_dst, void* stream) try {
  if (bcp_status s = check_reshard_args(plan, src_blobs, n_src, dst_buffers, n_dst, "bcp_reshard_noalloc")) return s;
  if (plan->dev.n_tiles == 0) return BCP_OK;
  plan->used = true;
  plan->last_stream = (hipStream_t)stream;
  return launch_reshard_noalloc(plan->dev, src_blobs, plan->n_src, dst_buffers, plan->n_dst, (hipStream_t)stream);
} catch (...) {
  return on_exception("bcp_reshard_noalloc");
}

bcp_status bcp_reshard_arrived(bcp_plan_t plan, const void* const* src_blobs, int32_t n_src, void* const* dst_buffers,
                               int32_t n_dst, int32_t src_buf, int64_t byte_begin, int64_t byte_end, void* stream) try {
  if (src_buf < 0 || byte_begin < 0 || byte_end < byte_begin || (byte_end >> kKeyShift)) {
    set_error("bcp_reshard_arrived: bad source range");
    return BCP_ERR_INVALID_ARG;
  }
  if (plan && plan->dev.n_tiles && !plan->dev.batch_key) {
    set_error("bcp_reshard_arrived: the plan was not built with BCP_ORDER_BY_SOURCE");
    return BCP_ERR_INVALID_ARG;
  }
  const uint64_t range[2] = {((uint64_t)src_buf << kKeyShift) | (uint64_t)byte_begin,
                             ((uint64_t)src_buf << kKeyShift) | (uint64_t)byte_end};
  return reshard_impl(plan, src_blobs, n_src, dst_buffers, n_dst, stream, range, "bcp_reshard_arrived");
} catch (...) {
  return on_exception("bcp_reshard_arrived");
}

bcp_status bcp_reshard_from_host(bcp_plan_t plan, const void* const* host_blobs, const int64_t* blob_bytes,
                                 void* const* src_blobs, int32_t n_src, void* const* dst_buffers, int32_t n_dst,
                                 int64_t chunk_bytes, void* copy_stream, void* stream) try {
  if (!plan || !host_blobs || !blob_bytes || chunk_bytes <= 0) {
    set_error("bcp_reshard_from_host: bad argument");
    return BCP_ERR_INVALID_ARG;
  }
  if (copy_stream == stream) {
    set_error("bcp_reshard_from_host: the copy stream and the reshard stream must differ");
    return BCP_ERR_INVALID_ARG;
  }
  if (bcp_status s = check_reshard_args(plan, src_blobs, n_src, dst_buffers, n_dst, "bcp_reshard_from_host")) return s;
  if (plan->dev.n_tiles == 0) return BCP_OK;
  if (!plan->dev.batch_key) {
    set_error("bcp_reshard_from_host: the plan was not built with BCP_ORDER_BY_SOURCE");
    return BCP_ERR_INVALID_ARG;
  }
  // every blob is looked at before anything is queued
  for (int32_t b = 0; b < plan->n_src; ++b) {
    if (blob_bytes[b] < 0 || (blob_bytes[b] > 0 && !host_blobs[b])) {
      set_error("bcp_reshard_from_host: blob " + std::to_string(b) + " has no host buffer");
      return BCP_ERR_INVALID_ARG;
    }
    if (blob_bytes[b] < plan->src_extent[(size_t)b]) {  // its last regions would wait for bytes that never arrive
      set_error("bcp_reshard_from_host: blob " + std::to_string(b) + " holds " + std::to_string(blob_bytes[b]) +
                " bytes, the plan reads " + std::to_string(plan->src_extent[(size_t)b]));
      return BCP_ERR_OUT_OF_BOUNDS;
    }
  }
  hipStream_t cs = (hipStream_t)copy_stream;
  hipStream_t st = (hipStream_t)stream;
  // the copy stream starts after whatever the reshard stream has queued (buffers may still be in use)
  hipEvent_t ev;
  std::vector<hipEvent_t>& pool = plan->chunk_events;
  size_t used = 0;
  auto next_event = [&](hipEvent_t* out) -> hipError_t {
    if (used == pool.size()) {
      hipEvent_t e;
      hipError_t rc = hipEventCreateWithFlags(&e, hipEventDisableTiming);
      if (rc != hipSuccess) return rc;
      pool.push_back(e);
    }
    *out = pool[used++];
    return hipSuccess;
  };
  std::lock_guard<std::mutex> g(plan->chunk_mu);
  BCP_HIP(next_event(&ev));
  BCP_HIP(hipEventRecord(ev, st));
  BCP_HIP(hipStreamWaitEvent(cs, ev, 0));
  for (int32_t b = 0; b < plan->n_src; ++b) {
    for (int64_t off = 0; off < blob_bytes[b]; off += chunk_bytes) {
      const int64_t n = std::min(chunk_bytes, blob_bytes[b] - off);
      BCP_HIP(hipMemcpyAsync((char*)src_blobs[b] + off, (const char*)host_blobs[b] + off, (size_t)n,
                             hipMemcpyHostToDevice, cs));
      BCP_HIP(next_event(&ev));
      BCP_HIP(hipEventRecord(ev, cs));
      BCP_HIP(hipStreamWaitEvent(st, ev, 0));
      // everything whose last source byte lies in this chunk can go now
      if (bcp_status s = bcp_reshard_arrived(plan, src_blobs, n_src, dst_buffers, n_dst, b, off, off + n, stream)) return s;
    }
  }
  return BCP_OK;
} catch (...) {
  return on_exception("bcp_reshard_from_host");
}

}  // extern "C"
