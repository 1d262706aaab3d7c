// GPU planner: from saved / target shard records to copy regions, tiles and batches.
//
// Sec. 3.3 Step 2 of the paper ("identifying matching segments between the saved tensor shards
// and the sharding specification of new shards") run as data-parallel kernels:
//   1. validate every record and count the regular boxes it decomposes into (Sec. 3.2
//      "Decomposing irregular tensors"), exclusive scan, emit the boxes;
//   2. sort the saved boxes by FQN (LSD radix sort, 4-bit digits, stable);
//   3. per target box, find its FQN's run of saved boxes; scan the candidate-pair counts;
//   4. one thread per candidate pair: intersect the two boxes; wave ballot + prefix to list the
//      non-empty intersections of every block of pairs; then one thread per listed pair: the region,
//      normalised on the spot (unit dims dropped, dims contiguous on both sides merged) and tiled,
//      written into a dense, deterministic region list;
//   5. scan the tile counts; weigh the tiles, group runs of small tiles into batches, and write one
//      fully decoded descriptor per batch head (and per small tile);
//   plus the checks: coverage of every target record, saved shards pairwise disjoint, records of
//   one FQN agreeing on shape and itemsize.
// Temporaries live in a process-wide, grow-only workspace, so a plan costs three device
// allocations of its own (regions, descriptors, queue words) and four host synchronisations.
#include <algorithm>
#include <cstring>
#include <mutex>
#include <vector>

#include "bcp_internal.h"

namespace bcp {
namespace {

constexpr int kBlock = 256;
constexpr int kScanItems = 4;         // items per thread in the multi-block scan
constexpr int kSmallScanThreads = 1024;
constexpr int64_t kSmallScanMax = 1 << 14;  // up to here one workgroup scans alone (one launch)
constexpr uint64_t kSegmentAlign = 256;     // destination alignment of the cuts inside long rows

using ull = unsigned long long;

__device__ inline unsigned lane_id() { return threadIdx.x & 63u; }

template <typename T>
__device__ inline T wave_inclusive_scan(T v) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    T o = __shfl_up(v, d, 64);
    if (lane_id() >= (unsigned)d) v += o;
  }
  return v;
}

// Exclusive scan of one value per thread over the workgroup (a multiple of 64 threads, at most
// 1024); *total gets the workgroup sum.  lds: at least 16 entries.
template <typename T>
__device__ inline T block_exclusive_scan(T v, T* total, T* lds) {
  const T inc = wave_inclusive_scan(v);
  const unsigned w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  if (lane_id() == 63) lds[w] = inc;
  __syncthreads();
  T woff = 0, tot = 0;
  for (unsigned i = 0; i < nw; ++i) {
    const T c = lds[i];
    if (i < w) woff += c;
    tot += c;
  }
  __syncthreads();
  *total = tot;
  return woff + inc - v;
}

// ---- device-wide exclusive scan: out[i] = sum(in[0..i)), out[n] = total --------------------
template <typename Tin, typename T>
__global__ __launch_bounds__(kBlock) void k_scan_reduce(const Tin* in, int64_t n, T* part) {
  __shared__ T lds[16];
  const int64_t base = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * kScanItems;
  T s = 0;
  for (int i = 0; i < kScanItems; ++i)
    if (base + i < n) s += (T)in[base + i];
  T tot;
  block_exclusive_scan(s, &tot, lds);
  if (threadIdx.x == 0) part[blockIdx.x] = tot;
}

template <typename T>
__global__ __launch_bounds__(kSmallScanThreads) void k_scan_parts(T* part, int64_t nb) {
  __shared__ T lds[16];
  T carry = 0;
  for (int64_t base = 0; base < nb; base += blockDim.x) {
    const int64_t i = base + threadIdx.x;
    const T v = i < nb ? part[i] : (T)0;
    T tot;
    const T ex = block_exclusive_scan(v, &tot, lds);
    if (i < nb) part[i] = carry + ex;
    carry += tot;
  }
}

template <typename Tin, typename T>
__global__ __launch_bounds__(kBlock) void k_scan_final(const Tin* in, int64_t n, const T* part, T* out) {
  __shared__ T lds[16];
  const int64_t base = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * kScanItems;
  T v[kScanItems];
  T s = 0;
  for (int i = 0; i < kScanItems; ++i) {
    v[i] = base + i < n ? (T)in[base + i] : (T)0;
    s += v[i];
  }
  T tot;
  T run = block_exclusive_scan(s, &tot, lds) + part[blockIdx.x];
  for (int i = 0; i < kScanItems; ++i) {
    if (base + i < n) out[base + i] = run;
    run += v[i];
  }
  // the thread that owns the last element also writes the grand total
  if (base < n && base + kScanItems >= n) out[n] = run;
}

// the whole scan in one workgroup (small inputs: one launch instead of three); n >= 0
template <typename Tin, typename T>
__global__ __launch_bounds__(kSmallScanThreads) void k_scan_small(const Tin* in, int64_t n, T* out) {
  __shared__ T lds[16];
  T carry = 0;
  for (int64_t base = 0; base < n; base += (int64_t)blockDim.x * kScanItems) {
    const int64_t i0 = base + (int64_t)threadIdx.x * kScanItems;  // this thread's consecutive items
    T v[kScanItems];
    T s = 0;
#pragma unroll
    for (int u = 0; u < kScanItems; ++u) {
      v[u] = i0 + u < n ? (T)in[i0 + u] : (T)0;
      s += v[u];
    }
    T tot;
    T run = carry + block_exclusive_scan(s, &tot, lds);
#pragma unroll
    for (int u = 0; u < kScanItems; ++u) {
      if (i0 + u < n) out[i0 + u] = run;
      run += v[u];
    }
    carry += tot;
  }
  if (threadIdx.x == 0) out[n] = carry;
}

// ---- workspace -------------------------------------------------------------------------------
// Grow-only cache of device chunks shared by all bcp_plan calls of the process (planning is
// serialised by the mutex).  A plan's temporaries are bump-allocated from it and simply
// forgotten at the end of the call.
struct Workspace {
  struct Chunk {
    char* base;
    size_t size, used;
    int device;
  };
  std::vector<Chunk> chunks;
  std::mutex mu;
  int device = -1;
  void* landing = nullptr;  // pinned host memory the planner's read-backs arrive in: kernels write into it
  void* landing_dev = nullptr;  // its address on the device
  size_t landing_bytes = 0;
  hipEvent_t ev[2] = {nullptr, nullptr};  // bracket the planner's device work (reused from plan to plan)

  void reset(int dev) {
    if (dev != device) {  // another device: drop everything that belongs to the old one (rare)
      for (Chunk& c : chunks) (void)hipFree(c.base);
      chunks.clear();
      if (landing) {  // kernels of the old device wrote into it through that device's mapping
        (void)hipHostFree(landing);
        landing = landing_dev = nullptr;
        landing_bytes = 0;
      }
      for (hipEvent_t& e : ev)
        if (e) {
          (void)hipEventDestroy(e);
          e = nullptr;
        }
      device = dev;
    }
    for (Chunk& c : chunks) c.used = 0;
  }
  hipError_t raw(void** p, size_t bytes) {
    bytes = (std::max<size_t>(bytes, 1) + 255) & ~(size_t)255;
    for (Chunk& c : chunks)
      if (c.size - c.used >= bytes) {
        *p = c.base + c.used;
        c.used += bytes;
        return hipSuccess;
      }
    size_t sz = std::max<size_t>(bytes, (size_t)8 << 20);
    if (!chunks.empty()) sz = std::max(sz, chunks.back().size * 2);
    void* q = nullptr;
    hipError_t e = hipMalloc(&q, sz);
    if (e != hipSuccess && sz > bytes) e = hipMalloc(&q, sz = bytes);
    if (e != hipSuccess) return e;
    chunks.push_back(Chunk{(char*)q, sz, bytes, device});
    *p = q;
    return hipSuccess;
  }
  template <typename T>
  hipError_t alloc(T** p, size_t count) {
    return raw((void**)p, count * sizeof(T));
  }
};
Workspace g_ws;
}  // namespace

bcp_status release_workspace(int64_t* freed_bytes) {
  std::lock_guard<std::mutex> lock(g_ws.mu);
  int64_t total = 0;
  hipError_t first = hipSuccess;
  for (Workspace::Chunk& c : g_ws.chunks) {
    total += (int64_t)c.size;
    const hipError_t e = hipFree(c.base);
    if (first == hipSuccess) first = e;
  }
  g_ws.chunks.clear();
  if (g_ws.landing) {
    const hipError_t e = hipHostFree(g_ws.landing);
    if (first == hipSuccess) first = e;
    g_ws.landing = nullptr;
    g_ws.landing_dev = nullptr;
    g_ws.landing_bytes = 0;
  }
  for (hipEvent_t& e : g_ws.ev)
    if (e) {
      (void)hipEventDestroy(e);
      e = nullptr;
    }
  total += block_pool_release();
  if (freed_bytes) *freed_bytes = total;
  BCP_HIP(first);
  return BCP_OK;
}

namespace {

inline unsigned blocks_for(int64_t n, int per_block = kBlock) {
  return (unsigned)std::max<int64_t>(1, (n + per_block - 1) / per_block);
}

// in and out may alias when Tin == T.  out has n+1 entries.
template <typename Tin, typename T>
bcp_status device_scan(const Tin* in, T* out, int64_t n, Workspace& ws, hipStream_t st) {
  if (n <= kSmallScanMax) {
    hipLaunchKernelGGL((k_scan_small<Tin, T>), dim3(1), dim3(kSmallScanThreads), 0, st, in, std::max<int64_t>(n, 0), out);
    BCP_HIP(hipGetLastError());
    return BCP_OK;
  }
  const unsigned nb = blocks_for(n, kBlock * kScanItems);
  T* part = nullptr;
  BCP_HIP(ws.alloc(&part, nb));
  hipLaunchKernelGGL((k_scan_reduce<Tin, T>), dim3(nb), dim3(kBlock), 0, st, in, n, part);
  hipLaunchKernelGGL((k_scan_parts<T>), dim3(1), dim3(kSmallScanThreads), 0, st, part, (int64_t)nb);
  hipLaunchKernelGGL((k_scan_final<Tin, T>), dim3(nb), dim3(kBlock), 0, st, in, n, part, out);
  BCP_HIP(hipGetLastError());
  return BCP_OK;
}

// ---- step 1: validate, count and emit boxes --------------------------------------------------
__device__ inline void report(Ctl* ctl, int64_t record, unsigned code) {
  atomicMin(&ctl->err_key, ((ull)record << 8) | code);
}

// The plan's counters and maxima are one small struct, and an atomic on one cache line takes the L2 some
// nanoseconds whoever asks: tens of thousands of workgroups that each add their sums to the same line
// wait for each other longer than they compute.  So the struct exists kCtlStripes + 1 times, 256 bytes
// apart: workgroups add to the copy their index selects, and k_readback folds the copies into the first
// one (and clears them) before the host looks at it.  Errors are rare and go to the first copy directly.
constexpr uint32_t kCtlStripes = 256;
struct alignas(256) CtlStripe {
  Ctl c;
};
__device__ inline Ctl* ctl_stripe(Ctl* ctl) {
  return &(reinterpret_cast<CtlStripe*>(ctl) + 1 + blockIdx.x % kCtlStripes)->c;
}

// (also clears the coverage counters: a fill of its own is one more launch, and a plan for a few thousand
// records is made of launches)
__global__ __launch_bounds__(kBlock) void k_ctl_init(Ctl* ctl, Ctl init, ull* cov, int64_t n_cov) {
  if (blockIdx.x == 0)
    for (uint32_t i = threadIdx.x; i <= kCtlStripes; i += kBlock) reinterpret_cast<CtlStripe*>(ctl)[i].c = init;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n_cov; i += (int64_t)gridDim.x * kBlock) cov[i] = 0;
}

// A record is 304 bytes, and a wave whose lanes each read their own record asks for 64 cache lines with
// every load instruction, most of them several times over.  So the records of a workgroup (they are
// consecutive) come into LDS as one coalesced copy, 16 bytes per lane and instruction, and are looked at there.
constexpr int kRecChunks = (int)(sizeof(bcp_shard_meta) / 16);
static_assert(sizeof(bcp_shard_meta) % 16 == 0, "records are staged in 16-byte pieces");
constexpr int kRecBlock = 128;  // records (threads) per workgroup of the kernels that stage records

// Records rec0 .. rec0 + count of the concatenation [saved | target] come from two arrays (n_saved records in the
// first); `gather`, if not null, receives them as well, as one array: the caller's two arrays -- in device memory,
// or in pinned host memory that the device reads over the bus -- then need no copy of their own before the kernel.
template <bool GATHER>
__device__ inline void stage_records(const bcp_shard_meta* saved, const bcp_shard_meta* target, int64_t n_saved,
                                     int64_t rec0, int count, uint4* lds, bcp_shard_meta* gather) {
  const uint4* __restrict__ from_s = reinterpret_cast<const uint4*>(saved);
  const uint4* __restrict__ from_t = reinterpret_cast<const uint4*>(target);
  uint4* __restrict__ to = reinterpret_cast<uint4*>(gather);
  const int64_t g0 = rec0 * kRecChunks, split = n_saved * kRecChunks;  // in 16-byte pieces
  const int chunks = count * kRecChunks;
  uint4 v[kRecChunks];
#pragma unroll
  for (int j = 0; j < kRecChunks; ++j) {
    const int i = j * kRecBlock + (int)threadIdx.x;
    const int64_t g = g0 + (i < chunks ? i : chunks - 1);  // (count >= 1; the copies of the last piece are not stored)
    const uint4* at = g < split ? from_s + g : from_t + (g - split);  // (the address is chosen, not the value: one load)
    v[j] = *at;
  }
#pragma unroll
  for (int j = 0; j < kRecChunks; ++j) {
    const int i = j * kRecBlock + (int)threadIdx.x;
    if (i < chunks) lds[i] = v[j];
  }
  __syncthreads();
  if (GATHER) {  // (from LDS, not from the registers of the loads: holding them for a second store spills them)
#pragma unroll
    for (int j = 0; j < kRecChunks; ++j) {
      const int i = j * kRecBlock + (int)threadIdx.x;
      if (i < chunks) to[g0 + i] = lds[i];
    }
  }
}

template <bool GATHER>
__global__ __launch_bounds__(kRecBlock) void k_validate_count(const bcp_shard_meta* saved, const bcp_shard_meta* target,
                                                              bcp_shard_meta* gather, int64_t n_saved, int64_t n_total,
                                                              uint32_t* nboxes, Ctl* ctl) {
  // largest saved FQN id and largest buffer indices of the block: one global atomic per block, not per record
  __shared__ ull block_max;
  __shared__ int block_sbuf, block_tbuf;
  __shared__ uint4 staged[kRecBlock * kRecChunks];
  if (threadIdx.x == 0) {
    block_max = 0;
    block_sbuf = block_tbuf = -1;
  }
  const int64_t rec0 = (int64_t)blockIdx.x * kRecBlock;
  stage_records<GATHER>(saved, target, n_saved, rec0, (int)(n_total - rec0 < kRecBlock ? n_total - rec0 : kRecBlock), staged, gather);
  const int64_t i = rec0 + threadIdx.x;
  if (i < n_total) {
    const bcp_shard_meta& r = reinterpret_cast<const bcp_shard_meta*>(staged)[threadIdx.x];
    const unsigned code = validate_record(r);
    if (code) {
      report(ctl, i, code);
      nboxes[i] = 0;
    } else {
      int64_t len[kDims];
      const int n = local_shape(r, len);
      const int nb = decompose_flat_range(len, n, r.flat_begin, r.flat_end, nullptr);
      nboxes[i] = (uint32_t)nb;
      if (i < n_saved && nb && block_max < (ull)r.fqn_id) atomicMax(&block_max, (ull)r.fqn_id);
      int* bb = i < n_saved ? &block_sbuf : &block_tbuf;
      if (*bb < r.buf) atomicMax(bb, r.buf);
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    Ctl* part = ctl_stripe(ctl);
    if (block_max) atomicMax(&part->max_saved_fqn, block_max);
    if (block_sbuf >= 0) atomicMax(&part->max_saved_rec_buf, (long long)block_sbuf);
    if (block_tbuf >= 0) atomicMax(&part->max_target_rec_buf, (long long)block_tbuf);
  }
}

// The boxes of a block's records are consecutive in the output (box_start is a scan), so they are
// put together in LDS and leave as one coalesced copy; a block whose records decompose into more
// boxes than the staging area holds writes them directly.
constexpr uint32_t kStageBoxes = 320;

__global__ __launch_bounds__(kBlock) void k_emit_boxes(const bcp_shard_meta* recs, int64_t n_saved, int64_t n_total,
                                                       const uint32_t* box_start, Box* boxes) {
  __shared__ __attribute__((aligned(16))) char stage[kStageBoxes * sizeof(Box)];
  const int64_t rec0 = (int64_t)blockIdx.x * kBlock;
  const int64_t rec1 = rec0 + kBlock < n_total ? rec0 + kBlock : n_total;
  const uint32_t b0 = box_start[rec0], b1 = box_start[rec1];
  const bool staged = b1 - b0 <= kStageBoxes;
  const int64_t i = rec0 + threadIdx.x;
  if (i < n_total) {
    const uint32_t first = box_start[i];
    const int nb = (int)(box_start[i + 1] - first);
    if (nb) {
      int nb_general = nb;
      const bcp_shard_meta& r = recs[i];
      int64_t len[kDims];
      const int n = local_shape(r, len);
      bool strided = false;
      int64_t vol = 1;
      for (int k = 0; k < r.ndim; ++k) {
        strided |= r.strides[k] != 0;
        vol *= r.lengths[k];
      }
      Box* out = staged ? reinterpret_cast<Box*>(stage) + (first - b0) : boxes + first;
      if (r.flat_begin == 0 && r.flat_end == vol) {
        // a regular shard (the usual case): its one box is the record's box itself, and the general path below,
        // whose list of up to fifteen boxes lives in scratch memory, is not entered
        Box& b = out[0];
        b.fqn = r.fqn_id;
        b.rec = (int32_t)(i < n_saved ? i : i - n_saved);
        b.ndim = n;
        b.itemsize = r.itemsize;
        b.buf = r.buf;
        int64_t st = 1;
        for (int k = kDims - 1; k >= 0; --k) {
          b.off[k] = k < r.ndim ? r.offsets[k] : 0;
          b.len[k] = k < n ? len[k] : 1;
          b.stride[k] = k >= n ? 0 : (strided ? r.strides[k] : st);
          if (k < n) st *= len[k];
        }
        b.byte_base = r.byte_offset;
        nb_general = 0;
      }
      LocalBox lb[kMaxBoxesPerRecord];
      if (nb_general) decompose_flat_range(len, n, r.flat_begin, r.flat_end, lb);
      for (int j = 0; j < nb_general; ++j) {
        Box& b = out[j];
        b.fqn = r.fqn_id;
        b.rec = (int32_t)(i < n_saved ? i : i - n_saved);
        b.ndim = n;
        b.itemsize = r.itemsize;
        b.buf = r.buf;
        for (int k = 0; k < kDims; ++k) {
          b.off[k] = (k < r.ndim ? r.offsets[k] : 0) + (k < n ? lb[j].off[k] : 0);
          b.len[k] = k < n ? lb[j].len[k] : 1;
          b.stride[k] = 0;
        }
        if (strided) {
          for (int k = 0; k < n; ++k) b.stride[k] = r.strides[k];
          b.byte_base = r.byte_offset;
        } else {
          int64_t st = 1;
          for (int k = n - 1; k >= 0; --k) {
            b.stride[k] = st;
            st *= b.len[k];
          }
          b.byte_base = r.byte_offset + (int64_t)r.itemsize * (lb[j].flat_start - r.flat_begin);
        }
      }
    }
  }
  if (!staged) return;  // uniform over the block
  __syncthreads();
  static_assert(sizeof(Box) % 8 == 0, "copied in 8-byte words");
  const uint32_t words = (b1 - b0) * (uint32_t)(sizeof(Box) / 8);
  const uint64_t* from = reinterpret_cast<const uint64_t*>(stage);
  uint64_t* to = reinterpret_cast<uint64_t*>(boxes + b0);
  for (uint32_t w = threadIdx.x; w < words; w += kBlock) to[w] = from[w];
}

// ---- step 2: stable LSD radix sort of (fqn, box index), 4 bits per pass ------------------------
__global__ __launch_bounds__(kBlock) void k_sort_init(const Box* boxes, int64_t n, uint64_t* keys, uint32_t* idx) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= n) return;
  keys[i] = (uint64_t)boxes[i].fqn;
  idx[i] = (uint32_t)i;
}

// The same sort for at most kSortSmallMax boxes in ONE workgroup, keys and both index arrays in LDS: for a plan
// of a few thousand records a pass of the device-wide sort is three launches that take longer to start than to
// run.  Every thread owns kSortSmallItems consecutive positions; per pass it counts its digits (four 16-bit
// counters to a 64-bit word, so four workgroup scans give the sixteen digits' offsets), the totals are
// stacked into digit bases, and the positions are scattered in order: stable like the big one.
constexpr int kSortSmallThreads = 1024;
constexpr int kSortSmallItems = 4;
constexpr int kSortSmallMax = kSortSmallThreads * kSortSmallItems;

__global__ __launch_bounds__(kSortSmallThreads) void k_sort_small(const Box* boxes, int n, int bits, uint64_t* keys_out,
                                                                  uint32_t* idx_out) {
  __shared__ uint64_t key[kSortSmallMax];      // by box index
  __shared__ uint16_t order[2][kSortSmallMax];  // box indices in the current / next order
  __shared__ ull wave_tot[kSortSmallThreads / 64][4];
  const int t = threadIdx.x;
  for (int i = t; i < n; i += kSortSmallThreads) {
    key[i] = (uint64_t)boxes[i].fqn;
    order[0][i] = (uint16_t)i;
  }
  __syncthreads();
  int cur = 0;
  for (int shift = 0; shift < bits; shift += 4) {
    const int j0 = t * kSortSmallItems;
    unsigned dig[kSortSmallItems];
    ull cnt[4] = {0, 0, 0, 0};  // cnt[q]: digits 4q .. 4q+3, 16 bits each (a digit occurs at most 4096 times)
#pragma unroll
    for (int u = 0; u < kSortSmallItems; ++u) {
      dig[u] = j0 + u < n ? (unsigned)(key[order[cur][j0 + u]] >> shift) & 15u : 16u;
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if ((dig[u] >> 2) == (unsigned)q) cnt[q] += 1ull << (16 * (dig[u] & 3u));
    }
    // exclusive scan of the four words over the workgroup, all four side by side: one pair of barriers
    ull inc[4], before[4], total[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) inc[q] = cnt[q];
#pragma unroll
    for (int dlt = 1; dlt < 64; dlt <<= 1) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const ull o = __shfl_up(inc[q], dlt, 64);
        if (lane_id() >= (unsigned)dlt) inc[q] += o;
      }
    }
    if (lane_id() == 63)
#pragma unroll
      for (int q = 0; q < 4; ++q) wave_tot[t >> 6][q] = inc[q];
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      ull below = 0, all = 0;
      for (int w = 0; w < kSortSmallThreads / 64; ++w) {
        const ull c = wave_tot[w][q];
        if (w < (t >> 6)) below += c;
        all += c;
      }
      before[q] = below + inc[q] - cnt[q];
      total[q] = all;
    }
    // base of digit d: occurrences of all smaller digits
    unsigned base[16];
    unsigned run = 0;
#pragma unroll
    for (int d = 0; d < 16; ++d) {
      base[d] = run + (unsigned)((before[d >> 2] >> (16 * (d & 3))) & 0xffffu);
      run += (unsigned)((total[d >> 2] >> (16 * (d & 3))) & 0xffffu);
    }
#pragma unroll
    for (int u = 0; u < kSortSmallItems; ++u) {
      if (dig[u] > 15u) continue;
      unsigned pos = 0;
#pragma unroll
      for (int d = 0; d < 16; ++d)
        if (dig[u] == (unsigned)d) pos = base[d]++;
      order[cur ^ 1][pos] = order[cur][j0 + u];
    }
    __syncthreads();
    cur ^= 1;
  }
  for (int i = t; i < n; i += kSortSmallThreads) {
    const uint16_t b = order[cur][i];
    keys_out[i] = key[b];
    idx_out[i] = b;
  }
}

__global__ __launch_bounds__(kBlock) void k_radix_hist(const uint64_t* keys, int64_t n, int shift, uint32_t* hist,
                                                       unsigned nblk) {
  __shared__ uint32_t h[16];
  if (threadIdx.x < 16) h[threadIdx.x] = 0;
  __syncthreads();
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < n) atomicAdd(&h[(keys[i] >> shift) & 15u], 1u);
  __syncthreads();
  if (threadIdx.x < 16) hist[threadIdx.x * nblk + blockIdx.x] = h[threadIdx.x];
}

__global__ __launch_bounds__(kBlock) void k_radix_scatter(const uint64_t* keys_in, const uint32_t* idx_in, int64_t n,
                                                          int shift, const uint32_t* hist_scan, unsigned nblk,
                                                          uint64_t* keys_out, uint32_t* idx_out) {
  __shared__ uint32_t wc[kBlock / 64][16];
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const bool valid = i < n;
  const uint64_t key = valid ? keys_in[i] : 0;
  const unsigned d = valid ? (unsigned)((key >> shift) & 15u) : 16u;
  const unsigned w = threadIdx.x >> 6;
  const ull lt = (1ull << lane_id()) - 1ull;
  uint32_t rank = 0;
  for (unsigned b = 0; b < 16; ++b) {
    const ull m = __ballot(d == b);
    if (d == b) rank = (uint32_t)__popcll(m & lt);
    if (lane_id() == 0) wc[w][b] = (uint32_t)__popcll(m);
  }
  __syncthreads();
  if (valid) {
    uint32_t base = hist_scan[d * nblk + blockIdx.x];
    for (unsigned v = 0; v < w; ++v) base += wc[v][d];
    keys_out[base + rank] = key;
    idx_out[base + rank] = idx_in[i];
  }
}

// ---- step 3: candidate pairs per target box -----------------------------------------------------
__device__ inline int64_t lower_bound_u64(const uint64_t* a, int64_t n, uint64_t v) {
  int64_t lo = 0, hi = n;
  while (lo < hi) {
    const int64_t mid = (lo + hi) >> 1;
    if (a[mid] < v) lo = mid + 1; else hi = mid;
  }
  return lo;
}
__device__ inline int64_t upper_bound_u64(const uint64_t* a, int64_t n, uint64_t v) {
  int64_t lo = 0, hi = n;
  while (lo < hi) {
    const int64_t mid = (lo + hi) >> 1;
    if (a[mid] <= v) lo = mid + 1; else hi = mid;
  }
  return lo;
}

__global__ __launch_bounds__(kBlock) void k_pair_count(const Box* boxes, int64_t nbs, int64_t nbt,
                                                       const uint64_t* skeys, const uint32_t* sidx,
                                                       const bcp_shard_meta* recs, int64_t n_saved, int convert,
                                                       uint32_t* grp_lo, uint64_t* pair_cnt, Ctl* ctl) {
  const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (t >= nbt) return;
  const Box& tb = boxes[nbs + t];
  const int64_t lo = lower_bound_u64(skeys, nbs, (uint64_t)tb.fqn);
  const int64_t hi = upper_bound_u64(skeys, nbs, (uint64_t)tb.fqn);
  grp_lo[t] = (uint32_t)lo;
  pair_cnt[t] = (uint64_t)(hi - lo);
  if (hi > lo) {
    const Box& sb = boxes[sidx[lo]];
    const unsigned code = same_tensor(recs[sb.rec], recs[n_saved + tb.rec], convert != 0);
    if (code) report(ctl, n_saved + tb.rec, code);
  }
}

__device__ inline bool boxes_intersect(const Box& a, const Box& b) {
  for (int k = 0; k < a.ndim; ++k) {
    const int64_t lo = a.off[k] > b.off[k] ? a.off[k] : b.off[k];
    const int64_t ha = a.off[k] + a.len[k], hb = b.off[k] + b.len[k];
    if (lo >= (ha < hb ? ha : hb)) return false;
  }
  return true;
}

// saved boxes of one FQN must agree on the tensor and be pairwise disjoint (one saver per element,
// Sec. 4.1 "Balancing saving workload"): every sorted position checks itself against the rest of
// its FQN's run.
constexpr int kCheckStep = 4;  // (eight gain nothing more)
__global__ __launch_bounds__(kBlock) void k_saved_check(const Box* boxes, int64_t nbs, const uint64_t* skeys,
                                                        const uint32_t* sidx, const bcp_shard_meta* recs,
                                                        int check_overlap, Ctl* ctl) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= nbs) return;
  const Box& a = boxes[sidx[i]];
  if (i + 1 < nbs && skeys[i + 1] == skeys[i]) {
    const Box& nx = boxes[sidx[i + 1]];
    const unsigned code = same_tensor(recs[a.rec], recs[nx.rec]);
    if (code) {
      report(ctl, nx.rec, code);
      return;
    }
  }
  if (!check_overlap) return;
  // kCheckStep positions of the run per step, their boxes' first dimensions loaded side by side (a step costs one
  // memory round trip, and a run of a flat-sharded tensor has hundreds of boxes, nearly all of them apart
  // in the first dimension already); the rest of a box is looked at only when that one overlaps.
  const uint64_t key = skeys[i];
  const int64_t a_lo = a.off[0], a_hi = a.off[0] + a.len[0];
  for (int64_t j = i + 1; j < nbs; j += kCheckStep) {
    bool in[kCheckStep];
    uint32_t ix[kCheckStep];
    int64_t lo[kCheckStep], ln[kCheckStep];
    int nd[kCheckStep];
#pragma unroll
    for (int u = 0; u < kCheckStep; ++u) {
      in[u] = j + u < nbs && skeys[j + u < nbs ? j + u : i] == key;
      ix[u] = sidx[in[u] ? j + u : i];
    }
#pragma unroll
    for (int u = 0; u < kCheckStep; ++u) {
      const Box& b = boxes[ix[u]];
      lo[u] = b.off[0];
      ln[u] = b.len[0];
      nd[u] = b.ndim;
    }
#pragma unroll
    for (int u = 0; u < kCheckStep; ++u) {
      const int64_t l = a_lo > lo[u] ? a_lo : lo[u], hb = lo[u] + ln[u], h = a_hi < hb ? a_hi : hb;
      if (in[u] && nd[u] == a.ndim && l < h) {
        const Box& b = boxes[ix[u]];
        if (boxes_intersect(a, b)) {
          report(ctl, a.rec > b.rec ? a.rec : b.rec, kErrOverlap);
          return;
        }
      }
    }
    if (!in[kCheckStep - 1]) break;  // the run ends inside this step
  }
}

// ---- step 4: intersect, compact, normalise, tile ------------------------------------------------
// The dimensions of the intersection are merged where both sides are contiguous across them.  The list of
// merged dimensions is written straight into R (lengths, and strides in elements for the moment) while the
// one being merged into stays in registers: the index of the next free slot depends on the data, and an
// array in registers indexed that way costs a chain of selects per access, which R, in LDS or memory, does not.
__device__ inline bool build_region(const Box& s, const Box& t, uint32_t tile_bytes, Region* R, int64_t* volume) {
  const int n = t.ndim;
  if (s.ndim != n) return false;  // reported as a shape mismatch elsewhere
  // element sizes of the two sides: they differ only for a converting pair (checked when the pairs
  // were counted), which moves 4-byte source elements into 2-byte destination elements
  const int64_t e = s.itemsize, et = t.itemsize;
  const bool conv = e != et;
  // a converting tile writes half of what it reads: twice the source bytes per tile keep the traffic per
  // tile (and per queue pop, descriptor and barrier) near that of a plain copy
  if (conv) tile_bytes *= 2;
  if (R) {
    for (int k = 0; k < kDims; ++k) {
      R->len[k] = 1;
      R->spitch[k] = 0;
      R->dpitch[k] = 0;
    }
  }
  int m = 0;                        // merged dimensions already in R
  int64_t oL = 1, oS = 0, oD = 0;  // the merged dimension still open (length, element strides), if any
  bool open = false;
  int64_t soff = 0, doff = 0, vol = 1;
#pragma unroll
  for (int k = 0; k < kDims; ++k) {
    if (k >= n) break;
    const int64_t lo = s.off[k] > t.off[k] ? s.off[k] : t.off[k];
    const int64_t hs = s.off[k] + s.len[k], ht = t.off[k] + t.len[k];
    const int64_t hi = hs < ht ? hs : ht;
    if (lo >= hi) return false;
    const int64_t sk = s.stride[k], tk = t.stride[k];
    soff += (lo - s.off[k]) * sk;
    doff += (lo - t.off[k]) * tk;
    const int64_t len = hi - lo;
    vol *= len;
    if (len == 1) continue;  // unit dimensions carry no stride
    if (open && oS == len * sk && oD == len * tk) {
      oL *= len;  // contiguous with the previous dimension on both sides: merge
      oS = sk;
      oD = tk;
    } else {
      if (open) {
        if (R) {
          R->len[m] = oL;
          R->spitch[m] = oS;
          R->dpitch[m] = oD;
        }
        ++m;
      }
      oL = len;
      oS = sk;
      oD = tk;
      open = true;
    }
  }
  if (!R) return true;
  *volume = vol;
  R->src_base = s.byte_base + soff * e;
  R->dst_base = t.byte_base + doff * et;
  R->src_buf = s.buf;
  R->dst_buf = t.buf;
  R->srec = s.rec;
  R->trec = t.rec;
  R->tile_bytes = tile_bytes;
  R->rows_per_tile = 1;
  R->segs_per_row = 1;
  R->tdim_a = 0;
  R->tdim_b = 0;
  R->tiles_b = 0;
  R->lead_mod = 0;
  int nd = m;  // row dimensions
  int64_t run_bytes = e;
  if (open && oS == 1 && oD == 1) {
    run_bytes = oL * e;  // the innermost dimension is contiguous on both sides: it is the run
  } else if (open) {
    R->len[m] = oL;
    R->spitch[m] = oS;
    R->dpitch[m] = oD;
    nd = ++m;
    int a = -1, b = -1;
    for (int k = 0; k < m; ++k) {
      if (R->spitch[k] == 1) a = k;
      if (R->dpitch[k] == 1) b = k;
    }
    if (!conv && a >= 0 && b >= 0 && a != b && R->len[a] >= 4 && R->len[b] >= 4) {
      // source-contiguous and destination-contiguous dimensions differ: LDS-staged transpose; the other
      // dimensions keep their order, then come the source-contiguous and the destination-contiguous one
      R->kind = kTranspose;
      R->run_bytes = e;
      const int64_t La = R->len[a], Sa = R->spitch[a], Da = R->dpitch[a];
      const int64_t Lb = R->len[b], Sb = R->spitch[b], Db = R->dpitch[b];
      int rest = 0;
      uint64_t groups = 1;
      for (int k = 0; k < m; ++k) {
        if (k == a || k == b) continue;
        const int64_t L = R->len[k];
        groups *= (uint64_t)L;
        R->len[rest] = L;
        R->spitch[rest] = R->spitch[k] * e;
        R->dpitch[rest] = R->dpitch[k] * e;
        ++rest;
      }
      R->len[rest] = La;
      R->spitch[rest] = Sa * e;
      R->dpitch[rest] = Da * e;
      R->len[rest + 1] = Lb;
      R->spitch[rest + 1] = Sb * e;
      R->dpitch[rest + 1] = Db * e;
      R->ndim = m;
      const uint32_t tda = transpose_edge_a((uint32_t)e), tdb = transpose_edge_b((uint32_t)e);
      R->tdim_a = tda;
      R->tdim_b = tdb;
      // (the edges are powers of two)
      const uint64_t ta = ((uint64_t)La + tda - 1) >> (31 - __clz((int)tda)), tb = ((uint64_t)Lb + tdb - 1) >> (31 - __clz((int)tdb));
      R->tiles_b = (uint32_t)(tb < 0xffffffffull ? tb : 0xffffffffull);
      const uint64_t tpg = ta * tb;
      R->tiles_per_group = (uint32_t)(tpg < 0xffffffffull ? tpg : 0xffffffffull);
      R->n_tiles = (tpg >> 32 || groups >> 31) ? ~0ull : groups * tpg;
      return true;
    }
  }
  R->kind = conv ? kConvert : kRows;
  R->run_bytes = run_bytes;
  R->ndim = nd;
  uint64_t misal = (uint64_t)(t.byte_base + doff * et);
  uint64_t groups = 1, L0 = 1;
  for (int k = 0; k < nd; ++k) {
    groups *= L0;  // (all but the last row dimension)
    L0 = (uint64_t)R->len[k];
    R->spitch[k] *= e;
    const int64_t dp = R->dpitch[k] * et;
    R->dpitch[k] = dp;
    misal |= (uint64_t)dp;
  }
  uint64_t tpg;
  if ((uint64_t)run_bytes >= tile_bytes) {
    // Two workgroups writing parts of one cache line cost bandwidth, so segments of a long row are
    // cut where the destination offset is a multiple of kSegmentAlign (buffers themselves are
    // assumed at least that aligned).  Rows whose destination starts are aligned anyway need no
    // lead-in; otherwise the first segment of a row is shorter and one more segment (possibly
    // empty) is reserved per row.
    const uint32_t lead_mod = (misal % kSegmentAlign) ? kSegmentAlign : 0;
    R->lead_mod = lead_mod;
    // (the lead-in is counted in source bytes: e / et of them per destination byte)
    const uint64_t segs = ((uint64_t)run_bytes + (lead_mod ? kSegmentAlign * (uint64_t)(e / et) - 1 : 0) + tile_bytes - 1) >>
                          (31 - __clz((int)tile_bytes));  // (the tile budget is a power of two)
    R->segs_per_row = (uint32_t)(segs < 0xffffffffull ? segs : 0xffffffffull);
    tpg = (segs >> 32 || L0 >> 31) ? ~0ull : L0 * segs;
  } else {
    uint64_t rpt = tile_bytes / (uint32_t)run_bytes;  // (32-bit: the run is shorter than the budget here)
    if (rpt > L0) rpt = L0;
    R->rows_per_tile = (uint32_t)rpt;
    tpg = (L0 >> 32) ? (L0 + rpt - 1) / rpt : (uint64_t)(((uint32_t)L0 + (uint32_t)rpt - 1) / (uint32_t)rpt);
  }
  R->tiles_per_group = (uint32_t)(tpg < 0xffffffffull ? tpg : 0xffffffffull);
  R->n_tiles = (tpg >> 32 || groups >> 31) ? ~0ull : groups * tpg;
  return true;
}

// Index of the first element of the ascending array a[0..n) that is greater than v, found by a whole wave:
// every step probes 64 evenly spaced elements at once, so an array of a million entries takes four
// dependent loads where a binary search takes twenty.  All 64 lanes call it with the same arguments.
__device__ inline int64_t wave_upper_bound_u64(const uint64_t* a, int64_t n, uint64_t v) {
  int64_t lo = 0, hi = n;  // the answer lies in [lo, hi]
  while (hi - lo > 64) {
    const int64_t step = (hi - lo + 63) >> 6;
    const int64_t i = lo + (int64_t)(lane_id() + 1) * step - 1;  // last element of the lane's slice
    const bool le = i < hi && a[i] <= v;
    const int c = __popcll(__ballot(le));  // (ascending: the lanes that say yes are the first c)
    lo += (int64_t)c * step;
    const int64_t end = lo + step - 1;  // the slice's last element is known to be greater
    if (end < hi) hi = end;
  }
  const int64_t i = lo + (int64_t)lane_id();
  const bool le = i < hi && a[i] <= v;
  return lo + __popcll(__ballot(le));
}

// Items numbered through consecutive segments (start[0..n] is the running count of items, ascending, with
// start[0] == 0 and start[n] == n_items), one workgroup of kBlock threads per kBlock consecutive items:
// the segment that holds this thread's item p0 + threadIdx.x, and the number of the segment's first item.
// A search per thread through the whole of start[] is a chain of some twenty dependent loads and nothing
// else, so: the block's first and last item are looked up by one wave each (wave_upper_bound_u64); the
// items in between belong to the segments in between, whose starts come into LDS in one load and are searched
// there.  Every thread of the block must call it (it synchronises); threads without an item (p >= n_items)
// get segment -1.
struct BlockSegments {
  uint64_t start[kBlock + 1];
  int64_t range[2];
};
__device__ inline int64_t locate_in_block(const uint64_t* start, int64_t n, uint64_t n_items, BlockSegments& lds,
                                          uint64_t* seg_first) {
  const uint64_t p0 = (uint64_t)blockIdx.x * kBlock;
  const uint64_t p = p0 + threadIdx.x;
  if (p0 >= n_items) return -1;  // (a block past the last item: the same for all its threads)
  const unsigned w = threadIdx.x >> 6;
  if (w == 0 || w == kBlock / 64 - 1) {
    const uint64_t q = w == 0 ? p0 : (p0 + kBlock - 1 < n_items ? p0 + kBlock - 1 : n_items - 1);
    // segment whose range contains q: last t with start[t] <= q
    const int64_t t = wave_upper_bound_u64(start, n + 1, q) - 1;
    if (lane_id() == 0) lds.range[w ? 1 : 0] = t;
  }
  __syncthreads();
  const int64_t t0 = lds.range[0];
  const int64_t span = lds.range[1] - t0 + 1;  // segments of this block (empty ones included)
  const bool staged = span <= kBlock;
  if (staged) {
    for (int64_t i = threadIdx.x; i <= span; i += kBlock) lds.start[i] = start[t0 + i];
    __syncthreads();
  }
  if (p >= n_items) return -1;
  if (staged) {
    int lo = 0, hi = (int)span + 1;  // first index with lds.start[i] > p
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (lds.start[mid] <= p) lo = mid + 1; else hi = mid;
    }
    *seg_first = lds.start[lo - 1];
    return t0 + lo - 1;
  }
  const int64_t t = t0 + upper_bound_u64(start + t0, span, p) - 1;
  *seg_first = start[t];
  return t;
}

// Candidate pairs are numbered target box by target box (pair_start is the running count), the pairs of one
// target in the FQN-sorted order of the saved boxes.  Pass 1, one thread per candidate: find the pair's two
// boxes, test whether they intersect, and write the block's hits -- (saved box, target box) -- densely
// at the start of the block's own 256 slots of `hits`, with their number in blk_cnt.  The order inside a
// block (rank from wave ballots and a prefix over the block's waves) is the order of the pairs, so the
// region list that pass 2 writes from these lists is ordered by (target box, saved box) and reproducible.
__global__ __launch_bounds__(kBlock) void k_pairs_find(const Box* boxes, int64_t nbs, int64_t nbt, const uint32_t* sidx,
                                                       const uint32_t* grp_lo, const uint64_t* pair_start,
                                                       uint64_t n_pairs, uint32_t* blk_cnt, uint2* hits,
                                                       uint64_t* tile_cnt_zero, ull* ext_zero, uint64_t ext_words) {
  __shared__ uint32_t wcnt[kBlock / 64];
  __shared__ BlockSegments seg;
  const uint64_t p0 = (uint64_t)blockIdx.x * kBlock;
  // what pass 2 expects to find cleared: the tile counts of a list sized by the number of candidates (slots
  // beyond the region count stay zero, so that the scan of the counts may run over all of them) and the extent table
  if (tile_cnt_zero) {
    if (p0 + threadIdx.x < n_pairs) tile_cnt_zero[p0 + threadIdx.x] = 0;
    if (p0 + threadIdx.x == 0) tile_cnt_zero[n_pairs] = 0;
  }
  for (uint64_t i = p0 + threadIdx.x; i < ext_words; i += (uint64_t)gridDim.x * kBlock) ext_zero[i] = 0;
  const unsigned w = threadIdx.x >> 6;
  uint64_t first = 0;
  const int64_t t = locate_in_block(pair_start, nbt, n_pairs, seg, &first);
  bool hit = false;
  uint32_t s_box = 0;
  if (t >= 0) {
    s_box = sidx[grp_lo[t] + (p0 + threadIdx.x - first)];
    hit = build_region(boxes[s_box], boxes[nbs + t], 0, nullptr, nullptr);
  }
  const ull m = __ballot(hit);
  if (lane_id() == 0) wcnt[w] = (uint32_t)__popcll(m);
  __syncthreads();
  uint32_t rank = (uint32_t)__popcll(m & ((1ull << lane_id()) - 1ull));
  for (unsigned i = 0; i < w; ++i) rank += wcnt[i];
  if (hit) hits[p0 + rank] = make_uint2(s_box, (uint32_t)t);
  if (threadIdx.x == 0) {
    uint32_t s = 0;
    for (unsigned i = 0; i < kBlock / 64; ++i) s += wcnt[i];
    blk_cnt[blockIdx.x] = s;
  }
}

// plan statistics are summed per workgroup in LDS first: one global atomic per counter and
// workgroup instead of one per region
struct WaveStats {
  ull payload, src_bytes, converted, transposed, dims[kDims + 1], src_end, lds_transpose;
  long long max_src, max_dst;
};

// Pass 2, one wave per 32 hits of a pass-1 block (workgroup (b, q) takes hits q*32.. of block b; most blocks find
// fewer than 128, so the later workgroups of a block leave at once): build the copy regions and write them at
// blk_off[b] + rank.  The regions of a workgroup are put together in LDS and leave as one contiguous,
// coalesced copy (a 280-byte struct stored by each thread on its own is 18 partial-line stores per region).
// Only half of the wave's lanes build: the kernel waits for its scattered loads and stores, the two boxes
// of a hit take 116 registers and 32 regions 9 KB of LDS, so 16 waves fit a CU this way -- with 64 hits per
// wave it is 8, and the kernel takes a quarter longer.  Waves share nothing, so no wave waits for another one's loads.
constexpr uint32_t kBuildWave = 64;
constexpr uint32_t kBuildHits = 32;  // hits of a workgroup

__global__ __launch_bounds__(kBuildWave) void k_pairs_build(const Box* boxes, int64_t nbs, const uint2* hits,
                                                            const uint32_t* blk_off, uint32_t tile_bytes, Region* regions,
                                                            uint64_t* tile_cnt, ull* cov, Ctl* ctl, ull* ext,
                                                            uint32_t ext_src_bufs, uint32_t ext_bufs, uint32_t ext_stripes) {
  __shared__ WaveStats ws;
  __shared__ __attribute__((aligned(16))) char stage[kBuildHits * sizeof(Region)];
  // (first every block's first 32 hits, then every block's second 32, ...: workgroups go to the chip's
  // eight dies in turn, and with the four waves of a block next to each other some dies would only ever see
  // the later waves, which mostly have nothing to do)
  const uint32_t n_find_blocks = gridDim.x / (kBlock / kBuildHits);
  const uint32_t b = blockIdx.x % n_find_blocks, q = blockIdx.x / n_find_blocks;
  const uint32_t first = blk_off[b], cnt = blk_off[b + 1] - first;
  if (q * kBuildHits >= cnt) return;
  const uint32_t mine = min(kBuildHits, cnt - q * kBuildHits);
  if (threadIdx.x == 0) {
    ws.payload = ws.src_bytes = ws.converted = ws.transposed = 0;
    for (int k = 0; k <= kDims; ++k) ws.dims[k] = 0;
    ws.max_src = ws.max_dst = -1;
    ws.src_end = 0;
    ws.lds_transpose = 0;
  }
  __syncthreads();
  const bool active = threadIdx.x < mine;
  ull send = 0, dend = 0, vol_u = 0;
  int src_buf = -1, dst_buf = -1;
  int64_t trec = -1;
  if (active) {
    const uint2 h = hits[(uint64_t)b * kBlock + q * kBuildHits + threadIdx.x];
    // (both boxes whole, in registers, before anything looks at them: their loads are in flight together
    // instead of one dimension's after the other's)
    const Box sbox = boxes[h.x], tbox = boxes[nbs + h.y];
    const Box *sb = &sbox, *tb = &tbox;
    const uint32_t pos = first + q * kBuildHits + threadIdx.x;
    Region& R = reinterpret_cast<Region*>(stage)[threadIdx.x];
    int64_t vol = 0;
    build_region(sbox, tbox, tile_bytes, &R, &vol);
    tile_cnt[pos] = R.n_tiles;
    vol_u = (ull)vol;
    trec = tb->rec;
    atomicAdd(&ws.payload, (ull)vol * (ull)tb->itemsize);
    atomicAdd(&ws.src_bytes, (ull)vol * (ull)sb->itemsize);
    if (R.kind == kConvert) atomicAdd(&ws.converted, 1ull);
    atomicAdd(&ws.dims[R.ndim + (R.kind != kTranspose && R.run_bytes > sb->itemsize ? 1 : 0)], 1ull);
    if (R.kind == kTranspose) {
      atomicAdd(&ws.transposed, 1ull);
      atomicMax(&ws.lds_transpose, (ull)transpose_lds_bytes(R.tdim_a, R.tdim_b, (uint32_t)R.run_bytes));
    }
    send = (ull)(R.src_base + R.run_bytes);
    dend = (ull)(R.dst_base + (R.kind == kConvert ? R.run_bytes / 2 : R.run_bytes));
    for (int k = 0; k < R.ndim; ++k) {
      send += (ull)((R.len[k] - 1) * R.spitch[k]);
      dend += (ull)((R.len[k] - 1) * R.dpitch[k]);
    }
    src_buf = R.src_buf;
    dst_buf = R.dst_buf;
    atomicMax(&ws.src_end, send);
    atomicMax(&ws.max_src, (long long)R.src_buf);
    atomicMax(&ws.max_dst, (long long)R.dst_buf);
    if (R.n_tiles == ~0ull) report(ctl, 0, kErrInvalid);
  }
  // What the wave adds to memory other waves add to as well leaves it once per distinct address, not once per
  // lane: an atomic costs the L2 the same few nanoseconds whether or not a neighbour lane's could have been
  // folded into it, and millions of regions share a few hundred buffers and half as many target records.
  //
  // Elements of each target record covered by saved data (Sec. 3.3 Step 2: every requested element must
  // be found).  The hits of a wave are in target-box order, so those of one record are neighbours:
  // runs of equal records are summed by a segmented scan and their last lane adds the sum.
  {
    const int64_t prev = __shfl_up(trec, 1);
    const bool head = lane_id() == 0 || prev != trec;
    const ull heads = __ballot(head);
    const int run = __popcll(heads & (~0ull >> (63 - lane_id())));  // runs that start at or below this lane
    ull v = vol_u;
    for (int o = 1; o < 64; o <<= 1) {
      const ull u = __shfl_up(v, o);
      const int r = __shfl_up(run, o);
      if (lane_id() >= o && r == run) v += u;
    }
    const bool tail = lane_id() == 63 || ((heads >> (lane_id() + 1)) & 1ull);
    if (active && tail) atomicAdd(&cov[trec], v);
  }
  // Per buffer, one past the highest byte the plan touches.  The table is kept in several copies (one per
  // group of workgroups, folded afterwards), and most regions lie below what an earlier one has recorded (the
  // values only grow, so a stale read costs an atomic, never a wrong maximum).  Of the lanes that still
  // have something to record, those that name the same buffer as the first of them reduce their maxima
  // among themselves and one of them updates the table (the regions of one target rank's buffer, or read
  // from one blob, are neighbours); after two such rounds whoever is left updates it on its own.
  {
    ull* e = ext + (size_t)(b % ext_stripes) * ext_bufs;
    for (int side = 0; side < 2; ++side) {
      const int buf = side ? dst_buf : src_buf;
      const ull end = side ? dend : send;
      ull* slot = &e[(side ? ext_src_bufs : 0u) + (uint32_t)(active ? buf : 0)];
      bool todo = active && *slot < end;
      for (int round = 0; round < 2; ++round) {
        const ull waiting = __ballot(todo);
        if (!waiting) break;
        const int leader = __ffsll((long long)waiting) - 1;
        const int which = __shfl(buf, leader);
        const bool same = todo && buf == which;
        ull m = same ? end : 0;
        for (int o = 32; o >= 1; o >>= 1) {
          const ull other = __shfl_xor(m, o);
          m = other > m ? other : m;
        }
        if (lane_id() == leader) atomicMax(slot, m);
        todo = todo && !same;
      }
      if (todo) atomicMax(slot, end);
    }
  }
  __syncthreads();
  static_assert(sizeof(Region) % 8 == 0, "copied in 8-byte words");
  const uint32_t words = mine * (uint32_t)(sizeof(Region) / 8);
  const uint64_t* from = reinterpret_cast<const uint64_t*>(stage);
  uint64_t* to = reinterpret_cast<uint64_t*>(regions + first + q * kBuildHits);
  for (uint32_t i = threadIdx.x; i < words; i += kBuildWave) to[i] = from[i];
  if (threadIdx.x == 0) {
    Ctl* part = &(reinterpret_cast<CtlStripe*>(ctl) + 1 + b % kCtlStripes)->c;
    atomicAdd(&part->payload_bytes, ws.payload);
    atomicAdd(&part->src_bytes, ws.src_bytes);
    if (ws.converted) atomicAdd(&part->n_convert, ws.converted);
    if (ws.transposed) {
      atomicAdd(&part->n_transposed, ws.transposed);
      atomicMax(&part->lds_transpose, ws.lds_transpose);
    }
    for (int k = 0; k <= kDims; ++k)
      if (ws.dims[k]) atomicAdd(&part->dims_hist[k], ws.dims[k]);
    atomicMax(&part->max_src_end, ws.src_end);
    atomicMax(&part->max_src_buf, ws.max_src);
    atomicMax(&part->max_dst_buf, ws.max_dst);
  }
}

__global__ __launch_bounds__(kBlock) void k_coverage(const bcp_shard_meta* recs, int64_t n_saved, int64_t n_target,
                                                     const ull* cov, int allow_uncovered, Ctl* ctl) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= n_target) return;
  const bcp_shard_meta& r = recs[n_saved + i];
  const ull want = (ull)(r.flat_end - r.flat_begin);
  if (cov[i] > want) report(ctl, n_saved + i, kErrOverlap);
  else if (cov[i] < want && !allow_uncovered) report(ctl, n_saved + i, kErrUncovered);
}

// ---- step 5: tiles and batches -------------------------------------------------------------------
// Decode tile `local` of region R completely -- leading row indices, row / segment range, byte
// offsets -- so the copy kernel does no index arithmetic beyond its own lanes.  Returns the
// tile's payload bytes.
__device__ inline uint64_t decode_tile(const Region& R, uint32_t local, TileDesc* out) {
  TileDesc t;
  t.src_buf = (uint32_t)R.src_buf;
  t.dst_buf = (uint32_t)R.dst_buf;
  t.kind = (uint32_t)R.kind;
  t.first = 0;
  t.count = 1;
  t.pad_ = 0;
  uint64_t bytes;
  int64_t so = R.src_base, dof = R.dst_base;
  const int nd = R.ndim;
  const uint32_t tpg = R.tiles_per_group;
  uint64_t group = local / tpg;
  const uint32_t w = local - (uint32_t)group * tpg;
  if (R.kind == kTranspose) {
    for (int k = nd - 3; k >= 0; --k) {
      const uint64_t L = (uint64_t)R.len[k];
      uint64_t c;
      if ((group | L) >> 32) {
        c = group % L;
        group /= L;
      } else {  // 32-bit division is several times cheaper, and this is the common case
        const uint32_t q = (uint32_t)group / (uint32_t)L;
        c = (uint32_t)group - q * (uint32_t)L;
        group = q;
      }
      so += (int64_t)c * R.spitch[k];
      dof += (int64_t)c * R.dpitch[k];
    }
    const uint32_t tda = R.tdim_a, tdb = R.tdim_b;
    const uint32_t ta = w / R.tiles_b, tb = w - ta * R.tiles_b;
    const uint64_t a0 = (uint64_t)ta * tda, b0 = (uint64_t)tb * tdb;
    const uint64_t ra = (uint64_t)R.len[nd - 2] - a0, rb = (uint64_t)R.len[nd - 1] - b0;
    t.a = (uint32_t)(ra < tda ? ra : tda);
    t.b = (uint32_t)(rb < tdb ? rb : tdb);
    t.p0 = R.spitch[nd - 1];
    t.p1 = R.dpitch[nd - 2];
    t.kind |= ((uint32_t)R.run_bytes << 8) | ((uint32_t)(31 - __clz((int)tda)) << 16) |
              ((uint32_t)(31 - __clz((int)tdb)) << 24);
    bytes = (uint64_t)t.a * t.b * (uint64_t)R.run_bytes;
    so += (int64_t)a0 * R.spitch[nd - 2] + (int64_t)b0 * R.spitch[nd - 1];
    dof += (int64_t)a0 * R.dpitch[nd - 2] + (int64_t)b0 * R.dpitch[nd - 1];
  } else {
    for (int k = nd - 2; k >= 0; --k) {
      const uint64_t L = (uint64_t)R.len[k];
      uint64_t c;
      if ((group | L) >> 32) {
        c = group % L;
        group /= L;
      } else {
        const uint32_t q = (uint32_t)group / (uint32_t)L;
        c = (uint32_t)group - q * (uint32_t)L;
        group = q;
      }
      so += (int64_t)c * R.spitch[k];
      dof += (int64_t)c * R.dpitch[k];
    }
    const int64_t sp = nd >= 1 ? R.spitch[nd - 1] : 0, dp = nd >= 1 ? R.dpitch[nd - 1] : 0;
    t.p0 = sp;
    t.p1 = dp;
    if ((uint64_t)R.run_bytes >= R.tile_bytes) {  // a segment of one long row
      const uint32_t row = w / R.segs_per_row, seg = w - row * R.segs_per_row;
      so += (int64_t)row * sp;
      dof += (int64_t)row * dp;
      // segments are counted in source bytes; a converting region writes half as many
      const int64_t ratio = R.kind == kConvert ? 2 : 1;
      int64_t lead = R.lead_mod ? dof & (int64_t)(R.lead_mod - 1) : 0;  // (a power of two)
      if (ratio > 1) lead &= ~(int64_t)1;  // whole destination elements
      int64_t begin = (int64_t)seg * R.tile_bytes - lead * ratio, end = begin + (int64_t)R.tile_bytes;
      if (begin < 0) begin = 0;
      if (end > R.run_bytes) end = R.run_bytes;
      if (begin > end) begin = end;  // the spare segment of a row that did not need it: empty, at the row's end
      so += begin;
      dof += begin / ratio;
      t.a = (uint32_t)((end - begin) / (R.kind == kConvert ? 4 : 1));
      t.b = 1;
    } else {  // a few whole short rows
      const uint64_t L0 = nd >= 1 ? (uint64_t)R.len[nd - 1] : 1;
      const uint64_t row0 = (uint64_t)w * R.rows_per_tile;
      const uint64_t left = L0 - row0;
      t.b = (uint32_t)(left < R.rows_per_tile ? left : R.rows_per_tile);
      t.a = (uint32_t)(R.run_bytes / (R.kind == kConvert ? 4 : 1));
      so += (int64_t)row0 * sp;
      dof += (int64_t)row0 * dp;
    }
    bytes = (uint64_t)t.a * t.b * (R.kind == kConvert ? 4u : 1u);  // source bytes
  }
  t.src_off = so;
  t.dst_off = dof;
  if (out) *out = t;
  return bytes;
}

// Pass A, one thread per tile: its region (located in the scanned tile counts) and what it
// counts towards a batch budget: 0 for big tiles, which are batches of their own.
// key (optional): source-order sort key, (source buffer, last source byte the tile reads).
__global__ __launch_bounds__(kBlock) void k_tile_weights(const uint64_t* tile_start, const Region* regions,
                                                         int64_t n_regions, uint64_t n_tiles, uint32_t* tile_region,
                                                         uint32_t* tile_local, uint64_t* weight, uint64_t* key,
                                                         uint32_t* order, unsigned long long* queue) {
  __shared__ BlockSegments seg;
  const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < 8) queue[i] = 0;  // the copy kernel's queue words start at zero (and put themselves back there)
  uint64_t first = 0;
  const int64_t r = locate_in_block(tile_start, n_regions, n_tiles, seg, &first);
  if (r < 0) return;
  tile_region[i] = (uint32_t)r;
  tile_local[i] = (uint32_t)(i - first);
  TileDesc t;
  const uint64_t bytes = decode_tile(regions[r], (uint32_t)(i - first), &t);
  weight[i] = bytes >= kSmallTileBytes ? 0 : (bytes > kMinBatchWeight ? bytes : (uint64_t)kMinBatchWeight);
  // a transpose tile of any useful size wants the whole workgroup and its LDS staging
  if ((t.kind & 0xffu) == kTranspose && bytes >= 1024) weight[i] = 0;
  if (key) {
    uint64_t last = (uint64_t)t.src_off;
    if ((t.kind & 0xffu) == kTranspose) {
      const uint64_t e = (t.kind >> 8) & 0xffu;
      last += (uint64_t)(t.a ? t.a - 1 : 0) * e + (uint64_t)(t.b ? t.b - 1 : 0) * (uint64_t)t.p0 + (e ? e - 1 : 0);
    } else if (bytes) {
      last += (uint64_t)(t.b - 1) * (uint64_t)t.p0 + (uint64_t)t.a * ((t.kind & 0xffu) == kConvert ? 4u : 1u) - 1;
    } else if (last) {
      --last;  // an empty tile (the spare segment of a long row) sits one past its row's last byte: it is keyed
               // to that byte, so that its batch's key never points beyond the bytes the plan reads
    }
    key[i] = ((uint64_t)t.src_buf << kKeyShift) | last;
    order[i] = (uint32_t)i;
  }
}

// source-ordered plans: bring the per-tile arrays into sorted order
__global__ __launch_bounds__(kBlock) void k_gather_tiles(const uint32_t* order, uint64_t n_tiles,
                                                         const uint32_t* region_in, const uint32_t* local_in,
                                                         const uint64_t* weight_in, uint32_t* region_out,
                                                         uint32_t* local_out, uint64_t* weight_out) {
  const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= n_tiles) return;
  const uint32_t o = order[i];
  region_out[i] = region_in[o];
  local_out[i] = local_in[o];
  weight_out[i] = weight_in[o];
}

// Batches.  A big tile (weight 0) is a batch of its own.  The small tiles form batches among themselves,
// in tile order but across the big tiles that stand between them (a long run's last few KiB, a bias between
// two matrices: alone in a batch each would cost a workgroup more than a full tile does): with wprefix the
// exclusive scan of the weights -- which the big tiles do not move -- a small tile belongs to the budget
// window its END falls into, (wprefix + weight - 1) / budget, and opens a batch when the small tile before
// it, which ends at wprefix, belongs to an earlier one.  Ends are at least kMinBatchWeight apart, so a batch
// has at most budget / kMinBatchWeight tiles, and less than budget + kSmallTileBytes of weight.
// key (optional, sorted; plans ordered by source): batches stay runs of consecutive tiles and never span
// two source buffers, so a small tile after a big one or in another buffer opens a batch as well.
// flags[i]: low word 1 for a small tile, high word 1 when it opens a batch; scanned, the words are the
// tile's index among the small tiles and its batch's index among the small-tile batches.
__global__ __launch_bounds__(kBlock) void k_batch_flags(const uint64_t* weight, const uint64_t* wprefix,
                                                        uint64_t n_tiles, uint32_t budget, const uint64_t* key,
                                                        uint64_t* flags) {
  const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= n_tiles) return;
  const uint64_t w = weight[i], before = wprefix[i];
  if (w == 0) {
    flags[i] = 0;
    return;
  }
  bool opens = before == 0 || (before + w - 1) / budget != (before - 1) / budget;
  if (key && i > 0 && (weight[i - 1] == 0 || (key[i] >> kKeyShift) != (key[i - 1] >> kKeyShift))) opens = true;
  flags[i] = opens ? (1ull << 32) | 1ull : 1ull;
}

// What the scanned flags say about tile i (scan[i], and scan[i + 1] for what the tile itself adds).
struct TileRank {
  uint32_t small_rank;   // small tiles before it
  uint32_t small_batch;  // small-tile batches opened before it
  bool small, opens;     // opens: a batch starts here (every big tile; a small one as flagged)
  __device__ uint32_t big_rank(uint64_t i) const { return (uint32_t)(i - small_rank); }
};
__device__ __forceinline__ TileRank tile_rank(const uint64_t* scan, uint64_t i) {
  const uint64_t a = scan[i], b = scan[i + 1];
  TileRank r;
  r.small_rank = (uint32_t)a;
  r.small_batch = (uint32_t)(a >> 32);
  r.small = (uint32_t)b != (uint32_t)a;
  r.opens = !r.small || (b >> 32) != (a >> 32);
  return r;
}

// bstart[k]: index among the small tiles of small-tile batch k's first tile, with a sentinel after the last batch.
__global__ __launch_bounds__(kBlock) void k_batch_starts(const uint64_t* scan, uint64_t n_tiles, uint32_t* bstart) {
  const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i > n_tiles) return;
  if (i == n_tiles) {
    bstart[(uint32_t)(scan[n_tiles] >> 32)] = (uint32_t)scan[n_tiles];
    return;
  }
  const TileRank r = tile_rank(scan, i);
  if (r.small && r.opens) bstart[r.small_batch] = r.small_rank;
}

// Where a batch goes in the queue.  Plans in plan order spread their small-tile batches evenly among the
// big tiles: a workgroup on a small-tile batch waits on memory latency most of the time, and the workgroups
// streaming big tiles beside it keep the memory busy meanwhile, which a stretch of the queue made of small-tile
// batches alone cannot.  With n batches, S of them small: the k-th small one takes the slot where
// floor(slot * S / n) steps to k + 1, the j-th big one slot floor(j * n / (n - S)); together a permutation.
__device__ __forceinline__ uint32_t small_batch_slot(uint32_t k, uint64_t n, uint64_t S) {
  return (uint32_t)((((uint64_t)k + 1) * n + S - 1) / S - 1);
}
__device__ __forceinline__ uint32_t big_tile_slot(uint32_t j, uint64_t n, uint64_t S) {
  return (uint32_t)(((uint64_t)j * n) / (n - S));
}

// Pass B, one thread per tile: the decoded descriptor goes to heads[slot of its batch] when the tile opens a
// batch and, when it is small, to tiles[its index among the small tiles] (members of multi-tile batches are
// fetched from there).
// key / batch_key (optional, source-ordered plans): batches keep tile order, slot = big tiles before it +
// small-tile batches before it; batch_key[slot] = key of the batch's last tile, the largest in the batch.
__global__ __launch_bounds__(kBlock) void k_fill_tiles(const Region* regions, const uint32_t* tile_region,
                                                       const uint32_t* tile_local, const uint64_t* scan,
                                                       const uint32_t* bstart, uint64_t n_tiles, TileDesc* tiles,
                                                       TileDesc* heads, const uint64_t* key, uint64_t* batch_key) {
  const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= n_tiles) return;
  const TileRank r = tile_rank(scan, i);
  if (key && (i + 1 == n_tiles || tile_rank(scan, i + 1).opens)) {
    // tile i closes its batch (the next tile opens one, or there is none)
    batch_key[r.big_rank(i) + r.small_batch + (r.small && r.opens ? 1u : 0u) - (r.small ? 1u : 0u)] = key[i];
  }
  TileDesc t;
  decode_tile(regions[tile_region[i]], tile_local[i], &t);
  t.first = r.small_rank;
  if (r.small) tiles[r.small_rank] = t;
  if (r.opens) {
    const uint64_t total = scan[n_tiles];
    const uint64_t S = total >> 32, n = n_tiles - (uint32_t)total + S;
    t.count = r.small ? bstart[r.small_batch + 1] - bstart[r.small_batch] : 1u;
    uint32_t slot;
    if (key || S == 0 || S == n) slot = r.big_rank(i) + r.small_batch;
    else slot = r.small ? small_batch_slot(r.small_batch, n, S) : big_tile_slot(r.big_rank(i), n, S);
    heads[slot] = t;
  }
}

// fold the copies of the per-buffer extent table: ext[b] = max over the stripes (at most 64 of them: one wave per
// buffer, one lane per stripe, so the copies are read side by side and not one after the other)
__global__ __launch_bounds__(kBlock) void k_extents_fold(ull* ext, uint32_t n_bufs, uint32_t stripes) {
  const uint32_t b = blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
  if (b >= n_bufs) return;  // (the same for all lanes of a wave)
  ull m = lane_id() < stripes ? ext[(size_t)lane_id() * n_bufs + b] : 0;
  for (int o = 32; o >= 1; o >>= 1) {
    const ull other = __shfl_xor(m, o);
    m = other > m ? other : m;
  }
  if (lane_id() == 0) ext[b] = m;
}

bcp_status device_error(const Ctl& ctl, int64_t n_saved) {
  if (ctl.err_key == ~0ull) return BCP_OK;
  const unsigned code = (unsigned)(ctl.err_key & 0xff);
  const int64_t rec = (int64_t)(ctl.err_key >> 8);
  const bool is_saved = rec < n_saved;
  return record_error(code, is_saved, is_saved ? rec : rec - n_saved);
}

// device memory a plan keeps; freed here on any early return
struct Owned {  // plan blocks until the plan takes them over
  void* p[2] = {nullptr, nullptr};
  size_t bytes[2] = {0, 0};
  hipStream_t st = nullptr;
  ~Owned() {
    for (int i = 0; i < 2; ++i)
      if (p[i]) block_free(p[i], bytes[i], true, st);
  }
};

struct BlockPool {
  struct Entry {
    void* p;
    size_t bytes;
    int device;
    hipEvent_t after;  // null: free to use at once
  };
  static constexpr size_t kMaxEntries = 8;
  static constexpr size_t kMaxBytes = (size_t)1 << 30;
  std::vector<Entry> kept;
  size_t kept_bytes = 0;
  std::mutex mu;
};
BlockPool g_pool;

}  // namespace

hipError_t block_alloc(void** p, size_t bytes, size_t* got, hipStream_t st) {
  bytes = std::max<size_t>(bytes, 256);
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  {
    std::lock_guard<std::mutex> lock(g_pool.mu);
    int best = -1;
    for (size_t i = 0; i < g_pool.kept.size(); ++i) {
      const BlockPool::Entry& c = g_pool.kept[i];
      if (c.device != dev || c.bytes < bytes || c.bytes > 2 * bytes + ((size_t)1 << 20)) continue;
      if (best < 0 || c.bytes < g_pool.kept[best].bytes) best = (int)i;
    }
    if (best >= 0) {
      const BlockPool::Entry c = g_pool.kept[best];
      g_pool.kept.erase(g_pool.kept.begin() + best);
      g_pool.kept_bytes -= c.bytes;
      if (c.after) {
        e = hipStreamWaitEvent(st, c.after, 0);
        (void)hipEventDestroy(c.after);  // released once the wait has gone through
        if (e != hipSuccess) {
          (void)hipFree(c.p);
          return e;
        }
      }
      *p = c.p;
      *got = c.bytes;
      return hipSuccess;
    }
  }
  *got = bytes;
  return hipMalloc(p, bytes);
}

void block_free(void* p, size_t bytes, bool used, hipStream_t last_use) {
  if (!p) return;
  int dev = 0;
  bool keep = hipGetDevice(&dev) == hipSuccess;
  hipEvent_t ev = nullptr;
  if (keep && used) {
    keep = hipEventCreateWithFlags(&ev, hipEventDisableTiming) == hipSuccess;
    if (keep && hipEventRecord(ev, last_use) != hipSuccess) {
      (void)hipEventDestroy(ev);
      keep = false;
    }
  }
  if (keep) {
    std::lock_guard<std::mutex> lock(g_pool.mu);
    if (g_pool.kept.size() < BlockPool::kMaxEntries && g_pool.kept_bytes + bytes <= BlockPool::kMaxBytes) {
      g_pool.kept.push_back(BlockPool::Entry{p, bytes, dev, ev});
      g_pool.kept_bytes += bytes;
      return;
    }
  }
  if (ev) (void)hipEventDestroy(ev);
  (void)hipFree(p);  // waits for the device, so a block still in use is safe here too
}

int64_t block_pool_release() {
  std::lock_guard<std::mutex> lock(g_pool.mu);
  const int64_t total = (int64_t)g_pool.kept_bytes;
  for (BlockPool::Entry& c : g_pool.kept) {
    if (c.after) (void)hipEventDestroy(c.after);
    (void)hipFree(c.p);
  }
  g_pool.kept.clear();
  g_pool.kept_bytes = 0;
  return total;
}

namespace {

// What the host needs between two phases -- the control block and up to three totals that sit at
// the end of scanned arrays -- gathered into one struct, so that it comes back with a single copy
// into pinned memory instead of one staged copy per value.
struct Readback {
  Ctl ctl;
  uint64_t v[3];
};
constexpr size_t kLandingBytes = 4096;  // at least; grows when a plan has many buffers (their extents land here)
constexpr size_t kLandingExtents = 64;  // offset of the per-buffer extents in the final read-back
static_assert(sizeof(Readback) <= kLandingBytes, "landing buffer");

// grow-only; the caller has made sure no copy into the old block is in flight
hipError_t ensure_landing(Workspace& ws, size_t bytes) {
  bytes = std::max(bytes, kLandingBytes);
  if (ws.landing && ws.landing_bytes >= bytes) return hipSuccess;
  if (ws.landing) (void)hipHostFree(ws.landing);
  ws.landing = nullptr;
  ws.landing_dev = nullptr;
  ws.landing_bytes = 0;
  hipError_t e = hipHostMalloc(&ws.landing, bytes, hipHostMallocDefault);
  if (e != hipSuccess) return e;
  e = hipHostGetDevicePointer(&ws.landing_dev, ws.landing, 0);
  if (e != hipSuccess) {
    (void)hipHostFree(ws.landing);
    ws.landing = nullptr;
    return e;
  }
  ws.landing_bytes = bytes;
  return hipSuccess;
}

// how the words of a Ctl combine
enum CtlOp : int { kOpAdd, kOpMaxU, kOpMaxS, kOpMinU };
__device__ inline int ctl_word_op(size_t word) {
  const size_t off = word * 8;
  if (off == offsetof(Ctl, err_key)) return kOpMinU;
  if (off == offsetof(Ctl, max_saved_fqn) || off == offsetof(Ctl, max_src_end) || off == offsetof(Ctl, lds_transpose)) return kOpMaxU;
  if (off == offsetof(Ctl, max_src_buf) || off == offsetof(Ctl, max_dst_buf) || off == offsetof(Ctl, max_saved_rec_buf) ||
      off == offsetof(Ctl, max_target_rec_buf))
    return kOpMaxS;
  return kOpAdd;
}
static_assert(sizeof(Ctl) % 8 == 0, "a Ctl is folded as 8-byte words");
constexpr int kCtlWords = (int)(sizeof(Ctl) / 8);

// One workgroup of kCtlStripes threads: folds the striped copies of the control block into the first one,
// leaves them as they were initialised (`neutral`), and copies the result and up to three values for the host.
__global__ __launch_bounds__(kCtlStripes) void k_readback(Ctl* ctl, Ctl neutral, const void* p0, int w0, const void* p1,
                                                          int w1, const void* p2, int w2, Readback* out) {
  __shared__ ull acc[kCtlWords];
  ull* main_words = reinterpret_cast<ull*>(ctl);
  if (threadIdx.x < kCtlWords) acc[threadIdx.x] = main_words[threadIdx.x];
  __syncthreads();
  ull* mine = reinterpret_cast<ull*>(&(reinterpret_cast<CtlStripe*>(ctl) + 1 + threadIdx.x)->c);
  const ull* none = reinterpret_cast<const ull*>(&neutral);
  ull words[kCtlWords];  // (all loads first: they are in flight together)
#pragma unroll
  for (int k = 0; k < kCtlWords; ++k) words[k] = mine[k];
#pragma unroll
  for (int k = 0; k < kCtlWords; ++k) {
    const ull v = words[k];
    if (v == none[k]) continue;
    mine[k] = none[k];
    switch (ctl_word_op(k)) {
      case kOpAdd: atomicAdd(&acc[k], v); break;
      case kOpMaxU: atomicMax(&acc[k], v); break;
      case kOpMaxS: atomicMax(reinterpret_cast<long long*>(&acc[k]), (long long)v); break;
      default: atomicMin(&acc[k], v); break;
    }
  }
  __syncthreads();
  if (threadIdx.x < kCtlWords) {
    main_words[threadIdx.x] = acc[threadIdx.x];
    reinterpret_cast<ull*>(&out->ctl)[threadIdx.x] = acc[threadIdx.x];
  }
  if (threadIdx.x != 0) return;
  const void* p[3] = {p0, p1, p2};
  const int w[3] = {w0, w1, w2};
  for (int i = 0; i < 3; ++i)
    out->v[i] = !p[i] ? 0 : (w[i] == 8 ? *(const uint64_t*)p[i] : (uint64_t) * (const uint32_t*)p[i]);
}

// Host memory the device can read in place (pinned: hipHostMalloc): its address on the device.
constexpr int64_t kDirectUploadRecords = 8192;  // more than these go by the copy engine, which moves large blocks faster
bool device_visible(const void* host, const void** dev) {
  void* d = nullptr;
  if (hipHostGetDevicePointer(&d, const_cast<void*>(host), 0) != hipSuccess || !d) {
    (void)hipGetLastError();  // pageable memory is unknown to the runtime: not an error of this call
    return false;
  }
  *dev = d;
  return true;
}

Ctl initial_ctl() {
  Ctl init{};
  init.err_key = ~0ull;
  init.max_src_buf = init.max_dst_buf = -1;
  init.max_saved_rec_buf = init.max_target_rec_buf = -1;
  return init;
}

// Synchronises the stream.  pK: device address of a 4-byte (wK == 4) or 8-byte value, or null.  The kernel writes
// what the host wants straight into the pinned landing block (a copy of its own would be one more operation
// on the stream, and a plan for a few thousand records is made of those).
bcp_status read_back(Workspace& ws, hipStream_t st, Ctl* ctl, Readback* host, const void* p0 = nullptr, int w0 = 4,
                     const void* p1 = nullptr, int w1 = 4, const void* p2 = nullptr, int w2 = 4) {
  hipLaunchKernelGGL(k_readback, dim3(1), dim3(kCtlStripes), 0, st, ctl, initial_ctl(), p0, w0, p1, w1, p2, w2,
                     (Readback*)ws.landing_dev);
  BCP_HIP(hipGetLastError());
  BCP_HIP(hipStreamSynchronize(st));
  std::memcpy(host, ws.landing, sizeof(Readback));
  return BCP_OK;
}

// the last read-back of a plan: the batch count and, per buffer the plan uses, one past the highest byte it touches
// (scan_total: the scanned batch flags' last entry, small tiles below, small-tile batches above)
__global__ __launch_bounds__(kBlock) void k_final_readback(const uint64_t* scan_total, uint64_t n_tiles, const ull* src_ext,
                                                           uint32_t n_src, const ull* dst_ext, uint32_t n_dst, char* landing) {
  if (threadIdx.x == 0)
    *reinterpret_cast<uint32_t*>(landing) = (uint32_t)(n_tiles - (uint32_t)*scan_total + (*scan_total >> 32));
  ull* out = reinterpret_cast<ull*>(landing + kLandingExtents);
  for (uint32_t i = threadIdx.x; i < n_src; i += kBlock) out[i] = src_ext[i];
  for (uint32_t i = threadIdx.x; i < n_dst; i += kBlock) out[n_src + i] = dst_ext[i];
}

}  // namespace

bcp_status run_planner(const bcp_shard_meta* saved, int64_t n_saved, const bcp_shard_meta* target,
                       int64_t n_target, uint32_t flags, hipStream_t st, PlannerResult* out) {
  const int64_t n_total = n_saved + n_target;
  const uint32_t tile_bytes = (uint32_t)config().tile_bytes;
  out->dev = PlanDevice{};
  out->n_saved_boxes = out->n_target_boxes = 0;
  out->device_ms = 0.f;

  const Ctl init = initial_ctl();
  out->ctl = init;
  if (n_target == 0) return BCP_OK;
  if (n_total > (int64_t)(0xffffffffu / kMaxBoxesPerRecord)) {  // box indices are 32-bit
    set_error("too many records");
    return BCP_ERR_INVALID_ARG;
  }
  out->src_extent.clear();
  out->dst_extent.clear();
  int dev = 0;
  BCP_HIP(hipGetDevice(&dev));
  std::lock_guard<std::mutex> ws_lock(g_ws.mu);
  Workspace& ws = g_ws;
  ws.reset(dev);
  Owned owned;
  owned.st = st;

  for (hipEvent_t& e : ws.ev)
    if (!e) BCP_HIP(hipEventCreate(&e));
  const hipEvent_t ev0 = ws.ev[0], ev1 = ws.ev[1];

  BCP_HIP(ensure_landing(ws, kLandingBytes));
  bcp_shard_meta* recs = nullptr;
  Ctl* ctl = nullptr;
  Readback rb;
  uint32_t* box_start = nullptr;
  BCP_HIP(ws.alloc(&recs, (size_t)n_total));
  {
    CtlStripe* copies = nullptr;  // the control block and its striped copies
    BCP_HIP(ws.alloc(&copies, (size_t)kCtlStripes + 1));
    ctl = &copies->c;
  }
  BCP_HIP(ws.alloc(&box_start, (size_t)n_total + 1));
  // The records reach `recs` (one array, saved then target) either by two copies, or -- records already in device
  // memory, or a few of them in pinned host memory the device can read -- through the validation kernel, which
  // has to read them anyway: two operations fewer on the stream, and for device metadata one pass over it.
  const bcp_shard_meta *from_s = recs, *from_t = recs + n_saved;
  bcp_shard_meta* gather = nullptr;
  {
    const bool aligned = (((uintptr_t)saved | (uintptr_t)target) & 15u) == 0;
    const void *ds = saved, *dt = target;
    bool direct = aligned && (flags & BCP_META_ON_DEVICE);
    if (aligned && !direct && n_total <= kDirectUploadRecords)
      direct = (n_saved == 0 || device_visible(saved, &ds)) && device_visible(target, &dt);
    if (direct) {
      from_s = (const bcp_shard_meta*)ds;
      from_t = (const bcp_shard_meta*)dt;
      gather = recs;
    } else {
      const hipMemcpyKind up = (flags & BCP_META_ON_DEVICE) ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
      if (n_saved) BCP_HIP(hipMemcpyAsync(recs, saved, sizeof(bcp_shard_meta) * (size_t)n_saved, up, st));
      BCP_HIP(hipMemcpyAsync(recs + n_saved, target, sizeof(bcp_shard_meta) * (size_t)n_target, up, st));
    }
  }
  ull* cov = nullptr;  // per target record: elements found in saved shards
  BCP_HIP(ws.alloc(&cov, (size_t)n_target));
  hipLaunchKernelGGL(k_ctl_init, dim3(std::min(blocks_for(n_target), 1024u)), dim3(kBlock), 0, st, ctl, init, cov, n_target);
  BCP_HIP(hipGetLastError());
  BCP_HIP(hipEventRecord(ev0, st));

  // 1. validate + count boxes, scan                                                    (sync 1)
  if (gather)
    hipLaunchKernelGGL(k_validate_count<true>, dim3(blocks_for(n_total, kRecBlock)), dim3(kRecBlock), 0, st, from_s, from_t, gather,
                       n_saved, n_total, box_start, ctl);
  else
    hipLaunchKernelGGL(k_validate_count<false>, dim3(blocks_for(n_total, kRecBlock)), dim3(kRecBlock), 0, st, from_s, from_t, gather,
                       n_saved, n_total, box_start, ctl);
  BCP_HIP(hipGetLastError());
  if (bcp_status s = device_scan<uint32_t, uint32_t>(box_start, box_start, n_total, ws, st)) return s;
  if (bcp_status s = read_back(ws, st, ctl, &rb, box_start + n_saved, 4, box_start + n_total, 4)) return s;
  Ctl h = rb.ctl;
  if (bcp_status s = device_error(h, n_saved)) return s;
  const int64_t nbs = (int64_t)rb.v[0], nbt = (int64_t)(rb.v[1] - rb.v[0]), nbx = (int64_t)rb.v[1];
  out->n_saved_boxes = nbs;
  out->n_target_boxes = nbt;
  if (nbt == 0) {
    out->ctl = h;
    return BCP_OK;
  }

  Box* boxes = nullptr;
  BCP_HIP(ws.alloc(&boxes, (size_t)nbx));
  hipLaunchKernelGGL(k_emit_boxes, dim3(blocks_for(n_total)), dim3(kBlock), 0, st, recs, n_saved, n_total, box_start, boxes);
  BCP_HIP(hipGetLastError());

  // 2. sort saved boxes by fqn
  uint64_t *keys_a = nullptr, *keys_b = nullptr;
  uint32_t *idx_a = nullptr, *idx_b = nullptr;
  BCP_HIP(ws.alloc(&keys_a, (size_t)nbs));
  BCP_HIP(ws.alloc(&keys_b, (size_t)nbs));
  BCP_HIP(ws.alloc(&idx_a, (size_t)nbs));
  BCP_HIP(ws.alloc(&idx_b, (size_t)nbs));
  int bits = 0;  // significant bits of the largest saved FQN id
  while (bits < 64 && (h.max_saved_fqn >> bits) != 0) ++bits;
  if (nbs > 0 && nbs <= kSortSmallMax) {
    hipLaunchKernelGGL(k_sort_small, dim3(1), dim3(kSortSmallThreads), 0, st, boxes, (int)nbs, bits, keys_a, idx_a);
    BCP_HIP(hipGetLastError());
  } else if (nbs > 0) {
    const unsigned nblk = blocks_for(nbs);
    hipLaunchKernelGGL(k_sort_init, dim3(nblk), dim3(kBlock), 0, st, boxes, nbs, keys_a, idx_a);
    BCP_HIP(hipGetLastError());
    if (nbs > 1 && bits > 0) {
      uint32_t* hist = nullptr;
      BCP_HIP(ws.alloc(&hist, (size_t)16 * nblk + 1));
      for (int shift = 0; shift < bits; shift += 4) {
        hipLaunchKernelGGL(k_radix_hist, dim3(nblk), dim3(kBlock), 0, st, keys_a, nbs, shift, hist, nblk);
        BCP_HIP(hipGetLastError());
        if (bcp_status s = device_scan<uint32_t, uint32_t>(hist, hist, (int64_t)16 * nblk, ws, st)) return s;
        hipLaunchKernelGGL(k_radix_scatter, dim3(nblk), dim3(kBlock), 0, st, keys_a, idx_a, nbs, shift, hist, nblk, keys_b, idx_b);
        BCP_HIP(hipGetLastError());
        std::swap(keys_a, keys_b);
        std::swap(idx_a, idx_b);
      }
    }
  }

  // 3. candidate pairs                                                                     (sync 2)
  uint32_t* grp_lo = nullptr;
  uint64_t* pair_start = nullptr;
  BCP_HIP(ws.alloc(&grp_lo, (size_t)nbt));
  BCP_HIP(ws.alloc(&pair_start, (size_t)nbt + 1));
  hipLaunchKernelGGL(k_pair_count, dim3(blocks_for(nbt)), dim3(kBlock), 0, st, boxes, nbs, nbt, keys_a, idx_a, recs, n_saved,
                     (flags & BCP_CONVERT_F32_TO_BF16) ? 1 : 0, grp_lo, pair_start, ctl);
  BCP_HIP(hipGetLastError());
  if (bcp_status s = device_scan<uint64_t, uint64_t>(pair_start, pair_start, nbt, ws, st)) return s;
  if (nbs > 0) {
    hipLaunchKernelGGL(k_saved_check, dim3(blocks_for(nbs)), dim3(kBlock), 0, st, boxes, nbs, keys_a, idx_a, recs,
                       (flags & BCP_SKIP_OVERLAP_CHECK) ? 0 : 1, ctl);
    BCP_HIP(hipGetLastError());
  }
  if (bcp_status s = read_back(ws, st, ctl, &rb, pair_start + nbt, 8)) return s;
  h = rb.ctl;
  const uint64_t n_pairs = rb.v[0];
  if (bcp_status s = device_error(h, n_saved)) return s;
  if (n_pairs >= 0xffffffffull) {  // region indices are 32-bit
    set_error("too many candidate pairs");
    return BCP_ERR_OOM;
  }

  // 4. count, then write the non-empty intersections.  Regions are a plan-owned allocation: sized
  // by the pair count when that is cheap, else by the exact region count            (sync 3, rare)
  uint32_t n_regions = 0;
  Region* regions = nullptr;
  uint64_t* tile_start = nullptr;
  uint32_t* blk = nullptr;
  uint2* hits = nullptr;  // per block of 256 candidate pairs: the pairs that intersect
  ull* ext = nullptr;  // per-buffer extents: [source blobs | destination buffers] by record buffer index
  unsigned nblk_pairs = 0;
  if (n_pairs > 0) {
    nblk_pairs = blocks_for((int64_t)n_pairs);
    BCP_HIP(ws.alloc(&blk, (size_t)nblk_pairs + 1));
    BCP_HIP(ws.alloc(&hits, (size_t)nblk_pairs * kBlock));
    // what each buffer must hold: a table over every buffer index the records name, in up to 64 copies
    const uint32_t ext_src_bufs = (uint32_t)(h.max_saved_rec_buf + 1), ext_bufs = ext_src_bufs + (uint32_t)(h.max_target_rec_buf + 1);
    const uint32_t ext_stripes = (uint32_t)std::min<uint64_t>(64, std::max<uint64_t>(1, ((uint64_t)1 << 20) / std::max(ext_bufs, 1u)));
    BCP_HIP(ws.alloc(&ext, (size_t)ext_bufs * ext_stripes));
    size_t cap = (size_t)n_pairs;
    const bool exact = cap * sizeof(Region) > ((size_t)64 << 20);  // then the region list is sized after counting
    if (!exact) BCP_HIP(ws.alloc(&tile_start, cap + 1));
    hipLaunchKernelGGL(k_pairs_find, dim3(nblk_pairs), dim3(kBlock), 0, st, boxes, nbs, nbt, idx_a, grp_lo, pair_start,
                       n_pairs, blk, hits, tile_start, ext, (uint64_t)ext_bufs * ext_stripes);
    BCP_HIP(hipGetLastError());
    if (bcp_status s = device_scan<uint32_t, uint32_t>(blk, blk, nblk_pairs, ws, st)) return s;
    if (exact) {
      if (bcp_status s = read_back(ws, st, ctl, &rb, blk + nblk_pairs, 4)) return s;
      n_regions = (uint32_t)rb.v[0];
      cap = n_regions;
      BCP_HIP(ws.alloc(&tile_start, cap + 1));  // (pass 2 writes every count; the scan writes the entry after them)
    }
    BCP_HIP(block_alloc(&owned.p[0], std::max<size_t>(cap, 1) * sizeof(Region), &owned.bytes[0], st));
    regions = (Region*)owned.p[0];
    hipLaunchKernelGGL(k_pairs_build, dim3(nblk_pairs * (kBlock / kBuildHits)), dim3(kBuildWave), 0, st, boxes, nbs, hits, blk,
                       tile_bytes, regions, tile_start, cov, ctl, ext, ext_src_bufs, ext_bufs, ext_stripes);
    BCP_HIP(hipGetLastError());
    hipLaunchKernelGGL(k_extents_fold, dim3(blocks_for(ext_bufs, kBlock / 64)), dim3(kBlock), 0, st, ext, ext_bufs, ext_stripes);
    BCP_HIP(hipGetLastError());
    hipLaunchKernelGGL(k_coverage, dim3(blocks_for(n_target)), dim3(kBlock), 0, st, recs, n_saved, n_target, cov,
                       (flags & BCP_ALLOW_UNCOVERED) ? 1 : 0, ctl);
    BCP_HIP(hipGetLastError());
    if (bcp_status s = device_scan<uint64_t, uint64_t>(tile_start, tile_start, (int64_t)cap, ws, st)) return s;
    // tile total and region count                                                         (sync 4)
    if (bcp_status s = read_back(ws, st, ctl, &rb, tile_start + cap, 8, blk + nblk_pairs, 4)) return s;
    h = rb.ctl;
    const uint64_t n_tiles = rb.v[0];
    n_regions = (uint32_t)rb.v[1];
    if (bcp_status s = device_error(h, n_saved)) return s;
    if (n_tiles >= 0xffffffffull) {
      set_error("too many tiles; raise tile_bytes with bcp_configure");
      return BCP_ERR_OOM;
    }

    // 5. batches and descriptors: [heads | tiles] in one plan-owned allocation
    TileDesc* heads = nullptr;
    TileDesc* tiles = nullptr;
    uint32_t n_batches = 0;
    if (n_tiles > 0) {
      const bool by_source = (flags & BCP_ORDER_BY_SOURCE) != 0;
      // one allocation: heads | tiles | queue words | (source-ordered plans) one key per batch
      const size_t desc_bytes = sizeof(TileDesc) * 2 * (size_t)n_tiles;
      BCP_HIP(block_alloc(&owned.p[1], desc_bytes + 64 + (by_source ? sizeof(uint64_t) * (size_t)n_tiles : 0),
                          &owned.bytes[1], st));
      heads = (TileDesc*)owned.p[1];
      tiles = heads + n_tiles;
      out->dev.queue = (unsigned long long*)(tiles + n_tiles);
      out->dev.batch_key = by_source ? (uint64_t*)((char*)owned.p[1] + desc_bytes + 64) : nullptr;
      uint64_t* weight = nullptr;
      uint64_t* wprefix = nullptr;
      uint32_t* tile_region = nullptr;
      uint32_t* tile_local = nullptr;
      uint64_t* bflags = nullptr;
      uint32_t* bstart = nullptr;
      uint64_t* key = nullptr;
      uint32_t* order = nullptr;
      BCP_HIP(ws.alloc(&weight, (size_t)n_tiles));
      BCP_HIP(ws.alloc(&wprefix, (size_t)n_tiles + 1));
      BCP_HIP(ws.alloc(&tile_region, (size_t)n_tiles));
      BCP_HIP(ws.alloc(&tile_local, (size_t)n_tiles));
      BCP_HIP(ws.alloc(&bflags, (size_t)n_tiles + 2));
      BCP_HIP(ws.alloc(&bstart, (size_t)n_tiles + 1));
      if (by_source) {
        BCP_HIP(ws.alloc(&key, (size_t)n_tiles));
        BCP_HIP(ws.alloc(&order, (size_t)n_tiles));
      }
      const unsigned nblk = blocks_for((int64_t)n_tiles + 1);
      hipLaunchKernelGGL(k_tile_weights, dim3(nblk), dim3(kBlock), 0, st, tile_start, regions, (int64_t)n_regions,
                         n_tiles, tile_region, tile_local, weight, key, order, out->dev.queue);
      BCP_HIP(hipGetLastError());
      if (by_source) {
        // sort the tiles by (source buffer, last source byte): the plan can then run as blobs arrive
        if ((h.max_src_end >> kKeyShift) || h.max_src_buf >= ((long long)1 << (64 - kKeyShift))) {
          set_error("BCP_ORDER_BY_SOURCE: source offsets beyond 2^44 bytes or more than 2^20 source blobs");
          return BCP_ERR_INVALID_ARG;
        }
        uint64_t *key_b = nullptr, *w2 = nullptr;
        uint32_t *order_b = nullptr, *hist = nullptr, *r2 = nullptr, *l2 = nullptr;
        const unsigned nb = blocks_for((int64_t)n_tiles);
        BCP_HIP(ws.alloc(&key_b, (size_t)n_tiles));
        BCP_HIP(ws.alloc(&order_b, (size_t)n_tiles));
        BCP_HIP(ws.alloc(&hist, (size_t)16 * nb + 1));
        BCP_HIP(ws.alloc(&r2, (size_t)n_tiles));
        BCP_HIP(ws.alloc(&l2, (size_t)n_tiles));
        BCP_HIP(ws.alloc(&w2, (size_t)n_tiles));
        const uint64_t max_key = ((uint64_t)(h.max_src_buf < 0 ? 0 : h.max_src_buf) << kKeyShift) | (h.max_src_end ? h.max_src_end - 1 : 0);
        int bits = 0;
        while (bits < 64 && (max_key >> bits) != 0) ++bits;
        // low bits: byte offsets; then jump straight to the buffer-index bits
        int off_bits = 0;
        while (off_bits < kKeyShift && (h.max_src_end >> off_bits) != 0) ++off_bits;
        for (int shift = 0; shift < bits; shift += 4) {
          if (shift >= off_bits && shift + 4 <= kKeyShift) continue;  // all-zero digits
          hipLaunchKernelGGL(k_radix_hist, dim3(nb), dim3(kBlock), 0, st, key, (int64_t)n_tiles, shift, hist, nb);
          BCP_HIP(hipGetLastError());
          if (bcp_status s = device_scan<uint32_t, uint32_t>(hist, hist, (int64_t)16 * nb, ws, st)) return s;
          hipLaunchKernelGGL(k_radix_scatter, dim3(nb), dim3(kBlock), 0, st, key, order, (int64_t)n_tiles, shift, hist, nb, key_b, order_b);
          BCP_HIP(hipGetLastError());
          std::swap(key, key_b);
          std::swap(order, order_b);
        }
        hipLaunchKernelGGL(k_gather_tiles, dim3(nb), dim3(kBlock), 0, st, order, n_tiles, tile_region, tile_local, weight, r2, l2, w2);
        BCP_HIP(hipGetLastError());
        tile_region = r2;
        tile_local = l2;
        weight = w2;
      }
      if (bcp_status s = device_scan<uint64_t, uint64_t>(weight, wprefix, (int64_t)n_tiles, ws, st)) return s;
      hipLaunchKernelGGL(k_batch_flags, dim3(nblk), dim3(kBlock), 0, st, weight, wprefix, n_tiles, tile_bytes * kSmallBatchTiles, key, bflags);
      BCP_HIP(hipGetLastError());
      if (bcp_status s = device_scan<uint64_t, uint64_t>(bflags, bflags, (int64_t)n_tiles, ws, st)) return s;
      hipLaunchKernelGGL(k_batch_starts, dim3(nblk), dim3(kBlock), 0, st, bflags, n_tiles, bstart);
      hipLaunchKernelGGL(k_fill_tiles, dim3(nblk), dim3(kBlock), 0, st, regions, tile_region, tile_local,
                         bflags, bstart, n_tiles, tiles, heads, key, out->dev.batch_key);
      BCP_HIP(hipGetLastError());
      // the extents of the buffers the plan uses come back with the batch count
      const size_t n_src = (size_t)(h.max_src_buf + 1), n_dst = (size_t)(h.max_dst_buf + 1);
      BCP_HIP(ensure_landing(ws, kLandingExtents + sizeof(ull) * (n_src + n_dst)));  // (nothing is in flight into it)
      hipLaunchKernelGGL(k_final_readback, dim3(1), dim3(kBlock), 0, st, bflags + n_tiles, n_tiles, ext, (uint32_t)n_src,
                         ext + ext_src_bufs, (uint32_t)n_dst, (char*)ws.landing_dev);
      BCP_HIP(hipGetLastError());
      out->src_extent.resize(n_src);
      out->dst_extent.resize(n_dst);
    }
    BCP_HIP(hipEventRecord(ev1, st));
    BCP_HIP(hipStreamSynchronize(st));                                                 // (final sync)
    if (n_tiles > 0) {
      std::memcpy(&n_batches, ws.landing, sizeof(uint32_t));
      const char* e = (const char*)ws.landing + kLandingExtents;
      std::memcpy(out->src_extent.data(), e, sizeof(int64_t) * out->src_extent.size());
      std::memcpy(out->dst_extent.data(), e + sizeof(int64_t) * out->src_extent.size(), sizeof(int64_t) * out->dst_extent.size());
    }
    BCP_HIP(hipEventElapsedTime(&out->device_ms, ev0, ev1));
    h.n_tiles = n_tiles;
    out->dev.tiles = tiles;
    out->dev.heads = heads;
    out->dev.n_tiles = (int64_t)n_tiles;
    out->dev.n_batches = (int64_t)n_batches;
    out->dev.lds_transpose = (uint32_t)h.lds_transpose;
    out->dev.converts = h.n_convert != 0;
  } else {
    hipLaunchKernelGGL(k_coverage, dim3(blocks_for(n_target)), dim3(kBlock), 0, st, recs, n_saved, n_target, cov,
                       (flags & BCP_ALLOW_UNCOVERED) ? 1 : 0, ctl);
    BCP_HIP(hipGetLastError());
    if (bcp_status s = read_back(ws, st, ctl, &rb)) return s;
    h = rb.ctl;
    if (bcp_status s = device_error(h, n_saved)) return s;
  }

  h.n_pairs = n_pairs;
  h.n_regions = n_regions;
  out->ctl = h;
  out->dev.regions = regions;
  out->dev.n_regions = n_regions;
  out->dev.regions_bytes = owned.bytes[0];
  out->dev.desc_bytes = owned.bytes[1];
  owned.p[0] = owned.p[1] = nullptr;  // the plan owns them now
  return BCP_OK;
}

}  // namespace bcp
