// Internal data structures shared by the planner, the copy kernels and the C-ABI layer.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "bcp.h"
#include "bcp_decompose.h"
#include "bcp_host.h"
#include "bcp_validate.h"

namespace bcp {

static_assert(kDims == BCP_MAX_DIMS, "dimension limit");

// A regular box of one stored record, in global coordinates, with where its elements live.
struct Box {
  int64_t fqn;
  int64_t off[kDims];
  int64_t len[kDims];
  int64_t stride[kDims];  // element strides of the storage
  int64_t byte_base;      // byte offset (in buffer `buf`) of the box's first element
  int32_t rec;            // index of the record it came from (within its side)
  int32_t ndim;           // >= 1 (scalars are stored as one dimension of extent 1)
  int32_t itemsize;
  int32_t buf;
};

enum RegionKind : int32_t { kRows = 0, kTranspose = 1, kConvert = 2 };

// One copy region: `len[0..ndim)` rows (slowest first) of `run_bytes` contiguous bytes.
// kTranspose: run_bytes == itemsize, len[ndim-2] runs along the source-contiguous dimension
// (src pitch == itemsize) and len[ndim-1] along the destination-contiguous one.
// kConvert: rows of 4-byte source elements that arrive as 2-byte elements (binary32 -> bfloat16);
// run_bytes counts SOURCE bytes, the destination run is half as long; pitches are bytes of their side.
struct Region {
  int64_t src_base, dst_base;
  int64_t run_bytes;
  int64_t len[kDims];
  int64_t spitch[kDims];
  int64_t dpitch[kDims];
  int32_t ndim;
  int32_t src_buf, dst_buf;
  int32_t kind;
  int32_t trec, srec;
  // tiling (see tile_region)
  uint32_t tile_bytes;       // payload budget per tile
  uint32_t rows_per_tile;    // kRows, run < tile_bytes: rows of the last row dimension per tile
  uint32_t segs_per_row;     // kRows, run >= tile_bytes: tiles per row
  uint32_t tiles_per_group;  // tiles per index of the leading row dimensions
  uint32_t tdim_a, tdim_b;   // kTranspose: tile edges in elements (powers of two) along the
                             // source-contiguous / destination-contiguous dimension
  uint32_t tiles_b;          // kTranspose: tiles along the last dimension
  uint32_t lead_mod;         // kRows, long rows: cut segments where the destination offset is a
                             // multiple of this (0: offsets are aligned anyway, cut at multiples of
                             // tile_bytes from the row start)
  uint64_t n_tiles;
};

// One work item of the copy kernel, fully decoded at plan time so that the kernel needs a single
// 64-byte (scalar) load per tile.
//   kRows:      `b` rows of `a` contiguous bytes, row pitches p0 (source) / p1 (destination)
//   kTranspose: `a` x `b` elements of `esize` bytes; the source is contiguous along a with pitch
//               p0 along b, the destination contiguous along b with pitch p1 along a
//   kConvert:   `b` rows of `a` ELEMENTS (4 bytes in the source, 2 in the destination), pitches in bytes
//
// The queue of the copy kernel hands out BATCHES: one big tile, or a run of small tiles (each
// below kSmallTileBytes, together a few tile budgets) that the threads of a workgroup share.  The
// small tiles are numbered among themselves, in tile order, and `tiles[]` holds them by that number:
// a batch is a run of it, whatever big tiles stand between its members in tile order.
// `heads[slot]` is a copy of a batch's first tile descriptor with `first` and `count` filled in,
// so the kernel still needs one descriptor load per queue pop.  Slots are in queue order: the big
// tiles in tile order with the small-tile batches spread evenly among them (plans ordered by
// source keep tile order throughout, and their batches are runs of consecutive tiles).
struct TileDesc {
  int64_t src_off, dst_off;  // byte offsets inside the source / destination buffer
  int64_t p0, p1;
  uint32_t a, b;
  uint32_t src_buf, dst_buf;
  uint32_t kind;             // RegionKind | esize << 8 | kTranspose: log2 of the full tile's edges, a << 16, b << 24
  uint32_t first;            // heads[] only: index in tiles[] of the batch's first tile
  uint32_t count;            // heads[] only: tiles in the batch
  uint32_t pad_;
};
static_assert(sizeof(TileDesc) == 64, "one tile descriptor per 64-byte line");

constexpr int kKeyShift = 44;                    // source-order key: buffer index above, byte offset below
constexpr uint32_t kSmallTileBytes = 16 * 1024;  // tiles below this may share a batch
constexpr uint32_t kMinBatchWeight = 256;        // a tile counts at least this much: <= budget/256 tiles per batch
constexpr uint32_t kSmallBatchTiles = 4;         // budget of a batch of small tiles, in tile budgets: up to 1024 tiles,
                                                 // one per thread of the copy kernel's workgroup (measured: 4 beats 1 and 8)

// Device control block: written by kernels, read back by the host between phases.
struct Ctl {
  unsigned long long err_key;  // min over (record index << 8 | code); ~0 == no error
  unsigned long long max_saved_fqn;
  unsigned long long n_pairs;
  unsigned long long n_regions;
  unsigned long long n_tiles;
  unsigned long long payload_bytes;
  unsigned long long n_transposed;
  long long max_src_buf, max_dst_buf;
  unsigned long long dims_hist[kDims + 1];
  unsigned long long max_src_end;  // one past the highest source byte offset any region reads
  unsigned long long lds_transpose;  // LDS staging bytes the largest transposed tile needs
  unsigned long long src_bytes;      // bytes the copy reads (differs from payload_bytes when regions convert)
  unsigned long long n_convert;      // regions that convert
  long long max_saved_rec_buf, max_target_rec_buf;  // largest buffer index any saved / target RECORD names (-1: none)
};

struct PlanConfig {
  int64_t tile_bytes = 64 * 1024;
  int32_t persistent = 1;  // workgroups pop tiles from an atomic queue (0: one workgroup per tile)
  int32_t wg_per_cu = 1;   // persistent grid = wg_per_cu * number of CUs
  int32_t threads = 1024;  // threads per workgroup
};
PlanConfig config();  // a snapshot of the process-wide setting

bcp_status hip_fail(hipError_t e, const char* what);

#define BCP_HIP(expr)                                   \
  do {                                                  \
    hipError_t e_ = (expr);                             \
    if (e_ != hipSuccess) return hip_fail(e_, #expr);   \
  } while (0)

// ---- planner (bcp_planner.hip) -------------------------------------------------------------
struct PlanDevice {
  Region* regions = nullptr;
  TileDesc* tiles = nullptr;
  TileDesc* heads = nullptr;  // one per batch; heads, tiles and queue share one allocation
  unsigned long long* queue = nullptr;  // [next batch, finished workgroups, range begin, range end]
  uint64_t* batch_key = nullptr;        // source-ordered plans: (src_buf << kKeyShift | last source byte) per batch
  int64_t n_regions = 0;
  int64_t n_tiles = 0;
  int64_t n_batches = 0;
  uint32_t lds_transpose = 0;  // LDS staging bytes of the largest transposed tile (0: none)
  bool converts = false;       // some tiles narrow binary32 to bfloat16
  size_t regions_bytes = 0, desc_bytes = 0;  // sizes of the two allocations (regions; heads | tiles | queue | keys)
};

// Device blocks that plans own.  A destroyed plan's blocks are kept (a few, up to a byte limit) and
// handed to the next plan that they fit: a plan / destroy cycle then allocates nothing, and
// allocation is the one step of plan building whose duration is not predictable.
//   block_alloc: *got receives the block's real size (at least `bytes`); a recycled block is
//                ordered behind its previous user through an event that `st` waits for.
//   block_free:  `last_use`: the stream the block's last user ran on (`used` false: none).
//   block_pool_release: frees the kept blocks, returns their bytes.
hipError_t block_alloc(void** p, size_t bytes, size_t* got, hipStream_t st);
void block_free(void* p, size_t bytes, bool used, hipStream_t last_use);
int64_t block_pool_release();

struct PlannerResult {
  PlanDevice dev;
  Ctl ctl;
  std::vector<int64_t> src_extent, dst_extent;  // per buffer: one past the highest byte the plan touches
  int64_t n_saved_boxes = 0, n_target_boxes = 0;
  float device_ms = 0.f;
};

bcp_status release_workspace(int64_t* freed_bytes);
bcp_status run_planner(const bcp_shard_meta* saved, int64_t n_saved, const bcp_shard_meta* target,
                       int64_t n_target, uint32_t flags, hipStream_t stream, PlannerResult* out);

// ---- copy (bcp_copy.hip) ---------------------------------------------------------------------
constexpr int kMaxKernargPtrs = 256;  // buffer pointers that travel as kernel arguments
// Edges, in elements, of the tiles of a transposed region, by element size: 64 KiB of payload,
// runs of 512 bytes on both sides where that allows it.
constexpr uint32_t transpose_edge_a(uint32_t esize) { return esize <= 2 ? 256u : (esize <= 8 ? 128u : 64u); }
constexpr uint32_t transpose_edge_b(uint32_t esize) { return esize <= 2 ? 256u : (esize <= 4 ? 128u : 64u); }
// LDS staging of one tile: tdim_a rows (one per index along a) of tdim_b elements plus one
// element of padding, which spreads a column over the banks
constexpr uint32_t transpose_lds_bytes(uint32_t tdim_a, uint32_t tdim_b, uint32_t esize) {
  // 2-byte elements: full tiles go through per-wave blocks, 16 x 64 rows of 144 bytes
  return esize == 2 ? 16u * 64u * 144u : tdim_a * (tdim_b + 1) * esize;
}
static_assert(transpose_lds_bytes(256, 256, 2) >= 256 * 257 * 2, "also holds the workgroup-wide staging of a ragged 2-byte tile");
bcp_status launch_reshard(const PlanDevice& plan, const void* const* src, int32_t n_src, void* const* dst,
                          int32_t n_dst, const void* table, hipStream_t stream,
                          const uint64_t* key_range = nullptr);
// bcp_reshard_noalloc: pointer table and queue words in a static device array, no allocation
bcp_status launch_reshard_noalloc(const PlanDevice& plan, const void* const* src, int32_t n_src, void* const* dst,
                                  int32_t n_dst, hipStream_t stream);
int device_cu_count();

}  // namespace bcp
