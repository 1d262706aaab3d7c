/*
 * bcp -- load-time checkpoint resharding on one MI355X (gfx950): C-ABI boundary.
 *
 * The library takes saved tensor shards in the paper's parallelism-agnostic representation
 * (Sec. 3.2 "Decoupled Checkpoint Representation": FQN + global shape, ShardMeta =
 * (fqn, nD_offsets, nD_lengths), BasicMeta = itemsize/strides, ByteMeta = byte offset inside
 * a storage blob) and builds the shards a different TP/PP/DP/EP layout asks for
 * (Sec. 3.3 "Checkpoint Resharding Workflow", Step 2: matching segments between saved shards and
 * the new sharding specification).  Storage I/O is outside: saved blobs are byte buffers that
 * already sit in device memory.
 *
 * All functions return a bcp_status and never throw.  They may be called from several threads:
 * the process-wide state (the launch configuration of bcp_configure, the planner's workspace, the
 * pool of plan blocks) is guarded by locks -- concurrent bcp_plan calls take turns -- and the error
 * text is per thread; calls on ONE plan must be ordered by the caller.  "host" / "device" below
 * says where a pointer must point.
 */
#ifndef BCP_H_
#define BCP_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BCP_MAX_DIMS 8

/* One stored shard (saved or target): ShardMeta + BasicMeta + ByteMeta of Sec. 3.2.
 *
 * The shard holds elements [flat_begin, flat_end) of the row-major flattening of the box
 * (offsets, lengths) of tensor `fqn_id`.  flat range == [0, volume) is a regular shard; any other
 * range is an irregular (ZeRO flat) shard, Sec. 3.2 "Decomposing irregular tensors".
 * Storage: element j of that range sits at byte_offset + itemsize*j of buffer `buf` (packed),
 * unless `strides` is non-zero, in which case the shard must be regular and the element with
 * box-local coordinates y sits at byte_offset + itemsize * sum_k y[k]*strides[k].
 * ndim == 0 is a scalar (volume 1).  Zero-volume shards are legal and produce no work.
 * Limits (BCP_ERR_INVALID_ARG beyond them): byte_offset < 2^60, and the storage of one shard spans
 * at most 2^56 elements (volume for packed shards, offset of the last element for strided ones). */
typedef struct bcp_shard_meta {
  int64_t fqn_id;                     /* >= 0; identifies the tensor (string table stays with the caller) */
  int32_t ndim;                       /* 0..BCP_MAX_DIMS */
  int32_t itemsize;                   /* bytes per element: 1, 2, 4, 8 or 16; the dtype itself is opaque (the one
                                         cast there is: BCP_CONVERT_F32_TO_BF16) */
  int64_t global_shape[BCP_MAX_DIMS]; /* shape before sharding */
  int64_t offsets[BCP_MAX_DIMS];      /* nD_offsets */
  int64_t lengths[BCP_MAX_DIMS];      /* nD_lengths */
  int64_t flat_begin;                 /* element range inside the box, row-major */
  int64_t flat_end;
  int64_t strides[BCP_MAX_DIMS];      /* element strides; all zero == packed */
  int64_t byte_offset;                /* where the first stored element sits in the buffer */
  int32_t buf;                        /* index into src_blobs[] (saved) / dst_buffers[] (target) */
  int32_t reserved;                   /* must be 0 */
} bcp_shard_meta;

typedef struct bcp_plan_s* bcp_plan_t; /* opaque; owns device-side region and tile tables */

typedef enum bcp_status {
  BCP_OK = 0,
  BCP_ERR_INVALID_ARG = -1,     /* null pointer, negative count, bad ndim/itemsize/flat range/strides */
  BCP_ERR_SHAPE_MISMATCH = -2,  /* records of one FQN disagree on ndim or global shape */
  BCP_ERR_DTYPE_MISMATCH = -3,  /* records of one FQN disagree on itemsize (and no conversion covers the pair) */
  BCP_ERR_OUT_OF_BOUNDS = -4,   /* offsets+lengths beyond the global shape, or flat range beyond the box */
  BCP_ERR_SAVED_OVERLAP = -5,   /* two saved shards hold the same element (Sec. 4.1: one saver per shard) */
  BCP_ERR_UNCOVERED = -6,       /* a target element no saved shard holds */
  BCP_ERR_TOO_MANY_DIMS = -7,
  BCP_ERR_OOM = -8,
  BCP_ERR_HIP = -9,             /* a HIP runtime call failed; bcp_last_error() has its text */
  BCP_ERR_NO_DEVICE = -10       /* no usable GPU */
} bcp_status;

/* flags of bcp_plan */
#define BCP_PLAN_DEFAULT 0u
#define BCP_ALLOW_UNCOVERED 1u      /* target elements without a saved source keep their bytes */
#define BCP_SKIP_OVERLAP_CHECK 2u   /* trust the caller that saved shards are pairwise disjoint */
#define BCP_ORDER_BY_SOURCE 4u      /* order the work by (source blob, source byte) so that it can run
                                       while the blobs arrive: see bcp_reshard_arrived */
#define BCP_META_ON_DEVICE 8u       /* saved / target point to DEVICE memory (metadata produced or kept on the
                                       GPU): no host-to-device upload of the records */
#define BCP_CONVERT_F32_TO_BF16 16u /* dtype-converting load (Sec. 2.2: evaluation jobs load the model only, so
                                       fp32 master weights are read as bf16): a tensor whose saved records have
                                       itemsize 4 and whose target records have itemsize 2 is narrowed on the way,
                                       binary32 -> bfloat16, round to nearest, ties to even; infinities stay, NaN
                                       stays NaN (sign and upper seven fraction bits kept, quiet bit set).  Tensors
                                       whose sizes agree are moved as they are; any other disagreement stays
                                       BCP_ERR_DTYPE_MISMATCH */

typedef struct bcp_stats {
  int64_t n_saved_boxes;   /* regular boxes after decomposing the saved records */
  int64_t n_target_boxes;
  int64_t n_pairs;         /* candidate (saved box, target box) pairs with equal FQN */
  int64_t n_regions;       /* non-empty intersections == copy regions */
  int64_t n_tiles;         /* work items of the copy kernel */
  int64_t payload_bytes;   /* bytes the copy moves one way */
  int64_t n_transposed;    /* regions taken by the LDS-staged path (inner strides disagree) */
  int64_t max_src_buf;     /* largest buffer index used, -1 if none */
  int64_t max_dst_buf;
  int64_t region_dims_hist[BCP_MAX_DIMS + 1]; /* regions by number of dims after coalescing */
  double plan_device_ms;   /* device time of the planner kernels (HIP events) */
  double plan_wall_ms;     /* wall time of bcp_plan */
  int64_t n_batches;       /* queue items of the copy kernel: one big tile or a run of small ones */
  int64_t src_bytes;       /* bytes the copy reads: payload_bytes (which counts bytes written) unless tensors are
                              converted on the way */
} bcp_stats;

/* Region as the copy kernel sees it (for inspection and tests; many region lists are valid). */
typedef struct bcp_region_info {
  int64_t src_base, dst_base;         /* byte offsets inside src_blobs[src_buf] / dst_buffers[dst_buf] */
  int64_t run_bytes;                  /* contiguous inner run on both sides */
  int64_t len[BCP_MAX_DIMS];          /* outer extents (rows), slowest first */
  int64_t src_pitch[BCP_MAX_DIMS];    /* bytes */
  int64_t dst_pitch[BCP_MAX_DIMS];
  int32_t ndim;                       /* number of outer dims */
  int32_t src_buf, dst_buf;
  int32_t kind;                       /* 0: rows of contiguous runs, 1: LDS-staged transpose */
  int64_t target_index;               /* index of the target record the region belongs to */
  int64_t saved_index;                /* index of the saved record */
} bcp_region_info;

/* Step a1 (host helper): cut a flat ZeRO buffer at tensor boundaries.
 * `params_in_order[i]` are regular records (flat range == whole box) whose row-major flattenings,
 * concatenated in this order, form the flat buffer (Appendix A: TP-local shards are flattened and
 * merged before being sharded by the DP degree).  The slice [A, B) of that concatenation, stored
 * packed at `byte_offset` of buffer `buf`, is returned as one record per tensor it touches: same
 * box, flat range = the part of the tensor inside the slice, byte_offset advanced accordingly.
 * out (host) has room for *inout_n records; on return *inout_n is the number needed/written
 * (BCP_ERR_INVALID_ARG with *inout_n set if the room was too small).  No GPU involved. */
bcp_status bcp_meta_from_flat_slice(const bcp_shard_meta* params_in_order, int64_t n_params,
                                    int64_t A, int64_t B, int32_t buf, int64_t byte_offset,
                                    bcp_shard_meta* out, int64_t* inout_n);

/* Step a2 (host mirror of the device decomposer, for inspection and tests): the regular boxes of
 * one record, in ascending flat order; out_boxes[i] is a regular, packed record (global offsets and
 * lengths, byte_offset of its first element).  At most 2*ndim-1 (min 1) boxes; *inout_n as above.
 * Sec. 3.2 "Decomposing irregular tensors": an irregular shard becomes a series of regular ones. */
bcp_status bcp_decompose(const bcp_shard_meta* rec, bcp_shard_meta* out_boxes, int64_t* inout_n);

/* Save-side deduplication (Sec. 4.1 "Balancing saving workload"): under data parallelism the
 * same shard lives on several ranks; each must be saved by exactly one of them, and the savers are
 * chosen Worst-Fit so that the bytes to save are spread evenly.  recs[i] (host) is held by rank
 * rank_of[i] in [0, n_ranks).  Records with equal fqn_id, ndim, itemsize, offsets, lengths and flat
 * range are replicas of one shard.  The distinct shards are taken in order of first appearance; each
 * goes to the holder with the fewest bytes assigned so far (ties: the lowest rank).  keep[i]
 * (host, n entries) becomes 1 for the chosen record and 0 for its other replicas; load (host,
 * n_ranks entries, may be null) receives the bytes assigned per rank.  The kept records are pairwise
 * disjoint if the distinct shards were, i.e. they are a valid saved side for bcp_plan; planning
 * kept live records against a packed blob layout is the save-side "pack", the inverse of a load.
 * Host only, no GPU involved. */
bcp_status bcp_dedup_worst_fit(const bcp_shard_meta* recs, const int32_t* rank_of, int64_t n, int32_t n_ranks,
                               uint8_t* keep, int64_t* load);

/* The checks bcp_plan makes on the shard metadata, on the host and without a GPU: every record on its
 * own (fields, box inside the global shape, flat range inside the box: Sec. 3.2), the records of one
 * FQN against each other (rank, global shape, element size), saved shards pairwise disjoint (Sec. 4.1:
 * one saver per shard), every target element held by a saved shard.  Returns what bcp_plan would return
 * for the same arrays and flags (BCP_ALLOW_UNCOVERED, BCP_SKIP_OVERLAP_CHECK, BCP_CONVERT_F32_TO_BF16 are
 * honoured, BCP_ORDER_BY_SOURCE is accepted), with the offending record in bcp_last_error().  Host
 * arrays only.  Quadratic in the number of shards of one tensor: meant for checking metadata where no
 * GPU is at hand (a planning or CI host), not as a step before every bcp_plan. */
bcp_status bcp_validate_meta(const bcp_shard_meta* saved, int64_t n_saved,
                             const bcp_shard_meta* target, int64_t n_target, uint32_t flags);

/* Build a copy plan on the current HIP device (Sec. 3.3 Step 2 on the GPU).
 * saved/target: host arrays (device arrays with BCP_META_ON_DEVICE), borrowed for the duration of
 * the call; with very many records (the upload is 304 bytes each) pinned host memory pays.  stream: hipStream_t
 * (0 == default stream) the planner kernels run on; the call returns after they finished, so
 * the plan is usable on any stream.  On success *out_plan owns device memory until
 * bcp_plan_destroy.  Saved FQNs no target asks for are ignored.  A plan is immutable and may be
 * replayed on any buffers that have the layout it was planned for. */
bcp_status bcp_plan(const bcp_shard_meta* saved, int64_t n_saved,
                    const bcp_shard_meta* target, int64_t n_target,
                    uint32_t flags, void* stream, bcp_plan_t* out_plan);

/* Move the bytes: for every region, dst_buffers[dst_buf][...] = src_blobs[src_buf][...].
 * This is where the paper's load pipeline puts the deserialised bytes of the matching segments into the
 * new shards (Sec. 3.3 Step 5 and the read -> deserialize -> H2D pipeline of Sec. 4.2), with the saved
 * blobs already in device memory.
 * src_blobs / dst_buffers: HOST arrays of DEVICE pointers (n_src > max_src_buf, n_dst >
 * max_dst_buf), owned by the caller; buffers must stay valid until the work queued on `stream`
 * completed and must not overlap each other.  Asynchronous: enqueues on `stream` (hipStream_t)
 * and returns; errors detectable on the host are returned synchronously.  Calls on one plan must
 * be ordered by the caller (same stream, or synchronised) because they share the plan's pointer
 * tables and queue counter.
 * With at most 256 buffers in all (n_src + n_dst of the plan) the call is exactly one kernel launch
 * that leaves the plan ready for the next one, and may be captured into a HIP graph (call it once
 * outside the capture first); with more buffers it stages a pointer table through pinned memory
 * (allocations on first use, a host-to-device copy, possibly a wait) and must not be captured. */
bcp_status bcp_reshard(bcp_plan_t plan, const void* const* src_blobs, int32_t n_src,
                       void* const* dst_buffers, int32_t n_dst, void* stream);

/* bcp_reshard for callers that know their buffer sizes: src_bytes[i] / dst_bytes[i] (host arrays, n_src /
 * n_dst entries) are the sizes of src_blobs[i] / dst_buffers[i].  A buffer shorter than what the plan
 * reads from or writes to it is BCP_ERR_OUT_OF_BOUNDS, returned before anything is launched (the extents
 * are computed once, when the plan is built: the check costs a loop over the buffers on the host).
 * bcp_reshard itself never sees sizes: there an undersized buffer is a GPU memory fault. */
bcp_status bcp_reshard_checked(bcp_plan_t plan, const void* const* src_blobs, const int64_t* src_bytes, int32_t n_src,
                               void* const* dst_buffers, const int64_t* dst_bytes, int32_t n_dst, void* stream);

/* Chunked arrival (the step before this path in the paper's load pipeline, Sec. 4.2: read ->
 * deserialize -> H2D): run the part of a BCP_ORDER_BY_SOURCE plan whose LAST source byte lies in
 * bytes [byte_begin, byte_end) of src_blobs[src_buf].  Valid once bytes [0, byte_end) of that blob
 * are in place in stream order; calling it for consecutive chunks that cover every blob executes
 * every region exactly once.  Other arguments and rules as bcp_reshard. */
bcp_status bcp_reshard_arrived(bcp_plan_t plan, const void* const* src_blobs, int32_t n_src,
                               void* const* dst_buffers, int32_t n_dst,
                               int32_t src_buf, int64_t byte_begin, int64_t byte_end, void* stream);

/* The whole overlapped loop (the H2D stage of the load pipeline of Sec. 4.2 run against the reshard):
 * blob by blob, chunk by chunk, copy host_blobs[i] (HOST memory, pinned for real overlap, blob_bytes[i]
 * bytes) into src_blobs[i] (device, at least as large) on copy_stream and run bcp_reshard_arrived for
 * the chunk on `stream` as soon as it has landed.  Enqueues everything and returns; both streams keep
 * their default priority.  The plan must be BCP_ORDER_BY_SOURCE.  A blob shorter than what the plan
 * reads from it is BCP_ERR_OUT_OF_BOUNDS (its last regions would never run). */
bcp_status bcp_reshard_from_host(bcp_plan_t plan, const void* const* host_blobs, const int64_t* blob_bytes,
                                 void* const* src_blobs, int32_t n_src, void* const* dst_buffers, int32_t n_dst,
                                 int64_t chunk_bytes, void* copy_stream, void* stream);

/* bcp_reshard for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same result.  What bcp_reshard
 * keeps in memory the library allocates -- the queue words of the persistent grid, and the table of
 * buffer pointers when there are more than 256 buffers -- lives in a static array in device memory
 * instead (64 KiB + 256 bytes per GPU, held until the process ends), so the call is a few kernel
 * launches on `stream` and nothing else: no hipMalloc, no hipFree, no host-to-device copy, no wait.
 * Limit: n_src + n_dst of the plan at most BCP_NOALLOC_MAX_BUFFERS, else BCP_ERR_INVALID_ARG.
 * Every call on one GPU uses that GPU's one array (its words are put back to zero at the start of
 * each call, in stream order): calls that overlap in time on one GPU -- on different streams, or on
 * different plans -- race and must be ordered by the caller. */
#define BCP_NOALLOC_MAX_BUFFERS 8192
bcp_status bcp_reshard_noalloc(bcp_plan_t plan, const void* const* src_blobs, int32_t n_src,
                               void* const* dst_buffers, int32_t n_dst, void* stream);

bcp_status bcp_plan_stats(bcp_plan_t plan, bcp_stats* out);

/* Copy up to `capacity` regions to out (host); *n_regions receives the plan's region count. */
bcp_status bcp_plan_regions(bcp_plan_t plan, bcp_region_info* out, int64_t capacity, int64_t* n_regions);

/* Smallest buffer sizes the plan is safe on: src_extent[i] / dst_extent[i] (host arrays of n_src /
 * n_dst entries, at least max_*_buf + 1) receive one past the highest byte any region touches in
 * src_blobs[i] / dst_buffers[i] (0 if unused).  Computed when the plan is built; this call only
 * copies them out. */
bcp_status bcp_plan_buffer_extents(bcp_plan_t plan, int64_t* src_extent, int32_t n_src,
                                   int64_t* dst_extent, int32_t n_dst);

/* Releases the plan.  May be called as soon as the last bcp_reshard* call on the plan has returned,
 * also while that work is still queued or running: the plan's device blocks go to a small pool from
 * which later plans are served, ordered behind the work that still reads them (so a plan / destroy
 * cycle allocates nothing); what the pool does not keep is freed, which waits for the device. */
bcp_status bcp_plan_destroy(bcp_plan_t plan);

/* Launch configuration of the copy kernel (process-wide; takes effect at the next bcp_plan /
 * bcp_reshard).  tile_bytes: payload per work item, a power of two in [4 KiB, 4 MiB], used by
 * plans built afterwards (default 64 KiB).  persistent > 0: a fixed grid of wg_per_cu * CU-count
 * workgroups pops tiles from an atomic queue (default, wg_per_cu 1); 0: one workgroup per tile;
 * < 0 keeps the setting.  threads: 256, 512 or 1024 per workgroup (default 1024).  tile_bytes,
 * wg_per_cu, threads <= 0 keep the current setting. */
bcp_status bcp_configure(int64_t tile_bytes, int32_t persistent, int32_t wg_per_cu, int32_t threads);

/* bcp_plan keeps its temporaries (records, boxes, sort keys, scans) in a process-wide workspace in
 * device memory that only grows, so that a later plan of the same size allocates nothing, and
 * bcp_plan_destroy keeps a few device blocks of destroyed plans (at most 1 GiB) for the next ones.
 * This call frees both (they come back on demand); *freed_bytes, if not null, receives what was
 * released.  Plans already built are not affected.  Waits for no stream: the caller makes sure no
 * bcp_plan call is in flight on another thread (it would block until that call returned). */
bcp_status bcp_release_workspace(int64_t* freed_bytes);

const char* bcp_last_error(void); /* thread-local text of the last failure on this thread */
const char* bcp_status_name(bcp_status s);
int32_t bcp_abi_version(void);
int64_t bcp_sizeof_shard_meta(void);

#ifdef __cplusplus
}
#endif
#endif /* BCP_H_ */
