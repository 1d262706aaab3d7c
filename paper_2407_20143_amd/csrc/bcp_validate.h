// Checks of single shard records and of the records of one tensor against each other, compiled for
// host and device: the planner kernels run them per record on the GPU, the host entry point
// bcp_validate_meta() runs the very same code without one.
#pragma once
#include <stdint.h>

#include "bcp.h"
#include "bcp_decompose.h"

namespace bcp {

// error codes carried in the low byte of the planner's error key (mapped to bcp_status on the host)
enum DevErr : unsigned {
  kErrInvalid = 1,
  kErrTooManyDims = 2,
  kErrBounds = 3,
  kErrShape = 4,
  kErrDtype = 5,
  kErrOverlap = 6,
  kErrUncovered = 7,
};

// Sec. 3.2: a record is a box (nD offsets, nD lengths) inside the tensor's global shape, a range of
// the box's row-major flattening, and where those elements are stored.  0: the record is well formed.
BCP_HD inline unsigned validate_record(const bcp_shard_meta& r) {
  if (r.ndim < 0) return kErrInvalid;
  if (r.ndim > kDims) return kErrTooManyDims;
  const int e = r.itemsize;
  if (!(e == 1 || e == 2 || e == 4 || e == 8 || e == 16)) return kErrInvalid;
  if (r.fqn_id < 0 || r.buf < 0 || r.byte_offset < 0 || r.reserved != 0) return kErrInvalid;
  int64_t vol = 1;
  bool strided = false;
  for (int k = 0; k < r.ndim; ++k) {
    if (r.global_shape[k] < 0 || r.offsets[k] < 0 || r.lengths[k] < 0 || r.strides[k] < 0) return kErrInvalid;
    if (r.offsets[k] > r.global_shape[k] || r.lengths[k] > r.global_shape[k] - r.offsets[k]) return kErrBounds;
    if (r.lengths[k] != 0 && vol > (int64_t)(0x3fffffffffffffffLL / r.lengths[k])) return kErrInvalid;
    vol *= r.lengths[k];
    strided |= r.strides[k] != 0;
  }
  if (r.flat_begin < 0 || r.flat_end < r.flat_begin) return kErrInvalid;
  if (r.flat_end > vol) return kErrBounds;
  // byte addresses inside the buffer must stay far from the 64-bit limit: at most 2^56 elements of
  // storage behind byte_offset < 2^60
  constexpr int64_t kMaxSpan = (int64_t)1 << 56;
  if (r.byte_offset >= ((int64_t)1 << 60)) return kErrInvalid;
  if (strided) {
    if (!(r.flat_begin == 0 && r.flat_end == vol)) return kErrInvalid;  // flat shards are packed
    int64_t span = 0;  // element offset of the last element
    for (int k = 0; k < r.ndim; ++k) {
      if (r.lengths[k] > 1 && r.strides[k] == 0) return kErrInvalid;
      if (r.lengths[k] > 1) {
        if (r.strides[k] > (kMaxSpan - span) / (r.lengths[k] - 1)) return kErrInvalid;
        span += (r.lengths[k] - 1) * r.strides[k];
      }
    }
  } else if (vol > kMaxSpan) {
    return kErrInvalid;
  }
  return 0;
}

// Two records of one FQN describe the same tensor: equal rank and global shape, equal element size.
// `convert` (a saved record against a target record of a plan built with BCP_CONVERT_F32_TO_BF16):
// 4-byte saved elements may also be asked for as 2-byte elements.
BCP_HD inline unsigned same_tensor(const bcp_shard_meta& a, const bcp_shard_meta& b, bool convert = false) {
  if (a.ndim != b.ndim) return kErrShape;
  for (int k = 0; k < a.ndim; ++k)
    if (a.global_shape[k] != b.global_shape[k]) return kErrShape;
  if (a.itemsize != b.itemsize && !(convert && a.itemsize == 4 && b.itemsize == 2)) return kErrDtype;
  return 0;
}

// extents of the box a record's flat range is taken from (a scalar is one dimension of extent 1)
BCP_HD inline int local_shape(const bcp_shard_meta& r, int64_t* len) {
  if (r.ndim == 0) {
    len[0] = 1;
    return 1;
  }
  for (int k = 0; k < r.ndim; ++k) len[k] = r.lengths[k];
  return r.ndim;
}

}  // namespace bcp
