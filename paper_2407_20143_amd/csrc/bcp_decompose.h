// Decomposition of an irregular (flat) shard into regular boxes -- Sec. 3.2 "Decomposing
// irregular tensors": an irregular shard is represented by a series of regular shards, each with
// its own (nD offsets, nD lengths).  The paper fixes no granularity; this is the canonical
// minimal split: the boxes are disjoint, each is contiguous in the row-major order of the
// enclosing box, they come out in ascending flat order and there are at most 2*n-1 of them.
//
// One function, compiled for host and device: the planner kernels call it per record on the GPU,
// the host entry point bcp_decompose() exposes the very same code for inspection and tests.
#pragma once
#include <stdint.h>

#ifndef BCP_HD
#ifdef __HIPCC__
#define BCP_HD __host__ __device__
#else
#define BCP_HD
#endif
#endif

namespace bcp {

constexpr int kDims = 8;
constexpr int kMaxBoxesPerRecord = 2 * kDims - 1;

struct LocalBox {          // coordinates relative to the enclosing box
  int64_t off[kDims];
  int64_t len[kDims];
  int64_t flat_start;      // row-major position (in the enclosing box) of the box's first element
};

// Range [a, b) of the row-major flattening of a box with extents len[0..n).  Writes the boxes to
// out (may be null: count only) and returns their number.  n >= 1, 0 <= a <= b <= prod(len).
BCP_HD inline int decompose_flat_range(const int64_t* len, int n, int64_t a, int64_t b, LocalBox* out) {
  if (a >= b) return 0;
  int64_t inner[kDims];  // inner[k] = prod(len[k+1..n))
  inner[n - 1] = 1;
  for (int k = n - 2; k >= 0; --k) inner[k] = inner[k + 1] * len[k + 1];

  int64_t fixed[kDims];  // coordinates of the dimensions already pinned to one index
  int k = 0;
  int64_t ia, ra, ib, rb;
  // walk down while the whole range lies inside one index of dimension k
  for (;;) {
    ia = a / inner[k];
    ra = a - ia * inner[k];
    ib = b / inner[k];
    rb = b - ib * inner[k];
    if (ia != ib) break;  // (k == n-1 always breaks: inner == 1 and a < b)
    fixed[k] = ia;
    a = ra;
    b = rb;
    ++k;
  }
  // split level k: [ra, inner) of index ia, whole indices (ia', ib), [0, rb) of index ib
  int count = 0;
  int64_t pos = 0;  // flat position of the next box relative to the original a
  int64_t base = 0;
  for (int j = 0; j < k; ++j) base += fixed[j] * inner[j];
  const int64_t a_abs = base + ia * inner[k] + ra;

  auto emit = [&](const int64_t* pin, int upto, int dim, int64_t lo, int64_t hi) {
    // dimensions < upto pinned to pin[], dimension `dim` (== upto) in [lo, hi), deeper ones whole
    if (out) {
      LocalBox& bx = out[count];
      for (int j = 0; j < upto; ++j) {
        bx.off[j] = pin[j];
        bx.len[j] = 1;
      }
      bx.off[dim] = lo;
      bx.len[dim] = hi - lo;
      for (int j = dim + 1; j < n; ++j) {
        bx.off[j] = 0;
        bx.len[j] = len[j];
      }
      for (int j = n; j < kDims; ++j) {
        bx.off[j] = 0;
        bx.len[j] = 1;
      }
      bx.flat_start = a_abs + pos;
    }
    pos += (hi - lo) * inner[dim];
    ++count;
  };

  int64_t mid_lo = ia;
  if (ra != 0) {
    // digits of ra over dimensions k+1..n-1
    int64_t dig[kDims];
    int64_t r = ra;
    int deepest = k;
    for (int j = k + 1; j < n; ++j) {
      dig[j] = r / inner[j];
      r -= dig[j] * inner[j];
      if (dig[j] != 0) deepest = j;
    }
    fixed[k] = ia;
    for (int j = k + 1; j < deepest; ++j) fixed[j] = dig[j];
    emit(fixed, deepest, deepest, dig[deepest], len[deepest]);
    for (int j = deepest - 1; j > k; --j)
      if (dig[j] + 1 < len[j]) emit(fixed, j, j, dig[j] + 1, len[j]);
    mid_lo = ia + 1;
  }
  if (mid_lo < ib) emit(fixed, k, k, mid_lo, ib);
  if (rb != 0) {
    int64_t dig[kDims];
    int64_t r = rb;
    int deepest = k;
    for (int j = k + 1; j < n; ++j) {
      dig[j] = r / inner[j];
      r -= dig[j] * inner[j];
      if (dig[j] != 0) deepest = j;
    }
    fixed[k] = ib;
    for (int j = k + 1; j <= deepest; ++j) {
      if (dig[j] != 0) emit(fixed, j, j, 0, dig[j]);
      fixed[j] = dig[j];
    }
  }
  return count;
}

}  // namespace bcp
