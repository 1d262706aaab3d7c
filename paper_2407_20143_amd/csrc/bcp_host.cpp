// The part of the C-ABI that needs no GPU: cutting flat buffers at tensor boundaries (a1), the host
// mirror of the decomposer (a2), checks of shard metadata, the save-side Worst-Fit deduplication, and
// the error text.  Plain C++17 without HIP headers: it is compiled into libbcp.so, and on its own with
// g++ and sanitizers for the CPU tests.
#include <algorithm>
#include <cstring>
#include <new>
#include <numeric>
#include <string>
#include <unordered_map>
#include <vector>

#include "bcp_host.h"
#include "bcp_validate.h"

namespace bcp {

namespace {
thread_local std::string g_error;
}  // namespace

void set_error(const std::string& msg) { g_error = msg; }

// No exception leaves the library: every entry point that can allocate on the host is a function
// try block that ends here.
bcp_status on_exception(const char* who) noexcept {
  try {
    throw;
  } catch (const std::bad_alloc&) {
    try {
      set_error(std::string(who) + ": out of host memory");
    } catch (...) {
    }
    return BCP_ERR_OOM;
  } catch (const std::exception& e) {
    try {
      set_error(std::string(who) + ": " + e.what());
    } catch (...) {
    }
    return BCP_ERR_INVALID_ARG;
  } catch (...) {
    return BCP_ERR_INVALID_ARG;
  }
}

// status and text for an error of the record checks (DevErr code; the record's index on its side)
bcp_status record_error(unsigned code, bool is_saved, int64_t index) {
  const std::string who = std::string(is_saved ? "saved" : "target") + " record " + std::to_string(index);
  switch (code) {
    case kErrInvalid: set_error(who + ": invalid field (ndim, itemsize, fqn_id, buf, offsets, flat range or strides)"); return BCP_ERR_INVALID_ARG;
    case kErrTooManyDims: set_error(who + ": ndim exceeds BCP_MAX_DIMS"); return BCP_ERR_TOO_MANY_DIMS;
    case kErrBounds: set_error(who + ": box or flat range outside the tensor"); return BCP_ERR_OUT_OF_BOUNDS;
    case kErrShape: set_error(who + ": ndim / global shape differs from other records of its FQN"); return BCP_ERR_SHAPE_MISMATCH;
    case kErrDtype: set_error(who + ": itemsize differs from other records of its FQN"); return BCP_ERR_DTYPE_MISMATCH;
    case kErrOverlap: set_error(who + ": saved shards overlap (an element has two savers)"); return BCP_ERR_SAVED_OVERLAP;
    case kErrUncovered: set_error(who + ": no saved shard holds some of its elements"); return BCP_ERR_UNCOVERED;
  }
  set_error("unknown record error");
  return BCP_ERR_INVALID_ARG;
}

}  // namespace bcp

using namespace bcp;

extern "C" {

const char* bcp_last_error(void) { return g_error.c_str(); }

const char* bcp_status_name(bcp_status s) {
  switch (s) {
    case BCP_OK: return "BCP_OK";
    case BCP_ERR_INVALID_ARG: return "BCP_ERR_INVALID_ARG";
    case BCP_ERR_SHAPE_MISMATCH: return "BCP_ERR_SHAPE_MISMATCH";
    case BCP_ERR_DTYPE_MISMATCH: return "BCP_ERR_DTYPE_MISMATCH";
    case BCP_ERR_OUT_OF_BOUNDS: return "BCP_ERR_OUT_OF_BOUNDS";
    case BCP_ERR_SAVED_OVERLAP: return "BCP_ERR_SAVED_OVERLAP";
    case BCP_ERR_UNCOVERED: return "BCP_ERR_UNCOVERED";
    case BCP_ERR_TOO_MANY_DIMS: return "BCP_ERR_TOO_MANY_DIMS";
    case BCP_ERR_OOM: return "BCP_ERR_OOM";
    case BCP_ERR_HIP: return "BCP_ERR_HIP";
    case BCP_ERR_NO_DEVICE: return "BCP_ERR_NO_DEVICE";
  }
  return "BCP_ERR_UNKNOWN";
}

int32_t bcp_abi_version(void) { return 2; }
int64_t bcp_sizeof_shard_meta(void) { return (int64_t)sizeof(bcp_shard_meta); }

// ---- a1: flat slice of a concatenation -> per-tensor records ----------------------------------
bcp_status bcp_meta_from_flat_slice(const bcp_shard_meta* params, int64_t n_params, int64_t A, int64_t B,
                                    int32_t buf, int64_t byte_offset, bcp_shard_meta* out, int64_t* inout_n) try {
  if (!inout_n || n_params < 0 || (n_params > 0 && !params) || A < 0 || B < A || buf < 0 || byte_offset < 0) {
    set_error("bcp_meta_from_flat_slice: bad argument");
    return BCP_ERR_INVALID_ARG;
  }
  const int64_t room = *inout_n;
  int64_t written = 0, pos = 0;
  for (int64_t i = 0; i < n_params; ++i) {
    const bcp_shard_meta& p = params[i];
    if (p.ndim < 0 || p.ndim > BCP_MAX_DIMS) {
      set_error("bcp_meta_from_flat_slice: bad ndim in parameter " + std::to_string(i));
      return p.ndim < 0 ? BCP_ERR_INVALID_ARG : BCP_ERR_TOO_MANY_DIMS;
    }
    int64_t vol = 1;
    bool strided = false;
    for (int k = 0; k < p.ndim; ++k) {
      if (p.lengths[k] < 0) {
        set_error("bcp_meta_from_flat_slice: negative length");
        return BCP_ERR_INVALID_ARG;
      }
      vol *= p.lengths[k];
      strided |= p.strides[k] != 0;
    }
    if (strided || p.flat_begin != 0 || p.flat_end != vol || p.itemsize != params[0].itemsize) {
      set_error("bcp_meta_from_flat_slice: parameter " + std::to_string(i) +
                " must be a regular packed record of the common itemsize");
      return BCP_ERR_INVALID_ARG;
    }
    // the part of [A, B) inside this tensor's span [pos, pos + vol)
    const int64_t lo = std::max(A, pos), hi = std::min(B, pos + vol);
    if (lo < hi) {
      if (out && written < room) {
        bcp_shard_meta r = p;
        r.flat_begin = lo - pos;
        r.flat_end = hi - pos;
        r.buf = buf;
        r.byte_offset = byte_offset + (int64_t)p.itemsize * (lo - A);
        out[written] = r;
      }
      ++written;
    }
    pos += vol;
  }
  if (B > pos) {
    set_error("bcp_meta_from_flat_slice: slice ends beyond the concatenation");
    return BCP_ERR_OUT_OF_BOUNDS;
  }
  *inout_n = written;
  if (written > room || (written > 0 && !out)) {
    set_error("bcp_meta_from_flat_slice: output array too small");
    return BCP_ERR_INVALID_ARG;
  }
  return BCP_OK;
} catch (...) {
  return on_exception("bcp_meta_from_flat_slice");
}

// ---- a2: host mirror of the device decomposer ---------------------------------------------------
bcp_status bcp_decompose(const bcp_shard_meta* rec, bcp_shard_meta* out_boxes, int64_t* inout_n) try {
  if (!rec || !inout_n) {
    set_error("bcp_decompose: null argument");
    return BCP_ERR_INVALID_ARG;
  }
  if (rec->ndim < 0 || rec->ndim > BCP_MAX_DIMS) {
    set_error("bcp_decompose: bad ndim");
    return rec->ndim < 0 ? BCP_ERR_INVALID_ARG : BCP_ERR_TOO_MANY_DIMS;
  }
  int64_t len[kDims];
  int n = rec->ndim;
  int64_t vol = 1;
  for (int k = 0; k < n; ++k) {
    if (rec->lengths[k] < 0) {
      set_error("bcp_decompose: negative length");
      return BCP_ERR_INVALID_ARG;
    }
    len[k] = rec->lengths[k];
    vol *= len[k];
    if (rec->strides[k] != 0) {
      set_error("bcp_decompose: strided records are regular by definition");
      return BCP_ERR_INVALID_ARG;
    }
  }
  if (n == 0) {
    len[0] = 1;
    n = 1;
  }
  if (rec->flat_begin < 0 || rec->flat_end < rec->flat_begin || rec->flat_end > vol) {
    set_error("bcp_decompose: flat range outside the box");
    return BCP_ERR_OUT_OF_BOUNDS;
  }
  LocalBox lb[kMaxBoxesPerRecord];
  const int nb = decompose_flat_range(len, n, rec->flat_begin, rec->flat_end, lb);
  const int64_t room = *inout_n;
  *inout_n = nb;
  if (nb > room || (nb > 0 && !out_boxes)) {
    set_error("bcp_decompose: output array too small");
    return BCP_ERR_INVALID_ARG;
  }
  for (int j = 0; j < nb; ++j) {
    bcp_shard_meta b = *rec;
    int64_t v = 1;
    for (int k = 0; k < rec->ndim; ++k) {
      b.offsets[k] = rec->offsets[k] + lb[j].off[k];
      b.lengths[k] = lb[j].len[k];
      v *= lb[j].len[k];
    }
    b.flat_begin = 0;
    b.flat_end = v;
    b.byte_offset = rec->byte_offset + (int64_t)rec->itemsize * (lb[j].flat_start - rec->flat_begin);
    out_boxes[j] = b;
  }
  return BCP_OK;
} catch (...) {
  return on_exception("bcp_decompose");
}

// ---- save-side deduplication (Worst-Fit) ----------------------------------------------------------
namespace {
struct ShardIdentity {
  const bcp_shard_meta* r;
  bool operator==(const ShardIdentity& o) const {
    const bcp_shard_meta &a = *r, &b = *o.r;
    if (a.fqn_id != b.fqn_id || a.ndim != b.ndim || a.itemsize != b.itemsize || a.flat_begin != b.flat_begin ||
        a.flat_end != b.flat_end)
      return false;
    for (int k = 0; k < a.ndim; ++k)
      if (a.offsets[k] != b.offsets[k] || a.lengths[k] != b.lengths[k]) return false;
    return true;
  }
};
struct ShardIdentityHash {
  size_t operator()(const ShardIdentity& s) const {
    const bcp_shard_meta& a = *s.r;
    uint64_t h = 0x9e3779b97f4a7c15ull ^ (uint64_t)a.fqn_id;
    auto mix = [&](uint64_t v) { h = (h ^ v) * 0x100000001b3ull; h ^= h >> 29; };
    mix((uint64_t)a.flat_begin);
    mix((uint64_t)a.flat_end);
    for (int k = 0; k < a.ndim; ++k) {
      mix((uint64_t)a.offsets[k]);
      mix((uint64_t)a.lengths[k]);
    }
    return (size_t)h;
  }
};
}  // namespace

bcp_status bcp_dedup_worst_fit(const bcp_shard_meta* recs, const int32_t* rank_of, int64_t n, int32_t n_ranks,
                               uint8_t* keep, int64_t* load) try {
  if (n < 0 || n_ranks <= 0 || (n > 0 && (!recs || !rank_of || !keep))) {
    set_error("bcp_dedup_worst_fit: bad argument");
    return BCP_ERR_INVALID_ARG;
  }
  std::unordered_map<ShardIdentity, int64_t, ShardIdentityHash> group_of;  // identity -> group index
  std::vector<std::vector<int64_t>> groups;                                // in order of first appearance
  for (int64_t i = 0; i < n; ++i) {
    if (recs[i].ndim < 0 || recs[i].ndim > BCP_MAX_DIMS || rank_of[i] < 0 || rank_of[i] >= n_ranks ||
        recs[i].flat_end < recs[i].flat_begin || recs[i].itemsize <= 0) {
      set_error("bcp_dedup_worst_fit: bad record " + std::to_string(i));
      return BCP_ERR_INVALID_ARG;
    }
    auto it = group_of.find(ShardIdentity{&recs[i]});
    if (it == group_of.end()) {
      group_of.emplace(ShardIdentity{&recs[i]}, (int64_t)groups.size());
      groups.emplace_back(1, i);
    } else {
      groups[(size_t)it->second].push_back(i);
    }
  }
  std::vector<int64_t> assigned((size_t)n_ranks, 0);
  for (int64_t i = 0; i < n; ++i) keep[i] = 0;
  for (const std::vector<int64_t>& g : groups) {
    int64_t best = g[0];
    for (int64_t i : g) {
      const int64_t li = assigned[(size_t)rank_of[i]], lb = assigned[(size_t)rank_of[best]];
      if (li < lb || (li == lb && rank_of[i] < rank_of[best])) best = i;
    }
    keep[best] = 1;
    assigned[(size_t)rank_of[best]] += (recs[best].flat_end - recs[best].flat_begin) * (int64_t)recs[best].itemsize;
  }
  if (load)
    for (int32_t r = 0; r < n_ranks; ++r) load[r] = assigned[(size_t)r];
  return BCP_OK;
} catch (...) {
  return on_exception("bcp_dedup_worst_fit");
}

// ---- metadata checks without a GPU -------------------------------------------------------------------
namespace {
struct HostBox {
  int64_t fqn;
  int64_t off[kDims], len[kDims];
  int32_t rec, ndim;
};

void boxes_of(const bcp_shard_meta& r, int32_t rec, std::vector<HostBox>* out) {
  int64_t len[kDims];
  const int n = local_shape(r, len);
  LocalBox lb[kMaxBoxesPerRecord];
  const int nb = decompose_flat_range(len, n, r.flat_begin, r.flat_end, lb);
  for (int j = 0; j < nb; ++j) {
    HostBox b{};
    b.fqn = r.fqn_id;
    b.rec = rec;
    b.ndim = n;
    for (int k = 0; k < kDims; ++k) {
      b.off[k] = (k < r.ndim ? r.offsets[k] : 0) + (k < n ? lb[j].off[k] : 0);
      b.len[k] = k < n ? lb[j].len[k] : 1;
    }
    out->push_back(b);
  }
}

// volume of the intersection of two boxes of equal rank (0: disjoint)
int64_t overlap_volume(const HostBox& a, const HostBox& b) {
  int64_t v = 1;
  for (int k = 0; k < a.ndim; ++k) {
    const int64_t lo = std::max(a.off[k], b.off[k]);
    const int64_t hi = std::min(a.off[k] + a.len[k], b.off[k] + b.len[k]);
    if (lo >= hi) return 0;
    v *= hi - lo;
  }
  return v;
}

bcp_status status_of(unsigned long long key, int64_t n_saved) {
  const unsigned code = (unsigned)(key & 0xff);
  const int64_t rec = (int64_t)(key >> 8);
  const bool is_saved = rec < n_saved;
  return record_error(code, is_saved, is_saved ? rec : rec - n_saved);
}
}  // namespace

bcp_status bcp_validate_meta(const bcp_shard_meta* saved, int64_t n_saved, const bcp_shard_meta* target,
                             int64_t n_target, uint32_t flags) try {
  if (n_saved < 0 || n_target < 0 || (n_saved > 0 && !saved) || (n_target > 0 && !target)) {
    set_error("bcp_validate_meta: null metadata array or negative count");
    return BCP_ERR_INVALID_ARG;
  }
  if (flags & ~(BCP_ALLOW_UNCOVERED | BCP_SKIP_OVERLAP_CHECK | BCP_ORDER_BY_SOURCE | BCP_CONVERT_F32_TO_BF16)) {
    set_error("bcp_validate_meta: unknown flag (BCP_META_ON_DEVICE has no meaning here: the records are read on the host)");
    return BCP_ERR_INVALID_ARG;
  }
  if (n_target == 0) return BCP_OK;
  const bool convert = (flags & BCP_CONVERT_F32_TO_BF16) != 0;
  constexpr unsigned long long kNone = ~0ull;
  unsigned long long key = kNone;  // as in the planner: the smallest (record index, code) of a phase is reported
  auto report = [&](int64_t record, unsigned code) { key = std::min(key, ((unsigned long long)record << 8) | code); };
  auto rec_at = [&](int64_t i) -> const bcp_shard_meta& { return i < n_saved ? saved[i] : target[i - n_saved]; };

  // 1. every record on its own
  for (int64_t i = 0; i < n_saved + n_target; ++i)
    if (const unsigned code = validate_record(rec_at(i))) report(i, code);
  if (key != kNone) return status_of(key, n_saved);

  // 2. the records of one tensor against each other: the saved boxes of an FQN in (FQN, box) order
  std::vector<HostBox> sb, tb;
  for (int64_t i = 0; i < n_saved; ++i) boxes_of(saved[i], (int32_t)i, &sb);
  for (int64_t i = 0; i < n_target; ++i) boxes_of(target[i], (int32_t)i, &tb);
  std::vector<size_t> order(sb.size());
  std::iota(order.begin(), order.end(), (size_t)0);
  std::stable_sort(order.begin(), order.end(), [&](size_t a, size_t b) { return sb[a].fqn < sb[b].fqn; });
  std::unordered_map<int64_t, std::pair<size_t, size_t>> run_of;  // fqn -> [first, last) in `order`
  for (size_t i = 0; i < order.size();) {
    size_t j = i;
    while (j < order.size() && sb[order[j]].fqn == sb[order[i]].fqn) ++j;
    run_of[sb[order[i]].fqn] = {i, j};
    i = j;
  }
  for (size_t i = 0; i < order.size(); ++i) {
    const HostBox& a = sb[order[i]];
    if (i + 1 < order.size() && sb[order[i + 1]].fqn == a.fqn) {
      const HostBox& nx = sb[order[i + 1]];
      if (const unsigned code = same_tensor(saved[a.rec], saved[nx.rec])) {
        report(nx.rec, code);
        continue;
      }
    }
    if (flags & BCP_SKIP_OVERLAP_CHECK) continue;
    for (size_t j = i + 1; j < order.size() && sb[order[j]].fqn == a.fqn; ++j) {
      const HostBox& b = sb[order[j]];
      if (a.ndim == b.ndim && overlap_volume(a, b) > 0) {
        report(std::max(a.rec, b.rec), kErrOverlap);
        break;
      }
    }
  }
  for (const HostBox& t : tb) {
    auto it = run_of.find(t.fqn);
    if (it == run_of.end()) continue;
    const HostBox& first = sb[order[it->second.first]];
    if (const unsigned code = same_tensor(saved[first.rec], target[t.rec], convert)) report(n_saved + t.rec, code);
  }
  if (key != kNone) return status_of(key, n_saved);

  // 3. coverage: the saved boxes are pairwise disjoint here, so the volumes of their intersections
  //    with a target record's boxes add up to the record's element count exactly when it is covered
  std::vector<unsigned long long> cov((size_t)n_target, 0);
  for (const HostBox& t : tb) {
    auto it = run_of.find(t.fqn);
    if (it == run_of.end()) continue;
    for (size_t i = it->second.first; i < it->second.second; ++i) {
      const HostBox& s = sb[order[i]];
      if (s.ndim == t.ndim) cov[(size_t)t.rec] += (unsigned long long)overlap_volume(s, t);
    }
  }
  for (int64_t i = 0; i < n_target; ++i) {
    const unsigned long long want = (unsigned long long)(target[i].flat_end - target[i].flat_begin);
    if (cov[(size_t)i] > want) report(n_saved + i, kErrOverlap);
    else if (cov[(size_t)i] < want && !(flags & BCP_ALLOW_UNCOVERED)) report(n_saved + i, kErrUncovered);
  }
  if (key != kNone) return status_of(key, n_saved);
  return BCP_OK;
} catch (...) {
  return on_exception("bcp_validate_meta");
}

}  // extern "C"
