// CPU oracle for load-time checkpoint resharding.  TEST INFRASTRUCTURE ONLY: nothing on the
// product path may include, link or call this file.  It shares no code with the HIP library.
//
// What it computes is the plain definition of the transform, not the method:
//  * a tensor is named by its FQN and has a global shape; a stored shard holds the box
//    (nD offsets, nD lengths) along the axes of that global shape
//    (Sec. 3.2 "Decoupled Checkpoint Representation", ShardMeta);
//  * an irregular (ZeRO) shard is a slice of the concatenation of row-major-flattened boxes
//    (Sec. 3.2 "Decomposing irregular tensors"; Appendix A: TP-local shards are flattened and
//    merged before being cut by the DP degree);
//  * loading with a new layout gives every target element the saved element that has the same
//    FQN and the same global index (Sec. 3.3 Step 2, "matching segments").
// So, per FQN: scatter every saved element to G[global row-major index], then gather every
// target element from G.  Every element goes through its global index; there is no box
// intersection and no decomposition of flat ranges here.
//
// Parity status: pinned (tests/test_oracle_pins.py: library-slicing closed form, the paper's
// (3,2) worked example, reassembly / round-trip / exactly-once invariants, brute force).
// The region list of a plan has no counterpart here: many region lists are correct.
#include <algorithm>
#include <atomic>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

constexpr int kMaxDims = 8;

extern "C" {
struct orc_part {
  int64_t fqn;
  int32_t ndim;
  int32_t pad_;
  int64_t global_shape[kMaxDims];
  int64_t offsets[kMaxDims];
  int64_t lengths[kMaxDims];
};
struct orc_shard {
  int64_t part_begin;   // parts [part_begin, part_begin + part_count) of the part array, concatenated
  int64_t part_count;
  int64_t flat_begin;   // slice of that concatenation held by the shard
  int64_t flat_end;
  int64_t byte_offset;  // where the first stored element sits in buffer `buf`
  int64_t strides[kMaxDims];  // element strides when has_strides (single part, whole box)
  int32_t itemsize;
  int32_t buf;
  int32_t has_strides;
  int32_t pad_;
};
}

namespace {

enum : int {
  ORC_OK = 0,
  ORC_INVALID = 1,
  ORC_SAVED_OVERLAP = 2,
  ORC_UNCOVERED = 3,
  ORC_MISMATCH = 4,
  ORC_BOUNDS = 5,
};

int64_t volume(const int64_t* len, int n) {
  int64_t v = 1;
  for (int k = 0; k < n; ++k) v *= len[k];
  return v;
}

// row-major flat index -> coordinates
void unravel(int64_t flat, const int64_t* shape, int n, int64_t* out) {
  for (int k = n - 1; k >= 0; --k) {
    out[k] = flat % shape[k];
    flat /= shape[k];
  }
}

// coordinates -> row-major flat index
int64_t ravel(const int64_t* x, const int64_t* shape, int n) {
  int64_t f = 0;
  for (int k = 0; k < n; ++k) f = f * shape[k] + x[k];
  return f;
}

struct Ref {  // one part of one shard, with the position of its first element in the concatenation
  int64_t shard;
  int64_t part;
  int64_t concat_pos;
};

struct Side {
  const orc_part* parts;
  const orc_shard* shards;
  int64_t n;
  std::map<int64_t, std::vector<Ref>> by_fqn;
};

struct Error {
  std::mutex mu;
  int code = ORC_OK;
  std::string msg;
  void set(int c, const std::string& m) {
    std::lock_guard<std::mutex> g(mu);
    if (code == ORC_OK) {
      code = c;
      msg = m;
    }
  }
  bool failed() {
    std::lock_guard<std::mutex> g(mu);
    return code != ORC_OK;
  }
};

bool index_side(Side& s, Error& err) {
  for (int64_t i = 0; i < s.n; ++i) {
    const orc_shard& sh = s.shards[i];
    if (sh.itemsize <= 0 || sh.part_count < 0 || sh.flat_begin < 0 || sh.flat_end < sh.flat_begin) {
      err.set(ORC_INVALID, "bad shard record " + std::to_string(i));
      return false;
    }
    if (sh.has_strides && (sh.part_count != 1)) {
      err.set(ORC_INVALID, "strided shard must have exactly one part");
      return false;
    }
    int64_t pos = 0;
    for (int64_t k = 0; k < sh.part_count; ++k) {
      const orc_part& p = s.parts[sh.part_begin + k];
      if (p.ndim < 0 || p.ndim > kMaxDims) {
        err.set(ORC_INVALID, "bad ndim");
        return false;
      }
      for (int d = 0; d < p.ndim; ++d) {
        if (p.global_shape[d] < 0 || p.offsets[d] < 0 || p.lengths[d] < 0 ||
            p.offsets[d] + p.lengths[d] > p.global_shape[d]) {
          err.set(ORC_BOUNDS, "box outside global shape, shard " + std::to_string(i));
          return false;
        }
      }
      s.by_fqn[p.fqn].push_back(Ref{i, sh.part_begin + k, pos});
      pos += volume(p.lengths, p.ndim);
    }
    if (sh.flat_end > pos) {
      err.set(ORC_BOUNDS, "flat range beyond the concatenation, shard " + std::to_string(i));
      return false;
    }
    if (sh.has_strides && !(sh.flat_begin == 0 && sh.flat_end == pos)) {
      err.set(ORC_INVALID, "strided shard must hold its whole box");
      return false;
    }
  }
  return true;
}

// byte position, inside its buffer, of the stored element that is element `local` (row-major)
// of part `p` and element `concat_index` of the concatenation
int64_t stored_byte(const orc_shard& sh, const orc_part& p, int64_t concat_index, const int64_t* y) {
  if (!sh.has_strides) return sh.byte_offset + (int64_t)sh.itemsize * (concat_index - sh.flat_begin);
  int64_t e = 0;
  for (int d = 0; d < p.ndim; ++d) e += y[d] * sh.strides[d];
  return sh.byte_offset + (int64_t)sh.itemsize * e;
}

struct Job {
  Side saved, target;
  const uint8_t* const* src;
  const int64_t* src_bytes;
  uint8_t* const* dst;
  const int64_t* dst_bytes;
  uint8_t* const* dst_written;  // optional per-byte write counters (saturating), may be null
  bool allow_uncovered;
  Error err;
};

void do_fqn(Job& job, int64_t fqn, const std::vector<Ref>& trefs) {
  auto it = job.saved.by_fqn.find(fqn);
  // shape / dtype agreement over every part that names this FQN
  const orc_part& t0 = job.target.parts[trefs[0].part];
  const int n = t0.ndim;
  const int e = job.target.shards[trefs[0].shard].itemsize;
  auto agrees = [&](const Side& s, const Ref& r) {
    const orc_part& p = s.parts[r.part];
    if (p.ndim != n || s.shards[r.shard].itemsize != e) return false;
    for (int d = 0; d < n; ++d)
      if (p.global_shape[d] != t0.global_shape[d]) return false;
    return true;
  };
  for (const Ref& r : trefs)
    if (!agrees(job.target, r)) return job.err.set(ORC_MISMATCH, "target shards disagree on fqn " + std::to_string(fqn));
  if (it != job.saved.by_fqn.end())
    for (const Ref& r : it->second)
      if (!agrees(job.saved, r)) return job.err.set(ORC_MISMATCH, "saved/target disagree on fqn " + std::to_string(fqn));

  const int64_t gvol = volume(t0.global_shape, n);
  std::vector<uint8_t> G((size_t)gvol * e);
  std::vector<uint8_t> cnt((size_t)gvol, 0);
  int64_t y[kMaxDims], x[kMaxDims];

  if (it != job.saved.by_fqn.end()) {
    for (const Ref& r : it->second) {
      const orc_shard& sh = job.saved.shards[r.shard];
      const orc_part& p = job.saved.parts[r.part];
      const int64_t pvol = volume(p.lengths, n);
      // only the elements of this part that lie inside the shard's slice of the concatenation
      const int64_t first = std::max<int64_t>(sh.flat_begin - r.concat_pos, 0);
      const int64_t last = std::min<int64_t>(sh.flat_end - r.concat_pos, pvol);
      for (int64_t local = first; local < last; ++local) {
        const int64_t ci = r.concat_pos + local;  // index in the concatenation
        unravel(local, p.lengths, n, y);
        for (int d = 0; d < n; ++d) x[d] = p.offsets[d] + y[d];
        const int64_t gi = ravel(x, t0.global_shape, n);
        const int64_t b = stored_byte(sh, p, ci, y);
        if (b < 0 || b + e > job.src_bytes[sh.buf])
          return job.err.set(ORC_BOUNDS, "saved shard " + std::to_string(r.shard) + " reads outside its blob");
        if (cnt[gi]) return job.err.set(ORC_SAVED_OVERLAP, "two saved shards hold one element of fqn " + std::to_string(fqn));
        cnt[gi] = 1;
        std::memcpy(&G[(size_t)gi * e], job.src[sh.buf] + b, e);
      }
    }
  }
  for (const Ref& r : trefs) {
    const orc_shard& sh = job.target.shards[r.shard];
    const orc_part& p = job.target.parts[r.part];
    const int64_t pvol = volume(p.lengths, n);
    const int64_t first = std::max<int64_t>(sh.flat_begin - r.concat_pos, 0);
    const int64_t last = std::min<int64_t>(sh.flat_end - r.concat_pos, pvol);
    for (int64_t local = first; local < last; ++local) {
      const int64_t ci = r.concat_pos + local;
      unravel(local, p.lengths, n, y);
      for (int d = 0; d < n; ++d) x[d] = p.offsets[d] + y[d];
      const int64_t gi = ravel(x, t0.global_shape, n);
      if (!cnt[gi]) {
        if (job.allow_uncovered) continue;
        return job.err.set(ORC_UNCOVERED, "no saved shard holds an element of fqn " + std::to_string(fqn) +
                                               " needed by target shard " + std::to_string(r.shard));
      }
      const int64_t b = stored_byte(sh, p, ci, y);
      if (b < 0 || b + e > job.dst_bytes[sh.buf])
        return job.err.set(ORC_BOUNDS, "target shard " + std::to_string(r.shard) + " writes outside its buffer");
      std::memcpy(job.dst[sh.buf] + b, &G[(size_t)gi * e], e);
      if (job.dst_written) {
        uint8_t* w = job.dst_written[sh.buf] + b;
        for (int k = 0; k < e; ++k)
          if (w[k] != 255) ++w[k];  // distinct FQNs never share bytes in a sane layout; tests check == 1
      }
    }
  }
}

}  // namespace

extern "C" {

// only_fqns (optional, n_only entries): produce only these tensors; the rest of dst is untouched.
// Reshard on the host.  src[i] / dst[i] are host byte buffers of src_bytes[i] / dst_bytes[i]
// bytes.  dst_written (optional): per-byte counters the caller zeroed, incremented for every
// byte written.  Returns ORC_OK or an error code and copies a message into err (if non-null).
// Threads work on disjoint FQNs; dst_written increments can only collide if two FQNs share a
// destination byte, which is itself a layout bug the counters then may under-report.
int orc_reshard(const orc_part* sparts, const orc_shard* saved, int64_t n_saved,
                const uint8_t* const* src, const int64_t* src_bytes,
                const orc_part* tparts, const orc_shard* target, int64_t n_target,
                uint8_t* const* dst, const int64_t* dst_bytes, uint8_t* const* dst_written,
                int allow_uncovered, int n_threads, const int64_t* only_fqns, int64_t n_only,
                char* err, int err_len) {
  Job job;
  job.saved = Side{sparts, saved, n_saved, {}};
  job.target = Side{tparts, target, n_target, {}};
  job.src = src;
  job.src_bytes = src_bytes;
  job.dst = dst;
  job.dst_bytes = dst_bytes;
  job.dst_written = dst_written;
  job.allow_uncovered = allow_uncovered != 0;
  if (index_side(job.saved, job.err) && index_side(job.target, job.err)) {
    std::vector<const std::pair<const int64_t, std::vector<Ref>>*> work;
    for (auto& kv : job.target.by_fqn) {
      bool take = n_only <= 0;  // optional filter: only these tensors are produced
      for (int64_t i = 0; i < n_only && !take; ++i) take = only_fqns[i] == kv.first;
      if (take) work.push_back(&kv);
    }
    std::atomic<size_t> next{0};
    auto worker = [&]() {
      for (;;) {
        size_t i = next.fetch_add(1);
        if (i >= work.size() || job.err.failed()) return;
        do_fqn(job, work[i]->first, work[i]->second);
      }
    };
    if (n_threads < 1) n_threads = 1;
    std::vector<std::thread> th;
    for (int t = 1; t < n_threads; ++t) th.emplace_back(worker);
    worker();
    for (auto& t : th) t.join();
  }
  if (err && err_len > 0) {
    std::snprintf(err, (size_t)err_len, "%s", job.err.msg.c_str());
  }
  return job.err.code;
}

int orc_max_dims(void) { return kMaxDims; }

}  // extern "C"
