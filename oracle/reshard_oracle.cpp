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
// Dtype-converting load (Sec. 2.2: evaluation jobs load model states only, so fp32 master weights
// are read as bf16): with `convert` set, a tensor saved with 4-byte elements and asked for with 2-byte
// elements is narrowed element by element, binary32 -> bfloat16, round to nearest, ties to even,
// written out below from the IEEE 754 definition (the two neighbouring bfloat16 values are decoded
// and compared in fp64, where the differences are exact).
//
// Parity status: pinned (tests/test_oracle_pins.py: library-slicing closed form, the paper's
// (3,2) worked example, reassembly / round-trip / exactly-once invariants, brute force).
// The narrowing: tests/test_oracle_convert.py (hand values in tests/golden/bf16_rounding.txt, the
// library cast on every upper half x chosen lower halves and on random bits, closed form through the
// whole transform).
// The region list of a plan has no counterpart here: many region lists are correct.
#include <algorithm>
#include <atomic>
#include <cmath>
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

// ---- binary32 -> bfloat16, IEEE 754 roundTiesToEven ------------------------------------------------
// bfloat16 is the upper half of the binary32 encoding: 1 sign bit, 8 exponent bits (bias 127), 7
// fraction bits.  Magnitudes only below; the sign is carried over.
//
// value of a binary32 magnitude pattern (31 bits), finite
double f32_magnitude(uint32_t m) {
  const int exp = (int)(m >> 23);
  const double frac = (double)(m & 0x7fffffu);
  if (exp == 0) return std::ldexp(frac, -149);               // subnormal: frac * 2^-149
  return std::ldexp(8388608.0 + frac, exp - 150);            // (2^23 + frac) * 2^(exp - 127 - 23)
}
// value of a bfloat16 magnitude pattern (15 bits).  The pattern of infinity (exponent field 255,
// fraction 0) is given the value its binade would have, 2^128: rounding to nearest goes to infinity
// exactly when the value is at least half an ulp beyond the largest finite number, i.e. nearer to
// 2^128 than to it (IEEE 754-2019, 4.3.1).
double bf16_magnitude(uint32_t m) {
  const int exp = (int)(m >> 7);
  const double frac = (double)(m & 0x7fu);
  if (exp == 0) return std::ldexp(frac, -133);               // subnormal: frac * 2^-126 * 2^-7
  return std::ldexp(128.0 + frac, exp - 134);                // (2^7 + frac) * 2^(exp - 127 - 7)
}

uint16_t f32_to_bf16(uint32_t bits) {
  const uint32_t sign = bits >> 31, mag = bits & 0x7fffffffu;
  if (mag > 0x7f800000u) {
    // NaN: stays NaN.  Sign and the upper seven fraction bits are kept and the result is quiet
    // (IEEE 754-2019, 6.2.3: payload preserved as far as the narrower format holds it).
    return (uint16_t)((sign << 15) | 0x7f80u | ((mag >> 16) & 0x7fu) | 0x40u);
  }
  if (mag == 0x7f800000u) return (uint16_t)((sign << 15) | 0x7f80u);  // infinity
  const uint32_t below = mag >> 16;      // the bfloat16 neighbour towards zero (truncation) ...
  const uint32_t above = below + 1;      // ... and the next one away from zero
  const double x = f32_magnitude(mag), a = bf16_magnitude(below), b = bf16_magnitude(above);
  const double down = x - a, up = b - x;  // exact in fp64
  uint32_t pick;
  if (down < up) pick = below;
  else if (up < down) pick = above;
  else pick = (below & 1u) == 0 ? below : above;  // tie: the neighbour whose last fraction bit is 0
  return (uint16_t)((sign << 15) | pick);
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
  int convert;  // 0: element sizes must agree; 1: 4-byte saved elements -> 2-byte target elements as f32 -> bf16
  Error err;
};

void do_fqn(Job& job, int64_t fqn, const std::vector<Ref>& trefs) {
  auto it = job.saved.by_fqn.find(fqn);
  // shape / dtype agreement over every part that names this FQN
  const orc_part& t0 = job.target.parts[trefs[0].part];
  const int n = t0.ndim;
  const int et = job.target.shards[trefs[0].shard].itemsize;  // element size asked for
  int e = et;                                                 // element size saved
  if (it != job.saved.by_fqn.end() && !it->second.empty()) {
    const int es = job.saved.shards[it->second[0].shard].itemsize;
    if (job.convert == 1 && es == 4 && et == 2) e = es;
  }
  auto agrees = [&](const Side& s, const Ref& r, int esize) {
    const orc_part& p = s.parts[r.part];
    if (p.ndim != n || s.shards[r.shard].itemsize != esize) return false;
    for (int d = 0; d < n; ++d)
      if (p.global_shape[d] != t0.global_shape[d]) return false;
    return true;
  };
  for (const Ref& r : trefs)
    if (!agrees(job.target, r, et)) return job.err.set(ORC_MISMATCH, "target shards disagree on fqn " + std::to_string(fqn));
  if (it != job.saved.by_fqn.end())
    for (const Ref& r : it->second)
      if (!agrees(job.saved, r, e)) return job.err.set(ORC_MISMATCH, "saved/target disagree on fqn " + std::to_string(fqn));

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
      if (b < 0 || b + et > job.dst_bytes[sh.buf])
        return job.err.set(ORC_BOUNDS, "target shard " + std::to_string(r.shard) + " writes outside its buffer");
      if (e == et) {
        std::memcpy(job.dst[sh.buf] + b, &G[(size_t)gi * e], e);
      } else {  // 4-byte saved element, 2-byte target element: narrow
        uint32_t wide;
        std::memcpy(&wide, &G[(size_t)gi * e], 4);
        const uint16_t narrow = f32_to_bf16(wide);
        std::memcpy(job.dst[sh.buf] + b, &narrow, 2);
      }
      if (job.dst_written) {
        uint8_t* w = job.dst_written[sh.buf] + b;
        for (int k = 0; k < et; ++k)
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
// convert: 0, or 1 to narrow tensors saved with 4-byte elements and asked for with 2-byte elements as
// binary32 -> bfloat16 (other tensors are moved as they are).
// Threads work on disjoint FQNs; dst_written increments can only collide if two FQNs share a
// destination byte, which is itself a layout bug the counters then may under-report.
int orc_reshard(const orc_part* sparts, const orc_shard* saved, int64_t n_saved,
                const uint8_t* const* src, const int64_t* src_bytes,
                const orc_part* tparts, const orc_shard* target, int64_t n_target,
                uint8_t* const* dst, const int64_t* dst_bytes, uint8_t* const* dst_written,
                int allow_uncovered, int n_threads, const int64_t* only_fqns, int64_t n_only,
                int convert, char* err, int err_len) {
  Job job;
  job.saved = Side{sparts, saved, n_saved, {}};
  job.target = Side{tparts, target, n_target, {}};
  job.src = src;
  job.src_bytes = src_bytes;
  job.dst = dst;
  job.dst_bytes = dst_bytes;
  job.dst_written = dst_written;
  job.allow_uncovered = allow_uncovered != 0;
  job.convert = convert;
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

// the narrowing alone, for its pins: out[i] = bfloat16 pattern of the binary32 pattern in[i]
void orc_f32_to_bf16(const uint32_t* in, uint16_t* out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = f32_to_bf16(in[i]);
}

int orc_max_dims(void) { return kMaxDims; }

}  // extern "C"
