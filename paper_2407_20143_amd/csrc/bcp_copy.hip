// The copy kernel: executes a plan's tiles.  Pure byte movement, HBM-bandwidth bound:
// every payload byte is read once and written once; there is no contraction, hence no MFMA.
//
// A tile is at most tile_bytes of payload: a segment of one long row, or a few whole short
// rows, decoded at plan time into one 64-byte descriptor.  One workgroup per tile.  Per tile the
// kernel picks, workgroup-uniformly and from the actual addresses, one of
//   * 16-byte vector path   -- bases, run length and pitches all 16-byte aligned;
//   * misaligned-run path   -- long runs whose source and destination disagree modulo 16 (ZeRO
//                              slice boundaries): peel to a 16-byte aligned destination, then
//                              unaligned 16-byte loads + aligned 16-byte stores;
//   * granule path          -- short runs: 8/4/2/1-byte elements, flat over rows x run;
//   * LDS-staged transpose  -- the source-contiguous and destination-contiguous dimensions
//                              differ (strided shards): both global sides stay coalesced.
// Scheduling: a persistent grid of (CU count x wg_per_cu) workgroups pops batch indices from an
// atomic queue; a batch is one big tile (whole workgroup) or a run of small tiles whose waves
// each take tiles of their own, so 100k tiny tensors do not cost one queue pop each.  Measured on
// MI355X, ONE 1024-thread workgroup per CU streaming 64 KiB tiles with non-temporal accesses
// sustains the highest copy bandwidth: fewer concurrent streams keep more DRAM pages open than a
// grid of one workgroup per tile.  The head descriptor of the next batch is fetched (scalar loads)
// while the current batch is being copied, and the buffer-pointer table is staged in LDS once per
// workgroup, so no dependent global load sits between two batches.
#include <algorithm>

#include "bcp_internal.h"

namespace bcp {
namespace {

constexpr int kMaxThreads = 1024;
constexpr int kLdsBytes = 128 * 129 * 8;  // transpose staging incl. one pad column; the planner picks the tile
                                          // edge per element size (256 for 1-2 bytes, 128 for 4-8, 64 for 16).
                                          // With one workgroup per CU, 129 of the CU's 160 KiB of LDS are free.
constexpr int kLdsPtrs = 1024;           // buffer pointers staged in LDS (more: read from global)
constexpr int kArgPtrs = kMaxKernargPtrs;  // buffer pointers passed as kernel arguments

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// Buffer pointers come out of a table in memory, so the compiler cannot tell their address space
// and would emit flat accesses; they are device (global) memory by contract.
#define BCP_GLOBAL __attribute__((address_space(1)))
typedef const char BCP_GLOBAL* gsrc_t;
typedef char BCP_GLOBAL* gdst_t;

template <int G> struct Granule;
template <> struct Granule<16> { typedef u32x4 type; };
template <> struct Granule<8> { typedef u32x2 type; };
template <> struct Granule<4> { typedef uint32_t type; };
template <> struct Granule<2> { typedef uint16_t type; };
template <> struct Granule<1> { typedef uint8_t type; };

// streaming accesses: the data is touched once, keep it out of the caches' way
template <int G>
__device__ __forceinline__ typename Granule<G>::type ld(gsrc_t p) {
  return __builtin_nontemporal_load((const typename Granule<G>::type BCP_GLOBAL*)p);
}
template <int G>
__device__ __forceinline__ void st(gdst_t p, typename Granule<G>::type v) {
  __builtin_nontemporal_store(v, (typename Granule<G>::type BCP_GLOBAL*)p);
}
template <int G>
__device__ __forceinline__ typename Granule<G>::type lds_ld(const char* p) {
  return *reinterpret_cast<const typename Granule<G>::type*>(p);
}
template <int G>
__device__ __forceinline__ void lds_st(char* p, typename Granule<G>::type v) {
  *reinterpret_cast<typename Granule<G>::type*>(p) = v;
}


typedef u32x4 u32x4_unaligned __attribute__((aligned(1)));
template <> struct Granule<-16> { typedef u32x4 type; };
template <>
__device__ __forceinline__ u32x4 ld<-16>(gsrc_t p) {
  return __builtin_nontemporal_load((const u32x4_unaligned BCP_GLOBAL*)p);
}
template <>
__device__ __forceinline__ void st<-16>(gdst_t p, u32x4 v) {
  __builtin_nontemporal_store(v, (u32x4_unaligned BCP_GLOBAL*)p);
}

// rows x run_g granules of |GG| bytes (GG == -16: 16-byte granules at unaligned addresses); rows at
// pitches sp / dp.  `nt` threads cooperate, `tid` in [0, nt).
template <int GG>
__device__ __forceinline__ void copy_rows(gsrc_t __restrict__ s, gdst_t __restrict__ d, uint32_t nrows,
                                          uint32_t run_g, int64_t sp, int64_t dp, uint32_t tid, uint32_t nt) {
  constexpr int G = GG < 0 ? -GG : GG;
  typedef typename Granule<GG>::type V;
  if (nrows == 1) {
    uint32_t i = tid;
    for (; i + 3 * nt < run_g; i += 4 * nt) {
      const V a = ld<GG>(s + (size_t)i * G);
      const V b = ld<GG>(s + (size_t)(i + nt) * G);
      const V c = ld<GG>(s + (size_t)(i + 2 * nt) * G);
      const V e = ld<GG>(s + (size_t)(i + 3 * nt) * G);
      st<GG>(d + (size_t)i * G, a);
      st<GG>(d + (size_t)(i + nt) * G, b);
      st<GG>(d + (size_t)(i + 2 * nt) * G, c);
      st<GG>(d + (size_t)(i + 3 * nt) * G, e);
    }
    for (; i < run_g; i += nt) st<GG>(d + (size_t)i * G, ld<GG>(s + (size_t)i * G));
    return;
  }
  const uint32_t total = nrows * run_g;
  // (row, col) of granule tid, then advance by nt granules per step without dividing again
  uint32_t row = tid / run_g, col = tid - row * run_g;
  const uint32_t drow = nt / run_g, dcol = nt - drow * run_g;
  uint32_t i = tid;
  for (; i + 3 * nt < total; i += 4 * nt) {
    V v[4];
    int64_t so[4], dof[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      so[u] = (int64_t)row * sp + (int64_t)col * G;
      dof[u] = (int64_t)row * dp + (int64_t)col * G;
      col += dcol;
      row += drow;
      if (col >= run_g) {
        col -= run_g;
        ++row;
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = ld<GG>(s + so[u]);
#pragma unroll
    for (int u = 0; u < 4; ++u) st<GG>(d + dof[u], v[u]);
  }
  for (; i < total; i += nt) {
    st<GG>(d + (int64_t)row * dp + (int64_t)col * G, ld<GG>(s + (int64_t)row * sp + (int64_t)col * G));
    col += dcol;
    row += drow;
    if (col >= run_g) {
      col -= run_g;
      ++row;
    }
  }
}

// one contiguous run whose two sides disagree modulo 16: byte head up to the destination's next
// 16-byte boundary, aligned 16-byte stores fed by unaligned 16-byte loads, byte tail.  nt >= 16.
__device__ __forceinline__ void copy_run_misaligned(gsrc_t __restrict__ s, gdst_t __restrict__ d, uint32_t run,
                                                    uint32_t tid, uint32_t nt) {
  uint32_t head = (uint32_t)(-(uintptr_t)d) & 15u;
  if (head > run) head = run;
  if (tid < head) d[tid] = s[tid];
  const uint32_t body = (run - head) >> 4;
  gsrc_t s2 = s + head;
  gdst_t d2 = d + head;
  uint32_t i = tid;
  for (; i + 3 * nt < body; i += 4 * nt) {
    const u32x4 a = ld<-16>(s2 + (size_t)i * 16);
    const u32x4 b = ld<-16>(s2 + (size_t)(i + nt) * 16);
    const u32x4 c = ld<-16>(s2 + (size_t)(i + 2 * nt) * 16);
    const u32x4 e = ld<-16>(s2 + (size_t)(i + 3 * nt) * 16);
    st<16>(d2 + (size_t)i * 16, a);
    st<16>(d2 + (size_t)(i + nt) * 16, b);
    st<16>(d2 + (size_t)(i + 2 * nt) * 16, c);
    st<16>(d2 + (size_t)(i + 3 * nt) * 16, e);
  }
  for (; i < body; i += nt) st<16>(d2 + (size_t)i * 16, ld<-16>(s2 + (size_t)i * 16));
  const uint32_t done = head + (body << 4);
  const uint32_t tail = run - done;
  if (tid < tail) d[done + tid] = s[done + tid];
}

template <int E>
__device__ __forceinline__ void transpose_tile(gsrc_t __restrict__ s, gdst_t __restrict__ d, uint32_t na,
                                               uint32_t nb, int64_t spb, int64_t dpa, uint32_t td, char* lds) {
  // source: element (a, b) at s + a*E + b*spb (contiguous along a)
  // destination: element (a, b) at d + b*E + a*dpa (contiguous along b)
  const uint32_t pitch = td + 1;  // LDS row pitch in elements
  const uint32_t x = threadIdx.x % td, y0 = threadIdx.x / td, step = blockDim.x / td;
  if (x < na)
    for (uint32_t b = y0; b < nb; b += step)
      lds_st<E>(lds + (size_t)(b * pitch + x) * E, ld<E>(s + (size_t)x * E + (int64_t)b * spb));
  __syncthreads();
  if (x < nb)
    for (uint32_t a = y0; a < na; a += step)
      st<E>(d + (size_t)x * E + (int64_t)a * dpa, lds_ld<E>(lds + (size_t)(x * pitch + a) * E));
  __syncthreads();  // the staging area is free again
}

template <int E>
__device__ __forceinline__ typename Granule<E>::type get_elem(const u32x4& v, uint32_t i) {
  if constexpr (E == 16) return v;
  else if constexpr (E == 8) return u32x2{v[2 * i], v[2 * i + 1]};
  else if constexpr (E == 4) return v[i];
  else if constexpr (E == 2) return (uint16_t)(v[i >> 1] >> (16 * (i & 1)));
  else return (uint8_t)(v[i >> 2] >> (8 * (i & 3)));
}
template <int E>
__device__ __forceinline__ void set_elem(u32x4& v, uint32_t i, typename Granule<E>::type x) {
  if constexpr (E == 16) v = x;
  else if constexpr (E == 8) { v[2 * i] = x[0]; v[2 * i + 1] = x[1]; }
  else if constexpr (E == 4) v[i] = x;
  else if constexpr (E == 2) v[i >> 1] |= (uint32_t)x << (16 * (i & 1));
  else v[i >> 2] |= (uint32_t)x << (8 * (i & 3));
}

// Same transpose with 16-byte global accesses on both sides: a lane loads 16/E elements that are
// consecutive along a and scatters them into LDS rows a; after the barrier a lane gathers 16/E
// elements consecutive along b from one LDS row and stores them with one 16-byte store.  Needs
// na and nb to be multiples of 16/E and 16-byte aligned bases and pitches.
template <int E>
__device__ __forceinline__ void transpose_tile_vec(gsrc_t __restrict__ s, gdst_t __restrict__ d, uint32_t na,
                                                   uint32_t nb, int64_t spb, int64_t dpa, uint32_t td, char* lds) {
  constexpr uint32_t VE = 16 / E;
  const uint32_t pitch = td + 1, nt = blockDim.x, tid = threadIdx.x;
  const uint32_t vpr = na / VE, total = vpr * nb;
  for (uint32_t base = 0; base < total; base += 4 * nt) {
    u32x4 v[4];
    uint32_t bb[4], aa[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t idx = base + u * nt + tid;
      bb[u] = idx / vpr;
      aa[u] = (idx - bb[u] * vpr) * VE;
      if (idx < total) v[u] = ld<16>(s + (size_t)aa[u] * E + (int64_t)bb[u] * spb);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (base + u * nt + tid < total) {
#pragma unroll
        for (uint32_t i = 0; i < VE; ++i)
          lds_st<E>(lds + (size_t)((aa[u] + i) * pitch + bb[u]) * E, get_elem<E>(v[u], i));
      }
    }
  }
  __syncthreads();
  const uint32_t wpr = nb / VE, totw = wpr * na;
  for (uint32_t w = tid; w < totw; w += nt) {
    const uint32_t a = w / wpr, b0 = (w - a * wpr) * VE;
    u32x4 out = {0u, 0u, 0u, 0u};
#pragma unroll
    for (uint32_t i = 0; i < VE; ++i) set_elem<E>(out, i, lds_ld<E>(lds + (size_t)(a * pitch + b0 + i) * E));
    st<16>(d + (size_t)b0 * E + (int64_t)a * dpa, out);
  }
  __syncthreads();  // the staging area is free again
}

template <int E>
__device__ __forceinline__ void transpose_any(gsrc_t __restrict__ s, gdst_t __restrict__ d, uint32_t na, uint32_t nb,
                                              int64_t spb, int64_t dpa, uint32_t td, char* lds) {
  constexpr uint32_t VE = 16 / E;
  const uintptr_t al = (uintptr_t)s | (uintptr_t)d | (uintptr_t)spb | (uintptr_t)dpa;
  if ((al & 15u) == 0 && na % VE == 0 && nb % VE == 0) transpose_tile_vec<E>(s, d, na, nb, spb, dpa, td, lds);
  else transpose_tile<E>(s, d, na, nb, spb, dpa, td, lds);
}

// rows of `run` bytes where 16-byte alignment does not hold everywhere: unaligned 16-byte vectors
// over all rows at once, then the (run mod 16) tail bytes of every row.
__device__ __forceinline__ void copy_rows_unaligned(gsrc_t __restrict__ s, gdst_t __restrict__ d, uint32_t nrows,
                                                    uint32_t run, int64_t sp, int64_t dp, uint32_t tid, uint32_t nt) {
  const uint32_t body = run >> 4, tail = run & 15u;
  if (body) copy_rows<-16>(s, d, nrows, body, sp, dp, tid, nt);
  if (tail) {
    const uint32_t total = nrows * tail;
    const size_t off = (size_t)body << 4;
    for (uint32_t i = tid; i < total; i += nt) {
      const uint32_t r = i / tail, b = i - r * tail;
      d[(int64_t)r * dp + off + b] = s[(int64_t)r * sp + off + b];
    }
  }
}

// `nt` threads (tid in [0, nt)) copy one tile: the whole workgroup (WG == true, may use the LDS
// staging area and barriers) or a single wave (WG == false, no barriers).
template <bool WG>
__device__ __forceinline__ void process_tile(const TileDesc& T, gsrc_t s, gdst_t d, char* lds, uint32_t tid,
                                             uint32_t nt) {
  if ((T.kind & 0xffu) == kTranspose) {
    const uint32_t e = (T.kind >> 8) & 0xffu, td = T.kind >> 16, na = T.a, nb = T.b;
    const int64_t spb = T.p0, dpa = T.p1;
    const uintptr_t al = (uintptr_t)s | (uintptr_t)d | (uintptr_t)spb | (uintptr_t)dpa;
    if (WG && (al & (e - 1)) == 0) {
      switch (e) {
        case 1: transpose_any<1>(s, d, na, nb, spb, dpa, td, lds); break;
        case 2: transpose_any<2>(s, d, na, nb, spb, dpa, td, lds); break;
        case 4: transpose_any<4>(s, d, na, nb, spb, dpa, td, lds); break;
        case 8: transpose_any<8>(s, d, na, nb, spb, dpa, td, lds); break;
        default: transpose_any<16>(s, d, na, nb, spb, dpa, td, lds); break;
      }
    } else {  // single wave, or elements not aligned to their own size: plain byte moves
      const uint32_t total = na * nb * e;
      for (uint32_t i = tid; i < total; i += nt) {
        const uint32_t el = i / e, by = i - el * e;
        const uint32_t b = el / na, a = el - b * na;
        d[(int64_t)a * dpa + (int64_t)b * e + by] = s[(int64_t)a * e + (int64_t)b * spb + by];
      }
    }
    return;
  }
  const uint32_t run = T.a, nrows = T.b;
  const int64_t sp = T.p0, dp = T.p1;
  uintptr_t al = (uintptr_t)s | (uintptr_t)d | (uintptr_t)run;
  if (nrows > 1) al |= (uintptr_t)sp | (uintptr_t)dp;
  if ((al & 15u) == 0) {
    copy_rows<16>(s, d, nrows, run >> 4, sp, dp, tid, nt);
  } else if (run >= 64) {
    if (nrows == 1) copy_run_misaligned(s, d, run, tid, nt);
    else copy_rows_unaligned(s, d, nrows, run, sp, dp, tid, nt);
  } else if ((al & 7u) == 0) {
    copy_rows<8>(s, d, nrows, run >> 3, sp, dp, tid, nt);
  } else if ((al & 3u) == 0) {
    copy_rows<4>(s, d, nrows, run >> 2, sp, dp, tid, nt);
  } else if ((al & 1u) == 0) {
    copy_rows<2>(s, d, nrows, run >> 1, sp, dp, tid, nt);
  } else {
    copy_rows<1>(s, d, nrows, run, sp, dp, tid, nt);
  }
}

// Buffer pointers reach the kernel as kernel arguments (up to kArgPtrs of them: no host-to-device
// copy, no staging) or, for bigger tables, through a device array.  Either way they are staged in
// LDS once per workgroup when they fit.
struct PtrArgs {
  uint64_t p[kArgPtrs];
};

// queue[0]: next batch index; queue[1]: workgroups that are done.  The last workgroup to finish
// puts both back to zero, so the next launch on this plan needs no memset.
template <typename PTRS>
__device__ __forceinline__ void reshard_body(const TileDesc* __restrict__ heads, uint32_t n_batches,
                                             const TileDesc* __restrict__ tiles, const PTRS& ptr_table,
                                             uint32_t n_src, uint32_t n_ptrs, unsigned long long* queue,
                                             int persistent) {
  __shared__ __attribute__((aligned(16))) char lds[kLdsBytes];
  __shared__ uint64_t lds_ptrs[kLdsPtrs];
  __shared__ uint32_t slot[2];
  // ranged launch (a chunk of a source blob has arrived): the lookup kernel left the first batch in
  // the queue word and one past the last batch in queue[3]
  if (persistent == 2) n_batches = (uint32_t)queue[3];
  const bool ptrs_in_lds = n_ptrs <= (uint32_t)kLdsPtrs;
  if (ptrs_in_lds)
    for (uint32_t i = threadIdx.x; i < n_ptrs; i += blockDim.x) lds_ptrs[i] = ptr_table[i];
  auto src_of = [&](const TileDesc& T) -> gsrc_t {
    const uint64_t p = ptrs_in_lds ? lds_ptrs[T.src_buf] : ptr_table[T.src_buf];
    return (gsrc_t)p + T.src_off;
  };
  auto dst_of = [&](const TileDesc& T) -> gdst_t {
    const uint64_t p = ptrs_in_lds ? lds_ptrs[n_src + T.dst_buf] : ptr_table[n_src + T.dst_buf];
    return (gdst_t)p + T.dst_off;
  };
  // one batch: a single tile for the whole workgroup, or several small tiles dealt to the waves
  auto run_batch = [&](const TileDesc& H) {
    if (H.count == 1) {
      process_tile<true>(H, src_of(H), dst_of(H), lds, threadIdx.x, blockDim.x);
    } else {
      const uint32_t wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6, lane = threadIdx.x & 63u;
      for (uint32_t j = wave; j < H.count; j += n_waves) {
        const uint32_t t = __builtin_amdgcn_readfirstlane(H.first + j);
        const TileDesc T = tiles[t];
        process_tile<false>(T, src_of(T), dst_of(T), lds, lane, 64);
      }
    }
  };
  if (!persistent) {
    __syncthreads();
    const uint32_t b = blockIdx.x;
    if (b < n_batches) run_batch(heads[b]);
    return;
  }
  // Two batch indices are kept in flight: the current one and the next one, whose head descriptor
  // is loaded while the current batch is copied.  slot[ph] receives the index after that.
  if (threadIdx.x == 0) {
    slot[0] = (uint32_t)min(atomicAdd(queue, 1ull), (unsigned long long)n_batches);
    slot[1] = (uint32_t)min(atomicAdd(queue, 1ull), (unsigned long long)n_batches);
  }
  __syncthreads();
  uint32_t cur = __builtin_amdgcn_readfirstlane(slot[0]);
  uint32_t nxt = __builtin_amdgcn_readfirstlane(slot[1]);
  __syncthreads();  // both slots read before slot[0] is written again
  if (cur < n_batches) {
    TileDesc H = heads[cur];
    int ph = 0;
    for (;;) {
      TileDesc N = H;
      if (nxt < n_batches) N = heads[nxt];  // scalar loads, consumed only after this batch's copy
      unsigned long long popped = 0;
      if (threadIdx.x == 0) popped = atomicAdd(queue, 1ull);
      run_batch(H);
      if (threadIdx.x == 0) slot[ph] = (uint32_t)min(popped, (unsigned long long)n_batches);
      __syncthreads();
      if (nxt >= n_batches) break;  // uniform: the queue only grows, every workgroup gets here
      H = N;
      cur = nxt;
      nxt = __builtin_amdgcn_readfirstlane(slot[ph]);
      ph ^= 1;  // the other slot is written next, so no second barrier is needed
    }
  }
  // this workgroup pops no more; the last one to say so rearms the queue
  if (threadIdx.x == 0) {
    __threadfence();
    if (atomicAdd(queue + 1, 1ull) == (unsigned long long)gridDim.x - 1) {
      atomicExch(queue, 0ull);
      atomicExch(queue + 1, 0ull);
    }
  }
}

__global__ __launch_bounds__(kMaxThreads) void k_reshard(const TileDesc* __restrict__ heads, uint32_t n_batches,
                                                         const TileDesc* __restrict__ tiles, PtrArgs ptrs,
                                                         uint32_t n_src, uint32_t n_ptrs, unsigned long long* queue,
                                                         int persistent) {
  reshard_body(heads, n_batches, tiles, ptrs.p, n_src, n_ptrs, queue, persistent);
}

__global__ __launch_bounds__(kMaxThreads) void k_reshard_table(const TileDesc* __restrict__ heads, uint32_t n_batches,
                                                               const TileDesc* __restrict__ tiles,
                                                               const uint64_t* __restrict__ ptr_table, uint32_t n_src,
                                                               uint32_t n_ptrs, unsigned long long* queue,
                                                               int persistent) {
  reshard_body(heads, n_batches, tiles, ptr_table, n_src, n_ptrs, queue, persistent);
}

// Batches of a source-ordered plan whose key lies in [key_lo, key_hi): the queue starts at the
// first of them, queue[3] is one past the last.
__global__ void k_range_lookup(const uint64_t* __restrict__ batch_key, uint32_t n_batches, uint64_t key_lo,
                               uint64_t key_hi, unsigned long long* queue) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  uint32_t bound[2];
  const uint64_t want[2] = {key_lo, key_hi};
  for (int k = 0; k < 2; ++k) {
    uint32_t lo = 0, hi = n_batches;
    while (lo < hi) {
      const uint32_t mid = lo + ((hi - lo) >> 1);
      if (batch_key[mid] < want[k]) lo = mid + 1; else hi = mid;
    }
    bound[k] = lo;
  }
  queue[0] = bound[0];
  queue[1] = 0;
  queue[2] = bound[0];
  queue[3] = bound[1];
}

__global__ __launch_bounds__(256) void k_copy_baseline(u32x4* __restrict__ dst, const u32x4* __restrict__ src,
                                                       uint64_t n_vec, uint32_t vec_per_block) {
  const uint64_t base = (uint64_t)blockIdx.x * vec_per_block;
  const uint64_t end = min(n_vec, base + vec_per_block);
  uint64_t i = base + threadIdx.x;
  for (; i + 3 * 256 < end; i += 4 * 256) {
    const u32x4 a = src[i], b = src[i + 256], c = src[i + 2 * 256], e = src[i + 3 * 256];
    dst[i] = a;
    dst[i + 256] = b;
    dst[i + 2 * 256] = c;
    dst[i + 3 * 256] = e;
  }
  for (; i < end; i += 256) dst[i] = src[i];
}

}  // namespace

int device_cu_count() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  return n;
}

// src/dst: host arrays of device pointers when the table fits the kernel arguments
// (n_src + n_dst <= kMaxKernargPtrs), else `table` is a device array [src pointers | dst pointers].
bcp_status launch_reshard(const PlanDevice& plan, const void* const* src, int32_t n_src, void* const* dst,
                          int32_t n_dst, const void* table, hipStream_t stream, const uint64_t* key_range) {
  if (plan.n_batches == 0) return BCP_OK;
  PlanConfig cfg = config();
  if (key_range) {
    if (!plan.batch_key) {
      set_error("the plan was not built with BCP_ORDER_BY_SOURCE");
      return BCP_ERR_INVALID_ARG;
    }
    hipLaunchKernelGGL(k_range_lookup, dim3(1), dim3(64), 0, stream, plan.batch_key, (uint32_t)plan.n_batches,
                       key_range[0], key_range[1], plan.queue);
    BCP_HIP(hipGetLastError());
    cfg.persistent = 2;  // the range is only known on the device: always the queue-driven grid
  }
  unsigned grid;
  if (cfg.persistent) {
    const int cus = device_cu_count();
    if (cus <= 0) {
      set_error("cannot read the CU count");
      return BCP_ERR_NO_DEVICE;
    }
    grid = (unsigned)std::min<int64_t>(plan.n_batches, (int64_t)cus * cfg.wg_per_cu);
  } else {
    grid = (unsigned)plan.n_batches;
  }
  const uint32_t n_ptrs = (uint32_t)(n_src + n_dst);
  if (!table) {
    PtrArgs args;
    for (int32_t i = 0; i < n_src; ++i) args.p[i] = (uint64_t)(uintptr_t)src[i];
    for (int32_t i = 0; i < n_dst; ++i) args.p[n_src + i] = (uint64_t)(uintptr_t)dst[i];
    for (uint32_t i = n_ptrs; i < (uint32_t)kArgPtrs; ++i) args.p[i] = 0;
    hipLaunchKernelGGL(k_reshard, dim3(grid), dim3((unsigned)cfg.threads), 0, stream, plan.heads,
                       (uint32_t)plan.n_batches, plan.tiles, args, (uint32_t)n_src, n_ptrs, plan.queue,
                       cfg.persistent);
  } else {
    hipLaunchKernelGGL(k_reshard_table, dim3(grid), dim3((unsigned)cfg.threads), 0, stream, plan.heads,
                       (uint32_t)plan.n_batches, plan.tiles, (const uint64_t*)table, (uint32_t)n_src, n_ptrs,
                       plan.queue, cfg.persistent);
  }
  BCP_HIP(hipGetLastError());
  return BCP_OK;
}

bcp_status launch_copy_baseline(void* dst, const void* src, int64_t nbytes, hipStream_t stream) {
  if (nbytes <= 0) return BCP_OK;
  if ((((uintptr_t)dst | (uintptr_t)src) & 15u) || (nbytes & 15)) {
    set_error("bcp_copy_baseline needs 16-byte aligned pointers and size");
    return BCP_ERR_INVALID_ARG;
  }
  const uint64_t n_vec = (uint64_t)nbytes / 16;
  const uint32_t vpb = 65536 / 16;
  const uint64_t grid = (n_vec + vpb - 1) / vpb;
  if (grid >= 0x7fffffffull) {
    set_error("copy too large for one launch");
    return BCP_ERR_INVALID_ARG;
  }
  hipLaunchKernelGGL(k_copy_baseline, dim3((unsigned)grid), dim3(256), 0, stream, (u32x4*)dst, (const u32x4*)src,
                     n_vec, vpb);
  BCP_HIP(hipGetLastError());
  return BCP_OK;
}

}  // namespace bcp
