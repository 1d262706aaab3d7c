// The copy kernel: executes a plan's tiles.  Pure byte movement, HBM-bandwidth bound:
// every payload byte is read once and written once; there is no contraction, hence no MFMA.
//
// A tile is at most tile_bytes of payload: a segment of one long row, or a few whole short
// rows, decoded at plan time into one 64-byte descriptor.  Per tile the kernel picks, from the
// actual addresses, one of
//   * 16-byte vector path   -- bases, run length and pitches all 16-byte aligned;
//   * misaligned-run path   -- long runs whose source and destination disagree modulo 16 (ZeRO
//                              slice boundaries): peel to a 16-byte aligned destination; then aligned
//                              16-byte loads of the source chunks, each lane taking its right-hand
//                              neighbour's chunk by a shuffle and funnel-shifting the pair into one
//                              aligned 16-byte store;
//   * granule path          -- whole-workgroup tiles of short misaligned rows: 8/4/2/1-byte granules, flat
//                              over rows x run;
//   * small-tile batches    -- tiles below 16 KiB share a workgroup: per tile one item size (16 bytes, or the
//                              largest power of two a short row holds) at any address, a row's last item
//                              moved back to end with the row; tiles ordered by item size so that a wave
//                              issues one load and one store per round;
//   * LDS-staged transpose  -- the source-contiguous and destination-contiguous dimensions
//                              differ (strided shards): both global sides stay coalesced;
//   * narrowing rows        -- dtype-converting loads (fp32 saved, bf16 asked for): 4 bytes read and
//                              2 written per element; a wave takes 512 elements with two load instructions
//                              that each cover 1 KiB without gaps, neighbouring lanes swap halves and
//                              every lane stores 16 bytes.
// Scheduling: a persistent grid of (CU count x wg_per_cu) workgroups pops batch indices from an
// atomic queue; a batch is one big tile (whole workgroup) or a run of small tiles that share the
// workgroup's threads in proportion to their size, so 100k tiny tensors do not cost one queue pop
// each.  Measured on MI355X, ONE 1024-thread workgroup per CU streaming 64 KiB tiles with
// non-temporal accesses sustains the highest copy bandwidth of all launch shapes, persistent or
// one workgroup per tile.  The head descriptor of the next batch is fetched (scalar loads)
// while the current batch is being copied, and the buffer-pointer table is staged in LDS once per
// workgroup, so no dependent global load sits between two batches.
#include <algorithm>
#include <mutex>
#include <string>

#include "bcp_internal.h"

namespace bcp {
namespace {

constexpr int kMaxThreads = 1024;
// The staging area in LDS is sized at launch: what the plan's largest transposed tile needs, and
// at least the room the small-tile batches take (one descriptor and one counter per thread).
constexpr uint32_t kOrderWaves = 4;   // tiles are put in the order of their item sizes inside windows of this many waves
constexpr uint32_t kItemClasses = 8;  // item sizes 1 .. 16 bytes, converting tiles, and room to a power of two
constexpr uint32_t small_batch_lds_bytes(uint32_t threads) {
  return threads * (uint32_t)sizeof(TileDesc) + (threads + 1 + kMaxThreads / 64) * 4u + threads * 4u +
         kItemClasses * (kMaxThreads / 64) * 4u;
}
constexpr uint32_t kMaxDynamicLds = 144 * 1024;  // of the CU's 160 KiB; pointers and queue slots are static
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
// small tiles: neighbouring tiles share cache lines at their edges, and the L2 that has a line from one
// tile serves, or merges with, the next one's part of it -- ordinary (temporal) accesses
template <int G>
__device__ __forceinline__ typename Granule<G>::type ldc(gsrc_t p) {
  return *(const typename Granule<G>::type BCP_GLOBAL*)p;
}
template <int G>
__device__ __forceinline__ void stc(gdst_t p, typename Granule<G>::type v) {
  *(typename Granule<G>::type BCP_GLOBAL*)p = v;
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
typedef u32x2 u32x2_unaligned __attribute__((aligned(1)));
typedef uint32_t u32_unaligned __attribute__((aligned(1)));
typedef uint16_t u16_unaligned __attribute__((aligned(1)));
template <> struct Granule<-16> { typedef u32x4 type; };
template <>
__device__ __forceinline__ u32x4 ld<-16>(gsrc_t p) {
  return __builtin_nontemporal_load((const u32x4_unaligned BCP_GLOBAL*)p);
}
template <>
__device__ __forceinline__ void st<-16>(gdst_t p, u32x4 v) {
  __builtin_nontemporal_store(v, (u32x4_unaligned BCP_GLOBAL*)p);
}
template <>
__device__ __forceinline__ u32x4 ldc<-16>(gsrc_t p) {
  return *(const u32x4_unaligned BCP_GLOBAL*)p;
}
template <>
__device__ __forceinline__ void stc<-16>(gdst_t p, u32x4 v) {
  *(u32x4_unaligned BCP_GLOBAL*)p = v;
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
    if (i < run_g) {  // up to three granules of a lane are left: all in flight together, like a full round
      const bool two = i + nt < run_g, three = i + 2 * nt < run_g;
      V a = ld<GG>(s + (size_t)i * G), b = a, c = a;
      if (two) b = ld<GG>(s + (size_t)(i + nt) * G);
      if (three) c = ld<GG>(s + (size_t)(i + 2 * nt) * G);
      st<GG>(d + (size_t)i * G, a);
      if (two) st<GG>(d + (size_t)(i + nt) * G, b);
      if (three) st<GG>(d + (size_t)(i + 2 * nt) * G, c);
    }
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
  if (i < total) {  // up to three granules of a lane are left: all in flight together, like a full round
    V v[3];
    int64_t dof[3];
    bool have[3];
#pragma unroll
    for (int u = 0; u < 3; ++u) {
      have[u] = i + u * nt < total;
      dof[u] = (int64_t)row * dp + (int64_t)col * G;
      if (have[u]) v[u] = ld<GG>(s + (int64_t)row * sp + (int64_t)col * G);
      col += dcol;
      row += drow;
      if (col >= run_g) {
        col -= run_g;
        ++row;
      }
    }
#pragma unroll
    for (int u = 0; u < 3; ++u)
      if (have[u]) st<GG>(d + dof[u], v[u]);
  }
}

// Bytes m .. m + 15 of the 32 bytes [lo | hi], m = 4 q + r the same for every lane.
__device__ __forceinline__ u32x4 funnel16(const u32x4& lo, const u32x4& hi, uint32_t q, uint32_t r) {
  uint32_t w0, w1, w2, w3, w4;
  switch (q) {
    case 0: w0 = lo[0], w1 = lo[1], w2 = lo[2], w3 = lo[3], w4 = hi[0]; break;
    case 1: w0 = lo[1], w1 = lo[2], w2 = lo[3], w3 = hi[0], w4 = hi[1]; break;
    case 2: w0 = lo[2], w1 = lo[3], w2 = hi[0], w3 = hi[1], w4 = hi[2]; break;
    default: w0 = lo[3], w1 = hi[0], w2 = hi[1], w3 = hi[2], w4 = hi[3]; break;
  }
  u32x4 o;  // v_alignbyte_b32: ({high, low} >> 8 r), low word
  o[0] = __builtin_amdgcn_alignbyte(w1, w0, r);
  o[1] = __builtin_amdgcn_alignbyte(w2, w1, r);
  o[2] = __builtin_amdgcn_alignbyte(w3, w2, r);
  o[3] = __builtin_amdgcn_alignbyte(w4, w3, r);
  return o;
}

// one contiguous run whose two sides disagree modulo 16: byte head up to the destination's next
// 16-byte boundary, then aligned 16-byte stores, byte tail.  What is stored comes from ALIGNED 16-byte loads too
// (a vector load at an address that is no multiple of 4 is taken apart by the hardware, and one at a multiple of 4
// still touches two chunks): the wave loads 64 consecutive aligned source chunks, every lane gets its right-hand
// neighbour's chunk by a shuffle (the last lane loads one chunk more) and shifts the 16 bytes it needs out of
// the two.  Chunks are read whole, so up to 15 bytes before the run and after it are read as well: they lie in
// 16-byte pieces that also hold bytes of the run, hence inside the same allocation.
// nt: a multiple of 64.  U: consecutive strips of 64 output chunks a wave takes per round (its loads in flight).
template <uint32_t U>
__device__ __forceinline__ void copy_run_misaligned(gsrc_t __restrict__ s, gdst_t __restrict__ d, uint32_t run,
                                                    uint32_t tid, uint32_t nt) {
  uint32_t head = (uint32_t)(-(uintptr_t)d) & 15u;
  if (head > run) head = run;
  for (uint32_t i = tid; i < head; i += nt) d[i] = s[i];
  const uint32_t body = (run - head) >> 4;
  gsrc_t s2 = s + head;
  gdst_t d2 = d + head;
  const uint32_t m = (uint32_t)(uintptr_t)s2 & 15u;
  if (m == 0) {  // (the two sides agree after all)
    for (uint32_t i = tid; i < body; i += nt) st<16>(d2 + (size_t)i * 16, ld<16>(s2 + (size_t)i * 16));
  } else {
    gsrc_t sa = s2 - m;  // aligned; output chunk c is bytes m .. m + 15 of the source chunks c and c + 1
    const uint32_t q = m >> 2, r = m & 3u;
    const uint32_t lane = tid & 63u, wave = tid >> 6, nw = nt >> 6;
    const uint32_t rounds = (body + 64u * U - 1u) / (64u * U);
    for (uint32_t rd = wave; rd < rounds; rd += nw) {
      const uint32_t c0 = rd * (64u * U) + lane;   // this lane's chunk of the round's first strip
      u32x4 lo[U], last = {0u, 0u, 0u, 0u};
#pragma unroll
      for (uint32_t u = 0; u < U; ++u) {
        const uint32_t c = c0 + 64u * u;
        lo[u] = u32x4{0u, 0u, 0u, 0u};
        if (c <= body) lo[u] = ld<16>(sa + (size_t)c * 16);
      }
      // (the chunk after the round's last one: only the last lane of the last strip needs it from memory; inside
      // the round the next strip's first lane has it)
      if (lane == 63u && c0 + 64u * (U - 1u) + 1u <= body) last = ld<16>(sa + (size_t)(c0 + 64u * (U - 1u) + 1u) * 16);
#pragma unroll
      for (uint32_t u = 0; u < U; ++u) {
        const uint32_t c = c0 + 64u * u;
        u32x4 next;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          next[k] = (uint32_t)__shfl_down((int)lo[u][k], 1);
          const uint32_t first_of_next = u + 1u < U ? (uint32_t)__builtin_amdgcn_readfirstlane((int)lo[u + 1u < U ? u + 1u : u][k]) : last[k];
          if (lane == 63u) next[k] = first_of_next;
        }
        if (c < body) st<16>(d2 + (size_t)c * 16, funnel16(lo[u], next, q, r));
      }
    }
  }
  const uint32_t done = head + (body << 4);
  for (uint32_t i = done + tid; i < run; i += nt) d[i] = s[i];
}

// ---- transposed tiles ----------------------------------------------------------------------------
// source: element (a, b) at s + a*E + b*spb (contiguous along a)
// destination: element (a, b) at d + b*E + a*dpa (contiguous along b)
// A tile is na x nb elements, at most tda x tdb (the full tile's edges, powers of two).
// Staging: row a holds the tile's elements (a, 0 .. nb), tdb + 1 elements apart: the odd pitch
// spreads both a column and a row over the LDS banks.

// element by element, for tiles whose addresses or extents rule out 16-byte accesses
template <int E>
__device__ __forceinline__ void transpose_tile(gsrc_t __restrict__ s, gdst_t __restrict__ d, uint32_t na,
                                               uint32_t nb, int64_t spb, int64_t dpa, uint32_t tda, uint32_t tdb,
                                               char* lds) {
  const uint32_t pitch = tdb + 1;
  uint32_t tid = threadIdx.x;
  asm volatile("" : "+v"(tid));  // opaque, see transpose_full_tile
  {
    const uint32_t x = tid & (tda - 1), y0 = tid / tda, step = blockDim.x / tda;
    if (x < na)
      for (uint32_t b = y0; b < nb; b += step)
        lds_st<E>(lds + (size_t)(x * pitch + b) * E, ld<E>(s + (size_t)x * E + (int64_t)b * spb));
  }
  __syncthreads();
  {
    const uint32_t x = tid & (tdb - 1), y0 = tid / tdb, step = blockDim.x / tdb;
    if (x < nb)
      for (uint32_t a = y0; a < na; a += step)
        st<E>(d + (size_t)x * E + (int64_t)a * dpa, lds_ld<E>(lds + (size_t)(a * pitch + x) * E));
  }
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

// The same with 16-byte global accesses on both sides.  Going in, a lane loads a vector of 16/E
// elements consecutive along a and scatters them into LDS rows a .. a + 16/E; coming out, it
// gathers 16/E elements consecutive along b from one LDS row and stores them as one vector.  In
// both directions the 64 lanes of a wave form 8 x 8 blocks: 8 consecutive vectors (128 bytes of
// one row in memory) by 8 rows, which with the odd LDS pitch puts the lanes of a 4-byte access on
// different banks.  Needs na and nb to be multiples of 16/E and 16-byte aligned bases and pitches.
template <int E>
__device__ __forceinline__ void transpose_tile_vec(gsrc_t __restrict__ s, gdst_t __restrict__ d, uint32_t na,
                                                   uint32_t nb, int64_t spb, int64_t dpa, uint32_t tdb, char* lds) {
  constexpr uint32_t VE = 16 / E;
  constexpr int U = 4;
  uint32_t tid = threadIdx.x;
  asm volatile("" : "+v"(tid));  // opaque, see transpose_full_tile
  const uint32_t pitch = tdb + 1, nt = blockDim.x;
  const uint32_t lo = tid & 7u, hi = (tid >> 3) & 7u, blk0 = tid >> 6, dblk = nt >> 6;
  {  // in: blocks of 8 vectors along a by 8 rows b, wave after wave, U per thread at a time
    const uint32_t vpr = na / VE, chunks_a = (vpr + 7) >> 3, n_blk = chunks_a * ((nb + 7) >> 3);
    for (uint32_t base = 0; base < n_blk; base += U * dblk) {
      u32x4 v[U];
      uint32_t pos[U];  // of v[u]: vector index along a | row << 16, ~0: nothing loaded
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t blk = base + blk0 + u * dblk;
        const uint32_t cb = blk / chunks_a, ca = blk - cb * chunks_a;
        const uint32_t va = ca * 8 + lo, b = cb * 8 + hi;
        pos[u] = ~0u;
        if (va < vpr && b < nb) {
          pos[u] = va | (b << 16);
          v[u] = ld<16>(s + (size_t)va * 16 + (int64_t)b * spb);
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (pos[u] != ~0u) {
          const uint32_t a0 = (pos[u] & 0xffffu) * VE, b = pos[u] >> 16;
#pragma unroll
          for (uint32_t i = 0; i < VE; ++i)
            lds_st<E>(lds + (size_t)((a0 + i) * pitch + b) * E, get_elem<E>(v[u], i));
        }
      }
    }
  }
  __syncthreads();
  {  // out: blocks of 8 vectors along b by 8 rows a
    const uint32_t wpr = nb / VE, chunks_b = (wpr + 7) >> 3, n_blk = chunks_b * ((na + 7) >> 3);
    for (uint32_t blk = blk0; blk < n_blk; blk += dblk) {
      const uint32_t ca = blk / chunks_b, cb = blk - ca * chunks_b;
      const uint32_t vb = cb * 8 + lo, a = ca * 8 + hi;
      if (vb < wpr && a < na) {
        u32x4 out = {0u, 0u, 0u, 0u};
#pragma unroll
        for (uint32_t i = 0; i < VE; ++i) set_elem<E>(out, i, lds_ld<E>(lds + (size_t)(a * pitch + vb * VE + i) * E));
        st<16>(d + (size_t)vb * 16 + (int64_t)a * dpa, out);
      }
    }
  }
  __syncthreads();  // the staging area is free again
}

// A full tile with everything known at compile time (1024 threads, both edges full for this element
// size).  Every wave owns a block of the tile, 8 vectors along a by 32 rows along b (4 KiB), loads
// it, passes it through its own part of the staging area and stores it: no wave waits for another
// one's loads, so memory latency overlaps across the 16 waves as it does in a plain copy.
__device__ __forceinline__ void wave_lds_sync() {  // LDS operations of a wave execute in order; this
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // keeps the compiler from moving them
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int E>
__device__ __forceinline__ void transpose_full_tile(gsrc_t __restrict__ s, gdst_t __restrict__ d, int64_t spb,
                                                    int64_t dpa, char* lds) {
  constexpr uint32_t VE = 16 / E, TDA = transpose_edge_a(E), TDB = transpose_edge_b(E), P = TDB + 1;
  constexpr uint32_t WA = TDA / (8 * VE);  // waves side by side along a; the others stack up along b
  constexpr uint32_t VB = 32 / VE;         // coming out: vectors per row of the block,
  constexpr uint32_t RB = 64 / VB;         //             rows per pass of the wave
  static_assert(TDA * TDB * E == 4 * kMaxThreads * 16 && (kMaxThreads / 64 / WA) * 32 == TDB, "16 blocks of 4 KiB");
  uint32_t tid = threadIdx.x;
  asm volatile("" : "+v"(tid));  // opaque: keeps the index arithmetic of the instances of this function, one per
                                 // element size, inside their branches instead of hoisted above all of them
                                 // (which costs the whole kernel registers)
  const uint32_t lane = tid & 63u, w = tid >> 6;
  const uint32_t a_w = (w % WA) * 8 * VE, b_w = (w / WA) * 32;
  const uint32_t lo = lane & 7u, hi = lane >> 3;          // in: vector lo of rows hi + 8 u
  const uint32_t lo2 = lane & (VB - 1), hi2 = lane / VB;  // out: vector lo2 of rows hi2 + RB u
  gsrc_t sp = s + (size_t)(a_w + lo * VE) * E + (int64_t)(b_w + hi) * spb;
  gdst_t dp = d + (size_t)(b_w + lo2 * VE) * E + (int64_t)(a_w + hi2) * dpa;
  const int64_t s_step = 8 * spb, d_step = (int64_t)RB * dpa;
  char* l_in = lds + (size_t)((a_w + lo * VE) * P + b_w + hi) * E;
  const char* l_out = lds + (size_t)((a_w + hi2) * P + b_w + lo2 * VE) * E;
  u32x4 v[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) v[u] = ld<16>(sp + u * s_step);
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (uint32_t i = 0; i < VE; ++i) lds_st<E>(l_in + (size_t)(i * P + u * 8) * E, get_elem<E>(v[u], i));
  wave_lds_sync();
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    u32x4 out = {0u, 0u, 0u, 0u};
#pragma unroll
    for (uint32_t i = 0; i < VE; ++i) set_elem<E>(out, i, lds_ld<E>(l_out + (size_t)(u * RB * P + i) * E));
    st<16>(dp + u * d_step, out);
  }
  wave_lds_sync();  // the block's part of the staging area is free again
}

// A full 256 x 256 tile of 2-byte elements through the LDS transpose read of gfx950.  Every wave owns a
// 64 x 64 block (8 KiB): it loads the block's 64 source rows as 16-byte vectors (eight rows of 128 bytes
// per instruction), writes them to its part of the staging area as they are -- row b of the block at
// b * kTr16Pitch, 128 bytes along a -- and reads them back with ds_read_b64_tr_b16, which hands lane l of
// a group of sixteen lanes the elements M[l/4 + 4k][l%4], k = 0..3, of the 16 x 4 matrix whose row L is
// the four elements at the address lane L gives.  Lane L of group g points at row
// 32 (g & 1) + 8 (L & 3) + (L >> 2), columns a0 .. a0 + 3; lane l then holds column a0 + (l & 3), rows
// 32 (g & 1) + 8 (l >> 2) + k: four elements consecutive along b.  A second read four rows further
// completes a 16-byte vector, and a store instruction covers eight destination rows of 128 bytes.
// Three LDS instructions per vector instead of sixteen, and no workgroup barrier.
constexpr uint32_t kTr16Pitch = 144;  // 128 bytes of a row and 16 more: rows stay 16-byte aligned for the
                                      // 16-byte writes; rows 16 apart share banks, which the reads can afford
typedef short tr_v4i16 __attribute__((ext_vector_type(4)));
typedef tr_v4i16 __attribute__((address_space(3))) * tr_lds_ptr;

__device__ __forceinline__ void transpose_full_tile_b16(gsrc_t __restrict__ s, gdst_t __restrict__ d, int64_t spb,
                                                        int64_t dpa, char* lds) {
  constexpr uint32_t P = kTr16Pitch;
  static_assert(transpose_edge_a(2) == 256 && transpose_edge_b(2) == 256 && kMaxThreads / 64 == 16, "4 x 4 blocks of 64 x 64");
  uint32_t tid = threadIdx.x;
  asm volatile("" : "+v"(tid));  // opaque, see transpose_full_tile
  const uint32_t lane = tid & 63u, w = tid >> 6;
  const uint32_t a_w = (w & 3u) * 64u, b_w = (w >> 2) * 64u;
  char* wl = lds + (size_t)w * (64u * P);
  const uint32_t lo = lane & 7u, hi = lane >> 3;  // in: vector lo of rows hi + 8 j
  gsrc_t sp = s + (size_t)(a_w + lo * 8u) * 2u + (int64_t)(b_w + hi) * spb;
  const int64_t s_step = 8 * spb;
  u32x4 v[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = ld<16>(sp + j * s_step);
#pragma unroll
  for (int j = 0; j < 8; ++j) lds_st<16>(wl + (size_t)(hi + 8u * j) * P + lo * 16u, v[j]);
  wave_lds_sync();
  const uint32_t g = lane >> 4, L = lane & 15u;
  const char* rd = wl + (size_t)(32u * (g & 1u) + 8u * (L & 3u) + (L >> 2)) * P + 8u * (g >> 1);
  gdst_t dp = d + (int64_t)(a_w + 4u * (g >> 1) + (L & 3u)) * dpa + (size_t)(b_w + (4u * (g & 1u) + (L >> 2)) * 8u) * 2u;
  const int64_t d_step = 8 * dpa;
#pragma unroll
  for (int j = 0; j < 8; ++j) {  // destination rows a_w + 8 j .. + 7
    const tr_v4i16 x = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_lds_ptr)(rd + 16u * j));
    const tr_v4i16 y = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_lds_ptr)(rd + 16u * j + 4u * P));
    u32x4 out;
    out[0] = (uint32_t)(uint16_t)x[0] | ((uint32_t)(uint16_t)x[1] << 16);
    out[1] = (uint32_t)(uint16_t)x[2] | ((uint32_t)(uint16_t)x[3] << 16);
    out[2] = (uint32_t)(uint16_t)y[0] | ((uint32_t)(uint16_t)y[1] << 16);
    out[3] = (uint32_t)(uint16_t)y[2] | ((uint32_t)(uint16_t)y[3] << 16);
    st<16>(dp + j * d_step, out);
  }
  wave_lds_sync();  // the block's part of the staging area is free again
}

template <int E>
__device__ __forceinline__ void transpose_any(gsrc_t __restrict__ s, gdst_t __restrict__ d, uint32_t na, uint32_t nb,
                                              int64_t spb, int64_t dpa, uint32_t tda, uint32_t tdb, char* lds) {
  constexpr uint32_t VE = 16 / E;
  const uintptr_t al = (uintptr_t)s | (uintptr_t)d | (uintptr_t)spb | (uintptr_t)dpa;
  // Full tiles go block by block, a wave each; 1-byte elements (a 4 KiB block of them is only 64 bytes long
  // on either side) and ragged tiles take the workgroup-wide paths.
  if constexpr (E >= 2) {
    if ((al & 15u) == 0 && blockDim.x == kMaxThreads && tda == transpose_edge_a(E) && tdb == transpose_edge_b(E) &&
        na == tda && nb == tdb) {
      if constexpr (E == 2) transpose_full_tile_b16(s, d, spb, dpa, lds);
      else transpose_full_tile<E>(s, d, spb, dpa, lds);
      return;
    }
  }
  if ((al & 15u) == 0 && na % VE == 0 && nb % VE == 0) transpose_tile_vec<E>(s, d, na, nb, spb, dpa, tdb, lds);
  else transpose_tile<E>(s, d, na, nb, spb, dpa, tda, tdb, lds);
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

// ---- dtype-converting rows: binary32 -> bfloat16 -----------------------------------------------------
// Round to nearest, ties to even (IEEE 754 roundTiesToEven); infinities stay; NaN stays NaN with its
// sign and upper seven fraction bits, quiet; subnormal results are kept.  Pairs go through the packed
// conversion instruction of gfx950 (v_cvt_pk_bf16_f32), which does exactly that; single elements at the
// ends of a run use the same rounding on the bit pattern: bfloat16 is the upper half of binary32, so
// adding 0x7FFF plus the lowest kept bit carries into the kept half exactly when the dropped half is
// above one half, or equal to it with an odd kept half (and the carry may run on into the exponent,
// which is the right result there too: the next binade, or infinity).
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t narrow_bf16(uint32_t u) {
  const uint32_t rounded = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
  const uint32_t nan = (u >> 16) | 0x40u;
  return ((u & 0x7fffffffu) > 0x7f800000u ? nan : rounded) & 0xffffu;
}
__device__ __forceinline__ uint32_t narrow_pair(uint32_t lo, uint32_t hi) {
  const f32x2 x = {__uint_as_float(lo), __uint_as_float(hi)};
  const bf16x2 y = __builtin_convertvector(x, bf16x2);
  uint32_t packed;
  __builtin_memcpy(&packed, &y, 4);
  return packed;
}
__device__ __forceinline__ u32x4 narrow8(const u32x4& a, const u32x4& b) {
  return u32x4{narrow_pair(a[0], a[1]), narrow_pair(a[2], a[3]), narrow_pair(b[0], b[1]), narrow_pair(b[2], b[3])};
}
// one element at any address
__device__ __forceinline__ void narrow_one(gsrc_t s, gdst_t d) {
  uint32_t u;
  if (((uintptr_t)s & 3u) == 0) {
    u = ld<4>(s);
  } else {
    u = (uint32_t)(uint8_t)s[0] | ((uint32_t)(uint8_t)s[1] << 8) | ((uint32_t)(uint8_t)s[2] << 16) | ((uint32_t)(uint8_t)s[3] << 24);
  }
  const uint32_t v = narrow_bf16(u);
  if (((uintptr_t)d & 1u) == 0) {
    st<2>(d, (uint16_t)v);
  } else {
    d[0] = (char)(v & 0xffu);
    d[1] = (char)(v >> 8);
  }
}

// `nrows` rows of `n` elements; source rows sp bytes apart, destination rows dp bytes apart.  Fast
// path: groups of eight elements, two 16-byte loads (at any 4-byte aligned address) and one aligned
// 16-byte store; whole waves take 64 groups at a time (convert_units) and leave a lane a group of its
// own only for the last groups of a row.  One long row is peeled to the destination's next 16-byte boundary first; rows that
// rule the groups out (odd addresses, a destination pitch or run that breaks the alignment from row to
// row) go element by element.  No barriers: any group of threads may run it.
// Units of 64 groups, a wave each: 2 KiB of source as two load instructions that each cover 1 KiB without
// gaps (lane l: chunk l, then chunk 64 + l), where a lane reading the two chunks of its own group would
// leave every other chunk of the lines an instruction touches to the next one (measured: 73 -> 79 % of
// peak).  Narrowed, the chunks are half a store each: lane 2k keeps its first (elements 8k .. 8k+3 of the
// unit), sends its second to lane 2k+1 and gets that lane's first (8k+4 .. 8k+7): output chunk k; lane
// 2k+1 stores output chunk 32 + k.  `nrows` rows with the first `upr` units of each; tid counts whole waves.
__device__ __forceinline__ void convert_units(gsrc_t __restrict__ s, gdst_t __restrict__ d, uint32_t nrows, uint32_t upr,
                                              int64_t sp, int64_t dp, uint32_t tid, uint32_t nt) {
  asm volatile("" : "+v"(tid));  // opaque, see transpose_full_tile
  const uint32_t lane = tid & 63u, nw = nt >> 6, units = nrows * upr;
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid >> 6));  // (scalar: so is what follows from it)
  const bool odd = (lane & 1u) != 0;
  const uint32_t out_off = (odd ? 512u : 0u) + 16u * (lane >> 1);
  auto finish = [&](const u32x4& a, const u32x4& b, gdst_t du) {
    const uint32_t a0 = narrow_pair(a[0], a[1]), a1 = narrow_pair(a[2], a[3]);
    const uint32_t b0 = narrow_pair(b[0], b[1]), b1 = narrow_pair(b[2], b[3]);
    // (quad_perm [1,0,3,2]: every lane reads its neighbour in the pair)
    const uint32_t r0 = (uint32_t)__builtin_amdgcn_mov_dpp((int)(odd ? a0 : b0), 0xB1, 0xF, 0xF, true);
    const uint32_t r1 = (uint32_t)__builtin_amdgcn_mov_dpp((int)(odd ? a1 : b1), 0xB1, 0xF, 0xF, true);
    const u32x4 out = odd ? u32x4{r0, r1, b0, b1} : u32x4{a0, a1, r0, r1};
    st<16>(du + out_off, out);
  };
  auto place = [&](uint32_t unit, gsrc_t* su, gdst_t* du) {  // (the same for all lanes of the wave)
    const uint32_t row = nrows == 1 ? 0 : unit / upr, cu = unit - row * upr;
    *su = s + (int64_t)row * sp + (size_t)cu * 2048 + lane * 16u;
    *du = d + (int64_t)row * dp + (size_t)cu * 1024;
  };
  uint32_t unit = wave;
  for (; unit + 3 * nw < units; unit += 4 * nw) {  // four units of a wave in flight: 128 bytes of loads per lane
    u32x4 a[4], b[4];
    gdst_t du[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      gsrc_t su;
      place(unit + u * nw, &su, &du[u]);
      a[u] = ld<-16>(su);
      b[u] = ld<-16>(su + 1024);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) finish(a[u], b[u], du[u]);
  }
  if (unit < units) {  // up to three units of a wave are left: all in flight together, like a full round
    u32x4 a[3], b[3];
    gdst_t du[3];
    bool have[3];  // (the same for all lanes of the wave)
#pragma unroll
    for (int u = 0; u < 3; ++u) {
      have[u] = unit + u * nw < units;
      if (have[u]) {
        gsrc_t su;
        place(unit + u * nw, &su, &du[u]);
        a[u] = ld<-16>(su);
        b[u] = ld<-16>(su + 1024);
      }
    }
#pragma unroll
    for (int u = 0; u < 3; ++u)
      if (have[u]) finish(a[u], b[u], du[u]);
  }
}

// WAVES: tid counts whole waves (nt a multiple of 64, lane == tid % 64), which lets the lanes of a wave share a unit.
template <bool WAVES>
__device__ __forceinline__ void convert_rows(gsrc_t __restrict__ s, gdst_t __restrict__ d, uint32_t nrows, uint32_t n,
                                             int64_t sp, int64_t dp, uint32_t tid, uint32_t nt) {
  const bool src4 = (((uintptr_t)s | (nrows > 1 ? (uintptr_t)sp : 0)) & 3u) == 0;
  if (nrows == 1 && src4 && ((uintptr_t)d & 1u) == 0) {
    uint32_t head = ((uint32_t)(-(uintptr_t)d) & 15u) >> 1;  // elements before the destination's 16-byte boundary
    if (head > n) head = n;
    const uint32_t groups = (n - head) >> 3, done = head + (groups << 3);
    for (uint32_t i = tid; i < head; i += nt) narrow_one(s + (size_t)i * 4, d + (size_t)i * 2);
    gsrc_t s2 = s + (size_t)head * 4;
    gdst_t d2 = d + (size_t)head * 2;
    uint32_t g = tid;
    if constexpr (WAVES) {
      const uint32_t units = groups >> 6;
      convert_units(s2, d2, 1u, units, 0, 0, tid, nt);
      g = (units << 6) + tid;  // the groups after the last whole unit, one lane each
    }
    for (; g + 3 * nt < groups; g += 4 * nt) {  // four groups of a lane in flight: 128 bytes of loads
      u32x4 a[4], b[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        a[u] = ld<-16>(s2 + (size_t)(g + u * nt) * 32);
        b[u] = ld<-16>(s2 + (size_t)(g + u * nt) * 32 + 16);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) st<16>(d2 + (size_t)(g + u * nt) * 16, narrow8(a[u], b[u]));
    }
    for (; g < groups; g += nt) {
      const u32x4 a = ld<-16>(s2 + (size_t)g * 32), b = ld<-16>(s2 + (size_t)g * 32 + 16);
      st<16>(d2 + (size_t)g * 16, narrow8(a, b));
    }
    for (uint32_t i = done + tid; i < n; i += nt) narrow_one(s + (size_t)i * 4, d + (size_t)i * 2);
    return;
  }
  if (nrows > 1 && src4 && (((uintptr_t)d | (uintptr_t)dp) & 15u) == 0 && (n & 7u) == 0) {
    uint32_t gpr = n >> 3;  // groups per row
    if constexpr (WAVES) {  // whole units first, then what is left of every row, group by group
      const uint32_t upr = gpr >> 6;
      if (upr) {
        convert_units(s, d, nrows, upr, sp, dp, tid, nt);
        s += (size_t)upr * 2048;
        d += (size_t)upr * 1024;
        gpr &= 63u;
        if (gpr == 0) return;
      }
    }
    const uint32_t total = nrows * gpr;
    uint32_t row = tid / gpr, col = tid - row * gpr;
    const uint32_t drow = nt / gpr, dcol = nt - drow * gpr;
    auto advance = [&]() {
      col += dcol;
      row += drow;
      if (col >= gpr) {
        col -= gpr;
        ++row;
      }
    };
    uint32_t i = tid;
    for (; i + 3 * nt < total; i += 4 * nt) {  // four groups of a lane in flight
      u32x4 a[4], b[4];
      int64_t dof[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        gsrc_t sr = s + (int64_t)row * sp + (size_t)col * 32;
        dof[u] = (int64_t)row * dp + (int64_t)col * 16;
        a[u] = ld<-16>(sr);
        b[u] = ld<-16>(sr + 16);
        advance();
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) st<16>(d + dof[u], narrow8(a[u], b[u]));
    }
    for (; i < total; i += nt) {
      gsrc_t sr = s + (int64_t)row * sp + (size_t)col * 32;
      const u32x4 a = ld<-16>(sr), b = ld<-16>(sr + 16);
      st<16>(d + (int64_t)row * dp + (size_t)col * 16, narrow8(a, b));
      advance();
    }
    return;
  }
  const uint32_t total = nrows * n;
  for (uint32_t i = tid; i < total; i += nt) {
    const uint32_t row = nrows == 1 ? 0 : i / n, col = i - row * n;
    narrow_one(s + (int64_t)row * sp + (size_t)col * 4, d + (int64_t)row * dp + (size_t)col * 2);
  }
}

// ---- small tiles ---------------------------------------------------------------------------------
// The lanes of one wave work on different tiles of a few hundred bytes with different alignments.
// What such a copy costs is instructions and memory round trips, not bandwidth.  Both are kept down by
// cutting a tile into ITEMS -- one access of 16, 8, 4, 2 or 1 bytes on both sides -- by rules worked
// out ONCE per tile, by the thread that fetched its descriptor (one thread per tile: full waves), and
// left in LDS as a SmallTile record.  A tile then gets one lane per kRound items; a lane finds its tile
// by binary search in the scanned lane counts, reads the record, decodes its items with a few
// instructions each, and all loads of the wave are issued -- whatever their sizes and tiles -- before
// the first store: one round trip per round for lanes that work on different tiles and alignments.
// items of a lane in flight (measured: 3 beats 2 by 3 %, and 1 and 4 by more); the instance with the converting path
// has no registers left for the third
constexpr int kRound = 3;
constexpr int kRoundConverting = 2;

struct SmallTile {  // 64 bytes, takes the descriptor's place in LDS
  enum Mode : uint32_t {
    kRows,   // rows of items of g bytes, g the largest power of two that fits a row (16 at most); a row's last item
             // is moved back so that it ends with the row (it may copy some bytes a second time).  Items sit at any
             // address: what a batch of small tiles costs is vector memory instructions, not bytes or alignment,
             // and a wave whose lanes all move items of one size issues one load and one store per round
    kElems,  // transposed tile: items of g bytes inside elements, source contiguous along a, destination along b
  };
  uint64_t s, d;        // addresses of the tile's first byte on the two sides
  int64_t p0, p1;       // pitches of the descriptor
  uint32_t n_items;
  uint32_t ipr;         // items per row (kRows); items per element (kElems)
  float inv_ipr;        // 1 / ipr, a little high: (i * inv_ipr) truncates to i / ipr or one more
  uint32_t body;        // kRows: offset of a row's last item; kElems: element size
  uint32_t head;        // kElems: elements along a, and 1 / that
  float inv_na;
  uint32_t mode_glog;   // mode | log2 of g << 8
  uint32_t pad_;
};
static_assert(sizeof(SmallTile) == sizeof(TileDesc), "takes the descriptor's slot");

__device__ __forceinline__ float inv_high(uint32_t n) {  // for n, i < 2^22: floor(i * inv_high(n)) is i / n or i / n + 1
  return __uint_as_float(__float_as_uint(1.0f / (float)(n ? n : 1u)) + 2u);
}
__device__ __forceinline__ uint32_t div_small(uint32_t i, uint32_t n, float inv) {
  uint32_t q = (uint32_t)((float)i * inv);
  if (q * n > i) --q;
  return q;
}

__device__ __forceinline__ SmallTile small_tile(const TileDesc& T, gsrc_t s, gdst_t d) {
  SmallTile c;
  c.s = (uint64_t)(uintptr_t)s;
  c.d = (uint64_t)(uintptr_t)d;
  c.p0 = T.p0;
  c.p1 = T.p1;
  c.ipr = 1;
  c.body = c.head = c.pad_ = 0;
  c.inv_na = 0.f;
  uint32_t mode, glog;
  if ((T.kind & 0xffu) == kTranspose) {
    const uint32_t e = (T.kind >> 8) & 0xffu;
    const uintptr_t al = (uintptr_t)s | (uintptr_t)d | (uintptr_t)T.p0 | (uintptr_t)T.p1;
    const uint32_t g = (al & (e - 1)) == 0 ? e : 1u;  // elements not aligned to their own size move as bytes
    mode = SmallTile::kElems;
    glog = 31u - (uint32_t)__clz((int)g);
    c.ipr = e / g;
    c.head = T.a;
    c.inv_na = inv_high(T.a);
    c.body = e;
    c.n_items = T.a * T.b * c.ipr;
  } else {
    const uint32_t run = T.a, nrows = T.b;
    mode = SmallTile::kRows;
    glog = run >= 16u ? 4u : (run ? 31u - (uint32_t)__clz((int)run) : 0u);
    c.ipr = (run + (1u << glog) - 1u) >> glog;  // (0 for the empty spare segment of a long row)
    c.body = run - (run ? 1u << glog : 0u);
    c.n_items = nrows * c.ipr;
  }
  c.inv_ipr = inv_high(c.ipr);
  c.mode_glog = mode | (glog << 8);
  return c;
}

// item i of the tile: byte offsets on the two sides and log2 of its size
__device__ __forceinline__ void small_item(const SmallTile& c, uint32_t i, int64_t* so, int64_t* dof, uint32_t* gl) {
  const uint32_t mode = c.mode_glog & 0xffu, glog = c.mode_glog >> 8;
  const uint32_t row = div_small(i, c.ipr, c.inv_ipr), col = i - row * c.ipr;
  *gl = glog;
  if (mode == SmallTile::kElems) {  // row: element index, col: item inside the element
    const uint32_t b = div_small(row, c.head, c.inv_na), a = row - b * c.head, by = col << glog;
    *so = (int64_t)a * c.body + (int64_t)b * c.p0 + by;
    *dof = (int64_t)a * c.p1 + (int64_t)b * c.body + by;
    return;
  }
  const uint32_t off = min(col << glog, c.body);
  *so = (int64_t)row * c.p0 + off;
  *dof = (int64_t)row * c.p1 + off;
}

// One item: the load, and later the store.  Ordinary (temporal) accesses: neighbouring tiles share cache
// lines at their edges, and the L2 that holds a line for one tile serves, or merges with, the next one's
// part of it.  Items of any size may sit at any address on either side.
__device__ __forceinline__ u32x4 item_load(gsrc_t p, uint32_t gl) {
  u32x4 v = {0u, 0u, 0u, 0u};
  if (gl == 4) v = *(const u32x4_unaligned BCP_GLOBAL*)p;
  else if (gl == 3) { const u32x2 t = *(const u32x2_unaligned BCP_GLOBAL*)p; v[0] = t[0]; v[1] = t[1]; }
  else if (gl == 2) v[0] = *(const u32_unaligned BCP_GLOBAL*)p;
  else if (gl == 1) v[0] = *(const u16_unaligned BCP_GLOBAL*)p;
  else if (gl == 0) v[0] = *(const uint8_t BCP_GLOBAL*)p;
  return v;
}
__device__ __forceinline__ void item_store(gdst_t p, uint32_t gl, const u32x4& v) {
  if (gl == 4) *(u32x4_unaligned BCP_GLOBAL*)p = v;
  else if (gl == 3) *(u32x2_unaligned BCP_GLOBAL*)p = u32x2{v[0], v[1]};
  else if (gl == 2) *(u32_unaligned BCP_GLOBAL*)p = v[0];
  else if (gl == 1) *(u16_unaligned BCP_GLOBAL*)p = (uint16_t)v[0];
  else if (gl == 0) *(uint8_t BCP_GLOBAL*)p = (uint8_t)v[0];
}

// a whole tile by `nt` lanes (tid in [0, nt)), R items of a lane in flight at a time
template <int R>
__device__ __forceinline__ void small_tile_copy(const SmallTile& c, uint32_t tid, uint32_t nt) {
  gsrc_t s = (gsrc_t)c.s;
  gdst_t d = (gdst_t)c.d;
  for (uint32_t base = tid; base < c.n_items; base += R * nt) {
    int64_t dof[R];
    uint32_t gl[R];
    u32x4 v[R];
#pragma unroll
    for (int u = 0; u < R; ++u) {
      const uint32_t i = base + u * nt;
      gl[u] = ~0u;
      int64_t so = 0;
      if (i < c.n_items) small_item(c, i, &so, &dof[u], &gl[u]);
      v[u] = item_load(s + so, gl[u]);
    }
#pragma unroll
    for (int u = 0; u < R; ++u) item_store(d + dof[u], gl[u], v[u]);
  }
}

// The whole workgroup (`nt` threads, tid in [0, nt)) copies one tile; may use the LDS staging area and
// barriers.
// TR == false: the plan holds no transposed tile that needs the staging area, and the code for
// them is left out (it would cost the other paths registers).  CV: likewise for converting tiles.
template <bool TR, bool CV>
__device__ __forceinline__ void process_tile(const TileDesc& T, gsrc_t s, gdst_t d, char* lds, uint32_t tid,
                                             uint32_t nt) {
  if (CV && (T.kind & 0xffu) == kConvert) {
    convert_rows<true>(s, d, T.b, T.a, T.p0, T.p1, tid, nt);
    return;
  }
  if ((T.kind & 0xffu) == kTranspose) {
    const uint32_t e = (T.kind >> 8) & 0xffu, na = T.a, nb = T.b;
    const uint32_t tda = 1u << ((T.kind >> 16) & 0xffu), tdb = 1u << (T.kind >> 24);
    const int64_t spb = T.p0, dpa = T.p1;
    const uintptr_t al = (uintptr_t)s | (uintptr_t)d | (uintptr_t)spb | (uintptr_t)dpa;
    if (TR && (al & (e - 1)) == 0) {
      switch (e) {
        case 1: transpose_any<1>(s, d, na, nb, spb, dpa, tda, tdb, lds); break;
        case 2: transpose_any<2>(s, d, na, nb, spb, dpa, tda, tdb, lds); break;
        case 4: transpose_any<4>(s, d, na, nb, spb, dpa, tda, tdb, lds); break;
        case 8: transpose_any<8>(s, d, na, nb, spb, dpa, tda, tdb, lds); break;
        default: transpose_any<16>(s, d, na, nb, spb, dpa, tda, tdb, lds); break;
      }
    } else {  // elements not aligned to their own size (or a plan without staged tiles): item by item
      small_tile_copy<CV ? kRoundConverting : kRound>(small_tile(T, s, d), tid, nt);
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
    if (nrows == 1) copy_run_misaligned<4u>(s, d, run, tid, nt);
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
template <bool TR, bool CV, typename PTRS>
__device__ __forceinline__ void reshard_body(const TileDesc* __restrict__ heads, uint32_t n_batches,
                                             const TileDesc* __restrict__ tiles, const PTRS& ptr_table,
                                             uint32_t n_src, uint32_t n_ptrs, unsigned long long* queue,
                                             int persistent) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
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
  // One batch: a single tile for the whole workgroup, or up to a few hundred small tiles (a few tile
  // budgets of payload).  The threads fetch and classify one tile each, a scan over the workgroup turns
  // the lane counts into lane ranges, and every lane works for the tile whose range it falls in.
  auto run_batch = [&](const TileDesc& H) {
    if (H.count == 1) {
      process_tile<TR, CV>(H, src_of(H), dst_of(H), lds, threadIdx.x, blockDim.x);
      return;
    }
    const uint32_t nthr = blockDim.x, tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    SmallTile* ltile = reinterpret_cast<SmallTile*>(lds);                                // [nthr]
    uint32_t* lstart = reinterpret_cast<uint32_t*>(lds + sizeof(SmallTile) * nthr);      // [nthr + 1]
    uint32_t* lwave = lstart + nthr + 1;                                                 // [waves]
    uint32_t* lcount = lwave + kMaxThreads / 64;                                         // [nthr]
    uint32_t* lclass = lcount + nthr;                                                    // [kItemClasses][waves]
    for (uint32_t base = 0; base < H.count; base += nthr) {
      const uint32_t n = min(nthr, H.count - base);
      uint32_t c = 0, cls = kItemClasses - 1;
      SmallTile rec;
      if (tid < n) {
        const TileDesc T = tiles[H.first + base + tid];
        if (CV && (T.kind & 0xffu) == kConvert) {  // converting tiles: what convert_rows needs, marked by the mode
          SmallTile raw;
          raw.s = (uint64_t)(uintptr_t)src_of(T);
          raw.d = (uint64_t)(uintptr_t)dst_of(T);
          raw.p0 = T.p0;
          raw.p1 = T.p1;
          raw.n_items = max(T.b * ((T.a + 7u) >> 3), 1u);  // groups of eight elements
          raw.ipr = T.b;       // rows
          raw.body = T.a;      // elements per row
          raw.mode_glog = 0xffu;
          rec = raw;
          c = raw.n_items;
          cls = 5;
        } else {
          rec = small_tile(T, src_of(T), dst_of(T));
          c = (rec.n_items + (CV ? kRoundConverting : kRound) - 1) / (CV ? kRoundConverting : kRound);
          cls = rec.mode_glog >> 8;  // log2 of the item size: 0 .. 4
        }
        c = c < 1 ? 1u : (c > nthr ? nthr : c);
      }
      // The tiles of every kOrderWaves waves (256 tiles, neighbours in memory) are put in the order of their item sizes
      // (stable inside a size): the lanes of a wave then mostly move items of one size, and a wave issues one load
      // and one store per round and size.  (Ordering the whole slice makes the waves a little more uniform still,
      // but tiles that share cache lines at their edges are then copied so far apart in time that the lines leave the
      // L2 in between.)  Rank inside the class from ballots; bases from a scan of the table of counts, whose
      // entries run window by window, class by class, wave by wave.
      {
        uint32_t rank = 0, mine = 0;
#pragma unroll
        for (uint32_t k = 0; k < kItemClasses - 1; ++k) {
          const unsigned long long m = __ballot(cls == k);
          if (cls == k) rank = (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
          if (lane == k) mine = (uint32_t)__popcll(m);
        }
        constexpr uint32_t W = kOrderWaves;  // waves per window
        auto entry = [](uint32_t w, uint32_t k) { return (w / W) * (W * kItemClasses) + k * W + (w % W); };
        if (lane < kItemClasses) lclass[entry(wave, lane)] = mine;
        __syncthreads();
        if (wave == 0) {  // exclusive scan of the table: two entries per lane
          const uint32_t nw = nthr >> 6;
          const uint32_t e0 = 2u * lane, e1 = e0 + 1u;
          auto wave_of = [](uint32_t e) { return (e / (W * kItemClasses)) * W + (e % W); };
          const uint32_t a = wave_of(e0) < nw ? lclass[e0] : 0u, b = wave_of(e1) < nw ? lclass[e1] : 0u;
          uint32_t inc = a + b;
#pragma unroll
          for (uint32_t dlt = 1; dlt < 64; dlt <<= 1) {
            const uint32_t y = __shfl_up(inc, dlt);
            if (lane >= dlt) inc += y;
          }
          lclass[e0] = inc - a - b;
          lclass[e1] = inc - b;
        }
        __syncthreads();
        if (tid < n) {
          const uint32_t pos = lclass[entry(wave, cls)] + rank;
          ltile[pos] = rec;
          lcount[pos] = c;
        }
        __syncthreads();
        c = tid < n ? lcount[tid] : 0u;
      }
      uint32_t x = c;  // inclusive scan of the lane counts: within the wave, then over the waves' totals
#pragma unroll
      for (uint32_t dlt = 1; dlt < 64; dlt <<= 1) {
        const uint32_t y = __shfl_up(x, dlt);
        if (lane >= dlt) x += y;
      }
      if (lane == 63) lwave[wave] = x;
      __syncthreads();
      uint32_t before = 0;
      for (uint32_t w = 0; w < wave; ++w) before += lwave[w];
      lstart[tid + 1] = before + x;
      if (tid == 0) lstart[0] = 0;
      __syncthreads();
      const uint32_t total = lstart[n];
      for (uint32_t v = tid; v < total; v += nthr) {
        uint32_t lo = 0, hi = n;  // the tile j with lstart[j] <= v < lstart[j + 1]
        while (hi - lo > 1) {
          const uint32_t mid = (lo + hi) >> 1;
          if (lstart[mid] <= v) lo = mid;
          else hi = mid;
        }
        const SmallTile st = ltile[lo];
        const uint32_t t0 = lstart[lo], cnt = lstart[lo + 1] - t0;
        if (CV && st.mode_glog == 0xffu) convert_rows<false>((gsrc_t)st.s, (gdst_t)st.d, st.ipr, st.body, st.p0, st.p1, v - t0, cnt);
        else small_tile_copy<CV ? kRoundConverting : kRound>(st, v - t0, cnt);
      }
      __syncthreads();  // the staging area is written again by the next slice or batch
    }
    // (the next batch, which may want the whole staging area, starts behind the caller's barrier)
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

template <bool TR, bool CV>
__global__ __launch_bounds__(kMaxThreads) void k_reshard(const TileDesc* __restrict__ heads, uint32_t n_batches,
                                                         const TileDesc* __restrict__ tiles, PtrArgs ptrs,
                                                         uint32_t n_src, uint32_t n_ptrs, unsigned long long* queue,
                                                         int persistent) {
  reshard_body<TR, CV>(heads, n_batches, tiles, ptrs.p, n_src, n_ptrs, queue, persistent);
}

template <bool TR, bool CV>
__global__ __launch_bounds__(kMaxThreads) void k_reshard_table(const TileDesc* __restrict__ heads, uint32_t n_batches,
                                                               const TileDesc* __restrict__ tiles,
                                                               const uint64_t* __restrict__ ptr_table, uint32_t n_src,
                                                               uint32_t n_ptrs, unsigned long long* queue,
                                                               int persistent) {
  reshard_body<TR, CV>(heads, n_batches, tiles, ptr_table, n_src, n_ptrs, queue, persistent);
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
  const uint32_t lds_bytes = (std::max(small_batch_lds_bytes((uint32_t)cfg.threads), plan.lds_transpose) + 15u) & ~15u;
  if (lds_bytes > kMaxDynamicLds) {
    set_error("the plan needs more LDS than a workgroup can have");
    return BCP_ERR_INVALID_ARG;
  }
  typedef void (*ArgKernel)(const TileDesc*, uint32_t, const TileDesc*, PtrArgs, uint32_t, uint32_t, unsigned long long*, int);
  typedef void (*TableKernel)(const TileDesc*, uint32_t, const TileDesc*, const uint64_t*, uint32_t, uint32_t,
                              unsigned long long*, int);
  // instances by [transposed tiles][converting tiles]
  static const ArgKernel arg_kernel[2][2] = {{k_reshard<false, false>, k_reshard<false, true>},
                                             {k_reshard<true, false>, k_reshard<true, true>}};
  static const TableKernel table_kernel[2][2] = {{k_reshard_table<false, false>, k_reshard_table<false, true>},
                                                 {k_reshard_table<true, false>, k_reshard_table<true, true>}};
  static const hipError_t lds_attr = [] {
    const void* fns[8];
    for (int i = 0; i < 4; ++i) {
      fns[i] = reinterpret_cast<const void*>(arg_kernel[i >> 1][i & 1]);
      fns[4 + i] = reinterpret_cast<const void*>(table_kernel[i >> 1][i & 1]);
    }
    for (const void* f : fns) {
      const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxDynamicLds);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }();
  BCP_HIP(lds_attr);
  const int tr = plan.lds_transpose != 0, cv = plan.converts;
  const dim3 g(grid), b((unsigned)cfg.threads);
  if (!table) {
    PtrArgs args;
    for (int32_t i = 0; i < n_src; ++i) args.p[i] = (uint64_t)(uintptr_t)src[i];
    for (int32_t i = 0; i < n_dst; ++i) args.p[n_src + i] = (uint64_t)(uintptr_t)dst[i];
    for (uint32_t i = n_ptrs; i < (uint32_t)kArgPtrs; ++i) args.p[i] = 0;
    hipLaunchKernelGGL(arg_kernel[tr][cv], g, b, lds_bytes, stream, plan.heads,
                       (uint32_t)plan.n_batches, plan.tiles, args, (uint32_t)n_src, n_ptrs, plan.queue,
                       cfg.persistent);
  } else {
    hipLaunchKernelGGL(table_kernel[tr][cv], g, b, lds_bytes, stream, plan.heads,
                       (uint32_t)plan.n_batches, plan.tiles, (const uint64_t*)table, (uint32_t)n_src, n_ptrs,
                       plan.queue, cfg.persistent);
  }
  BCP_HIP(hipGetLastError());
  return BCP_OK;
}

// ---- the variant that allocates nothing ----------------------------------------------------------
// Queue words and pointer table of a launch in a static array in device memory: [4 queue words, padded
// to 256 bytes | BCP_NOALLOC_MAX_BUFFERS pointers].  Each GPU holds its own copy at its own address,
// looked up once per device; host code only ever uses that address, never the array's name.
namespace {
constexpr size_t kScratchQueueBytes = 256;
constexpr size_t kScratchBytes = kScratchQueueBytes + sizeof(uint64_t) * BCP_NOALLOC_MAX_BUFFERS;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_addr[kMaxDevices];  // per device, null until looked up

// the current device's copy of the array
bcp_status scratch_address(void** out) {
  int dev = -1;
  BCP_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) {
    set_error("device index beyond the static scratch table");
    return BCP_ERR_INVALID_ARG;
  }
  std::lock_guard<std::mutex> g(g_scratch_mu);
  if (!g_scratch_addr[dev]) {
    void* p = nullptr;
    BCP_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) {
      set_error("hipGetSymbolAddress returned no address for the static scratch array");
      return BCP_ERR_HIP;
    }
    g_scratch_addr[dev] = p;
  }
  *out = g_scratch_addr[dev];
  return BCP_OK;
}

// table[base + i] = chunk.p[i] for i < n; with `queue` also puts the queue words back to zero (a fill
// kernel rather than a memset node, so that the sequence may be recorded into a HIP graph)
__global__ __launch_bounds__(kArgPtrs) void k_scratch_store(uint64_t* __restrict__ table, PtrArgs chunk, uint32_t base,
                                                            uint32_t n, unsigned long long* queue) {
  const uint32_t i = threadIdx.x;
  if (i < n) table[base + i] = chunk.p[i];
  if (queue && i < 4) queue[i] = 0ull;
}
}  // namespace

bcp_status launch_reshard_noalloc(const PlanDevice& plan, const void* const* src, int32_t n_src, void* const* dst,
                                  int32_t n_dst, hipStream_t stream) {
  if (plan.n_batches == 0) return BCP_OK;
  if ((int64_t)n_src + n_dst > BCP_NOALLOC_MAX_BUFFERS) {
    set_error("bcp_reshard_noalloc: the plan uses " + std::to_string((int64_t)n_src + n_dst) +
              " buffers, the static pointer table holds " + std::to_string(BCP_NOALLOC_MAX_BUFFERS));
    return BCP_ERR_INVALID_ARG;
  }
  void* base = nullptr;
  if (bcp_status s = scratch_address(&base)) return s;
  unsigned long long* queue = reinterpret_cast<unsigned long long*>(base);
  uint64_t* table = reinterpret_cast<uint64_t*>(static_cast<char*>(base) + kScratchQueueBytes);
  const int32_t n_ptrs = n_src + n_dst;
  for (int32_t first = 0; first < n_ptrs || first == 0; first += kArgPtrs) {
    PtrArgs args;
    const int32_t n = std::min<int32_t>(kArgPtrs, n_ptrs - first);
    for (int32_t i = 0; i < kArgPtrs; ++i) {
      const int32_t j = first + i;
      args.p[i] = i >= n ? 0 : (uint64_t)(uintptr_t)(j < n_src ? src[j] : dst[j - n_src]);
    }
    hipLaunchKernelGGL(k_scratch_store, dim3(1), dim3(kArgPtrs), 0, stream, table, args, (uint32_t)first, (uint32_t)n,
                       first == 0 ? queue : nullptr);
    BCP_HIP(hipGetLastError());
  }
  PlanDevice view = plan;  // same tiles and batches, the queue words of the static array
  view.queue = queue;
  return launch_reshard(view, nullptr, n_src, nullptr, n_dst, table, stream, nullptr);
}

}  // namespace bcp
