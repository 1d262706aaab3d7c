// Measurement aid of bench.py (python bench.py --memfloor): what the memory system of the GPU allows for
// copying very many small tiles -- tiles of a given size at random source positions, destinations packed back to
// back or random as well -- with one 16-byte item per lane and next to no address arithmetic.  It is the floor the
// copy kernel's small-tile path is compared with; it shares no code with the library and is not part of it.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstdint>
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef u32x4 u32x4_u __attribute__((aligned(1)));
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("%s: %s\n", #x, hipGetErrorString(e)); exit(1);} } while (0)
__device__ inline uint64_t mix(uint64_t x) { x ^= x >> 33; x *= 0xff51afd7ed558ccdull; x ^= x >> 33; x *= 0xc4ceb9fe1a85ec53ull; x ^= x >> 33; return x; }
// tile t: ipt items of 16 bytes; source at a random position (multiple of `gran`) inside [0, range), destination
// at t * ipt * 16 + doff
template <bool RAND_DST>
__global__ __launch_bounds__(256) void k_scatter(const char* __restrict__ src, char* __restrict__ dst, uint64_t n_items, uint32_t ipt,
                                                 uint64_t range, uint32_t gran, uint32_t doff) {
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; g < n_items; g += stride) {
    const uint64_t t = g / ipt;
    const uint32_t i = (uint32_t)(g - t * ipt);
    const uint64_t so = (mix(t) % (range / gran)) * gran + (uint64_t)i * 16;
    const uint64_t dof = RAND_DST ? (mix(t ^ 0x9e3779b97f4a7c15ull) % (range / gran)) * gran + (uint64_t)i * 16 + doff
                                  : t * ipt * 16 + (uint64_t)i * 16 + doff;
    const u32x4 v = *(const u32x4_u*)(src + so);
    *(u32x4_u*)(dst + dof) = v;
  }
}
int main() {
  const uint64_t bytes = 810ull << 20;  // payload
  const uint64_t cap = bytes + (64 << 20);
  char *s, *d;
  CK(hipMalloc(&s, cap)); CK(hipMalloc(&d, cap));
  CK(hipMemset(s, 1, cap)); CK(hipMemset(d, 0, cap));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  const uint32_t ipts[] = {2, 4, 18, 64, 1024};
  const uint32_t grans[] = {256, 16, 4};
  for (int rd = 0; rd < 2; ++rd)
  for (uint32_t ipt : ipts) for (uint32_t gran : grans) {
    const uint64_t n_items = bytes / 16 / ipt * ipt;
    const uint32_t doff = gran == 4 ? 4 : 0;
    float best = 1e9f;
    for (int rep = 0; rep < 4; ++rep) {
      CK(hipEventRecord(e0, 0));
      if (rd) hipLaunchKernelGGL(k_scatter<true>, dim3(256 * 8), dim3(256), 0, 0, s, d, n_items, ipt, bytes - ipt * 16, gran, doff);
      else hipLaunchKernelGGL(k_scatter<false>, dim3(256 * 8), dim3(256), 0, 0, s, d, n_items, ipt, bytes - ipt * 16, gran, doff);
      CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1));
      float ms; CK(hipEventElapsedTime(&ms, e0, e1)); if (ms < best) best = ms;
    }
    printf("dst %s  tile %5u B  granularity %3u B : %.3f ms  (%.0f GB/s one way)\n", rd ? "random" : "packed", ipt * 16, gran, best, n_items * 16 / best / 1e6);
    fflush(stdout);
  }
  return 0;
}
