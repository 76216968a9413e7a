// A plain streaming read of a buffer: the reference the scoring sweeps are compared with.
// No step of the method: it only shows what a kernel that does nothing but read reaches on the
// machine at hand, on the same buffers (16 bytes per lane, every workgroup one contiguous span).
#include "common.h"

namespace adakv {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int PROBE_THREADS = 256;
constexpr int PROBE_UNROLL = 8;

__global__ __launch_bounds__(PROBE_THREADS) void probe_read_kernel(const u32x4 *__restrict__ src,
                                                                    long long n16,
                                                                    u32x4 *__restrict__ sink) {
  // a workgroup reads one contiguous span, 4 KiB per step of its 256 lanes, PROBE_UNROLL steps
  // in flight: the fastest of the plain patterns tried on this part
  const long long per = (n16 + gridDim.x - 1) / gridDim.x;
  const long long b0 = (long long)blockIdx.x * per;
  const long long b1 = b0 + per < n16 ? b0 + per : n16;
  long long i = b0 + threadIdx.x;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (; i + (PROBE_UNROLL - 1) * PROBE_THREADS < b1; i += PROBE_UNROLL * PROBE_THREADS) {
    u32x4 v[PROBE_UNROLL];
#pragma unroll
    for (int u = 0; u < PROBE_UNROLL; ++u) v[u] = src[i + u * PROBE_THREADS];
#pragma unroll
    for (int u = 0; u < PROBE_UNROLL; ++u) acc ^= v[u];
  }
  for (; i < b1; i += PROBE_THREADS) acc ^= src[i];
  // one 16-byte word per wave leaves the chip
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    acc.x ^= __shfl_xor(acc.x, m);
    acc.y ^= __shfl_xor(acc.y, m);
    acc.z ^= __shfl_xor(acc.z, m);
    acc.w ^= __shfl_xor(acc.w, m);
  }
  if ((threadIdx.x & 63) == 0) sink[blockIdx.x * (PROBE_THREADS / 64) + (threadIdx.x >> 6)] = acc;
}

hipError_t launch_probe_read(const void *src, long long n16, void *sink, int blocks,
                             hipStream_t s) {
  ADAKV_LAUNCH("probe_read", probe_read_kernel, dim3(blocks), dim3(PROBE_THREADS), s,
               (const u32x4 *)src, n16, (u32x4 *)sink);
  return hipGetLastError();
}

int probe_waves_per_block() { return PROBE_THREADS / 64; }

}  // namespace adakv
