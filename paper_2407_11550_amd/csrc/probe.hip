// A plain streaming read of a buffer: the reference the scoring sweeps are compared with.
// No step of the method: it only shows what a kernel that does nothing but read reaches on the
// machine at hand, on the same buffers, in the same launch shape class (long-running
// workgroups, 16 bytes per lane, 64-lane rows of 1 KiB).
#include "common.h"

namespace adakv {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int PROBE_THREADS = 256;
constexpr int PROBE_UNROLL = 4;

__global__ __launch_bounds__(PROBE_THREADS) void probe_read_kernel(const u32x4 *__restrict__ src,
                                                                    long long n16,
                                                                    u32x4 *__restrict__ sink) {
  const long long stride = (long long)gridDim.x * PROBE_THREADS;
  long long i = (long long)blockIdx.x * PROBE_THREADS + threadIdx.x;
  u32x4 acc = {0u, 0u, 0u, 0u};
  // PROBE_UNROLL independent loads in flight per lane, then the ragged rest
  for (; i + (PROBE_UNROLL - 1) * stride < n16; i += PROBE_UNROLL * stride) {
    u32x4 v[PROBE_UNROLL];
#pragma unroll
    for (int u = 0; u < PROBE_UNROLL; ++u) v[u] = src[i + u * stride];
#pragma unroll
    for (int u = 0; u < PROBE_UNROLL; ++u) acc ^= v[u];
  }
  for (; i < n16; i += stride) {
    acc ^= src[i];
  }
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
