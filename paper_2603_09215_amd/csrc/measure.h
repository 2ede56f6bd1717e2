// Measurement support: a plain streaming read, the simplest reader of HBM there is.  Its rate is
// what the weight-streaming kernels can be compared with next to the published peak.
#pragma once
#include "device_common.h"

namespace spark {

constexpr int READ_THREADS = 256;
constexpr int READ_UNROLL = 8;   // 16-byte loads a thread has in flight

typedef unsigned int read_u32x4 __attribute__((ext_vector_type(4)));

// sink[block * (READ_THREADS / 64) + wave] = XOR of the words the wave has read.
// A wave reads READ_UNROLL consecutive KiB per trip (eight loads in flight that lie next to each
// other, as a weight row's segments do in the projection kernels), then jumps by the grid's span.
template <bool NT>
__global__ void __launch_bounds__(READ_THREADS)
read_stream_k(const read_u32x4 *__restrict__ p, size_t n16, unsigned *__restrict__ sink) {
  const size_t wave = (size_t)blockIdx.x * (READ_THREADS / 64) + (threadIdx.x >> 6);
  const size_t n_waves = (size_t)gridDim.x * (READ_THREADS / 64);
  const int lane = threadIdx.x & 63;
  read_u32x4 acc = {0u, 0u, 0u, 0u};
  size_t base = wave * (64 * READ_UNROLL);
  for (; base + 64 * READ_UNROLL <= n16; base += n_waves * (64 * READ_UNROLL)) {
    read_u32x4 v[READ_UNROLL];
#pragma unroll
    for (int u = 0; u < READ_UNROLL; ++u)
      v[u] = NT ? __builtin_nontemporal_load(p + base + u * 64 + lane) : p[base + u * 64 + lane];
#pragma unroll
    for (int u = 0; u < READ_UNROLL; ++u) acc ^= v[u];
  }
  // the ragged end: the trip that does not fit, vector by vector
  for (size_t i = base + lane; i < n16 && base < n16; i += 64) {
    if (i < base + 64 * READ_UNROLL) acc ^= NT ? __builtin_nontemporal_load(p + i) : p[i];
  }
  unsigned r = acc.x ^ acc.y ^ acc.z ^ acc.w;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) r ^= __shfl_xor(r, o, 64);
  if (lane == 0) sink[wave] = r;
}

}  // namespace spark
