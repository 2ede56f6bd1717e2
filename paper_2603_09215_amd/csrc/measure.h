// Measurement support: a plain streaming read, the simplest reader of HBM there is.  Its rate is
// what the weight-streaming kernels can be compared with next to the published peak.
#pragma once
#include "device_common.h"

namespace spark {

constexpr int READ_THREADS = 256;
constexpr int READ_UNROLL = 8;   // 16-byte loads a thread has in flight

typedef unsigned int read_u32x4 __attribute__((ext_vector_type(4)));

// sink[block * (READ_THREADS / 64) + wave] = XOR of the words the wave has read
template <bool NT>
__global__ void __launch_bounds__(READ_THREADS)
read_stream_k(const read_u32x4 *__restrict__ p, size_t n16, unsigned *__restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * READ_THREADS;
  size_t i = (size_t)blockIdx.x * READ_THREADS + threadIdx.x;
  read_u32x4 acc = {0u, 0u, 0u, 0u};
  for (; i + (READ_UNROLL - 1) * stride < n16; i += READ_UNROLL * stride) {
    read_u32x4 v[READ_UNROLL];
#pragma unroll
    for (int u = 0; u < READ_UNROLL; ++u)
      v[u] = NT ? __builtin_nontemporal_load(p + i + u * stride) : p[i + u * stride];
#pragma unroll
    for (int u = 0; u < READ_UNROLL; ++u) acc ^= v[u];
  }
  for (; i < n16; i += stride) acc ^= NT ? __builtin_nontemporal_load(p + i) : p[i];
  unsigned r = acc.x ^ acc.y ^ acc.z ^ acc.w;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) r ^= __shfl_xor(r, o, 64);
  if ((threadIdx.x & 63) == 0) sink[blockIdx.x * (READ_THREADS / 64) + (threadIdx.x >> 6)] = r;
}

}  // namespace spark
