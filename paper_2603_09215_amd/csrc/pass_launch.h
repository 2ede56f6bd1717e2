// Entry points of the per-shape translation units that hold the persistent layer-pass kernel
// (one .hip file per (element type, head_dim, query heads per KV head), so they compile in
// parallel).
#pragma once
#include <hip/hip_runtime.h>

#include "pass_kernel.h"

namespace spark {

// Launch spark_pass_k<WT, mt, HD, G> on `grid` resident workgroups.  On the first call per
// instantiation the dynamic-LDS limit is raised and the occupancy checked (returns
// hipErrorLaunchOutOfResources if a workgroup does not fit on a CU).
#define SPARK_DECLARE_PASS(NAME, WT) \
  hipError_t NAME(const PassParams<WT> &p, int mt, int grid, size_t lds, size_t lds_limit, hipStream_t stream);

SPARK_DECLARE_PASS(launch_pass_bf16_128_7, bf16_t)
SPARK_DECLARE_PASS(launch_pass_bf16_128_16, bf16_t)
SPARK_DECLARE_PASS(launch_pass_bf16_64_2, bf16_t)
SPARK_DECLARE_PASS(launch_pass_f32_64_2, float)

#define SPARK_DEFINE_PASS(NAME, WT, HD, G)                                                          \
  template <int MT>                                                                                 \
  static hipError_t NAME##_mt(const PassParams<WT> &p, int grid, size_t lds, size_t lds_limit,      \
                              hipStream_t stream) {                                                 \
    auto kern = spark_pass_k<WT, MT, HD, G>;                                                        \
    static bool configured = false;                                                                 \
    if (!configured) {                                                                              \
      hipError_t e = hipFuncSetAttribute((const void *)kern,                                        \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_limit); \
      if (e != hipSuccess) return e;                                                                \
      int occ = 0;                                                                                  \
      e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kern, PASS_THREADS, lds_limit);        \
      if (e != hipSuccess) return e;                                                                \
      if (occ < 1) return hipErrorLaunchOutOfResources;                                             \
      configured = true;                                                                            \
    }                                                                                               \
    kern<<<grid, PASS_THREADS, lds, stream>>>(p);                                                   \
    return hipGetLastError();                                                                       \
  }                                                                                                 \
  hipError_t NAME(const PassParams<WT> &p, int mt, int grid, size_t lds, size_t lds_limit,          \
                  hipStream_t stream) {                                                             \
    switch (mt) {                                                                                   \
      case 1: return NAME##_mt<1>(p, grid, lds, lds_limit, stream);                                 \
      case 2: return NAME##_mt<2>(p, grid, lds, lds_limit, stream);                                 \
      case 3: return NAME##_mt<3>(p, grid, lds, lds_limit, stream);                                 \
      default: return NAME##_mt<4>(p, grid, lds, lds_limit, stream);                                \
    }                                                                                               \
  }

}  // namespace spark
