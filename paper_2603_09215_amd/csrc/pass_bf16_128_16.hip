// Persistent layer-pass kernel for bf16_t weights, head_dim 128, 16 query heads per KV head.
#include "pass_launch.h"
namespace spark {
SPARK_DEFINE_PASS(launch_pass_bf16_128_16, bf16_t, 128, 16)
}  // namespace spark
