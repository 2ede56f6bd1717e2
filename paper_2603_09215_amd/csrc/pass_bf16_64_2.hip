// Persistent layer-pass kernel for bf16_t weights, head_dim 64, 2 query heads per KV head.
#include "pass_launch.h"
namespace spark {
SPARK_DEFINE_PASS(launch_pass_bf16_64_2, bf16_t, 64, 2)
}  // namespace spark
