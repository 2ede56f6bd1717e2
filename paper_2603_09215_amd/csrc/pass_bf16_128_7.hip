// Persistent layer-pass kernel for bf16_t weights, head_dim 128, 7 query heads per KV head.
#include "pass_launch.h"
namespace spark {
SPARK_DEFINE_PASS(launch_pass_bf16_128_7, bf16_t, 128, 7)
}  // namespace spark
