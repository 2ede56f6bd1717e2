// Persistent layer-pass kernel for float weights, head_dim 64, 2 query heads per KV head.
#include "pass_launch.h"
namespace spark {
SPARK_DEFINE_PASS(launch_pass_f32_64_2, float, 64, 2)
}  // namespace spark
