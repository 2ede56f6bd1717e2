"""MI355X-native SPAR-K decoding: HIP kernels behind a C ABI (include/spark.h) and a thin binding."""
from .binding import Spark, SparkError, load_library, make_config  # noqa: F401
