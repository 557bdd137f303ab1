"""MI355X-native training hot path of a neural graph database (operator-level batching).

The compute lives in libngdb.so (HIP, gfx950); see include/ngdb.h for the C boundary.
"""
from .binding import (Engine, NgdbError, Plan, Sampler, plan_host, lib, load_library, LIB_PATH,  # noqa: F401
                      MLP_NAMES, TENSOR_NAMES)
