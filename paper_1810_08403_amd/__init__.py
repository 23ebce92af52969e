"""MI355X-native SAGA-NN layer (NGra, arXiv 1810.08403): Python binding of libsaga.

The compute lives in hand-written HIP kernels behind the C ABI declared in
include/saga.h; this package only marshals arguments. Importing the package
does not load the library; the first call does, and fails loudly if it has
not been built.
"""
from .binding import (ACT, AGG, BF16, EDGE_OP, EXPORTS, F32, LIB_PATH, Context, Graph, SagaError, Timings,
                      load_library, plan_reencoding, plan_work_list, version)

__all__ = ["ACT", "AGG", "BF16", "EDGE_OP", "EXPORTS", "F32", "LIB_PATH", "Context", "Graph", "SagaError",
           "Timings", "load_library", "plan_reencoding", "plan_work_list", "version"]
