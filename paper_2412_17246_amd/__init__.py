"""MI355X-native single-GPU share of live, layer-level model scaling: layer-by-layer weight ingest
from pinned host memory overlapped with execution of the resident layer prefix, with activation
hand-off at a layer boundary.  All compute lives in the HIP library under csrc/; this package is
its ctypes binding."""
from .binding import (  # noqa: F401
    BZ_FLAG_DRY_RUN,
    BZ_RUN_NOWAIT,
    BZ_ZZ_BEST_EFFORT,
    BZ_ZZ_ZIGZAG,
    Scheduler,
    zz_simulate,
    Batch,
    BzError,
    Instance,
    KERNEL_CLASSES,
    SIGNATURES,
    TENSOR_ORDER,
    load_library,
    make_config,
    op_gemm,
    op_gemm_static,
    op_gemm_workspace_bytes,
    op_rmsnorm,
    plan_generate,
)
