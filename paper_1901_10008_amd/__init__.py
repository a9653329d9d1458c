"""MI355X-native coalesced "superkernel" for multi-tenant low-batch inference.

Thin Python binding over the C ABI in include/superkernel.h.  All planning and
all arithmetic run in libsuperkernel.so (C++ planner + hand-written HIP kernels
for gfx950); this package only marshals arguments.  There is no CPU fallback:
if the library has not been built, importing the binding raises.
"""
from .binding import (  # noqa: F401
    SkError,
    Plan,
    PlanParams,
    lib,
    lib_path,
    make_problem,
    sk_plan_create,
    sk_plan_destroy,
    sk_launch,
    sk_launch_sequential,
    sk_launch_static,
    SK_STATIC_SCRATCH_BYTES,
    sk_plan_num_tiles,
    sk_plan_num_problems,
    sk_plan_get_tiles,
    sk_plan_get_order,
    sk_plan_get_ranges,
    sk_plan_get_xcd_lists,
    sk_plan_get_stamps,
    sk_plan_grid,
    sk_plan_params_default,
    sk_release_cached_memory,
    sk_strerror,
    sk_last_error,
    SK_F32, SK_BF16, SK_F16, SK_GEMM, SK_CONV2D_NHWC, SK_CONV2D_NCHW,
    DTYPE_CODE,
    SK_OK, SK_ERR_INVALID_ARG, SK_ERR_UNSUPPORTED, SK_ERR_OVERLAP, SK_ERR_ALLOC, SK_ERR_HIP, SK_ERR_BUSY, SK_ERR_STATE,
    EXPORTED_SYMBOLS,
    Queue, QueueParams, QueueStats, sk_completion, sk_problem,
    sk_queue_params_default, sk_queue_create, sk_queue_submit, sk_queue_poll, sk_queue_get_stats, sk_queue_destroy,
    SK_QUEUE_SEQUENTIAL, SK_QUEUE_COALESCE, SK_QUEUE_OOO, QUEUE_POLICY,
)
