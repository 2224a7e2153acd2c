"""MI355X-native QEM mesh decimation (the decimation hot path of the Picasso paper).

``binding`` is the ctypes front end of the HIP library (include/picasso.h);
``meshgen`` holds the seeded synthetic inputs; ``build`` compiles the library.
Importing the package does not load the library; the first call does, and it
raises if the library is missing (there is no CPU fallback).
"""
from . import meshgen  # noqa: F401
from .binding import (  # noqa: F401
    Context, PicassoError, load_library, picasso_stats, picasso_strerror, picasso_workspace_bytes, picasso_device_copy,
    picasso_replace_mapping_static, PICASSO_STATIC_MAX_CLUSTERS,
    PICASSO_OK, PICASSO_WARN_BUDGET_UNMET, PICASSO_ERR_INVALID_ARG, PICASSO_ERR_BAD_INDEX,
    PICASSO_ERR_NONFINITE, PICASSO_ERR_WORKSPACE, PICASSO_ERR_HIP, PICASSO_ERR_INTERNAL,
    PICASSO_OPT_MAX_ROUNDS, PICASSO_OPT_STAGE_TIMING, PICASSO_OPT_SUBROUND_BATCH, PICASSO_OPT_KERNEL_TIMING, PICASSO_OPT_OVERLAP, PICASSO_OPT_TRUNC_BLOCK_MAX,
    PICASSO_OPT_PLACEMENT, PICASSO_OPT_RCOND_MIN_BITS, PICASSO_OPT_ABSORB, PICASSO_OPT_SHUFFLE_SEED, PICASSO_OPT_HOST_POLL, PICASSO_OPT_LAUNCH_AHEAD, PICASSO_OPT_TRUNC_WIDTH, PICASSO_OPT_DROP_DEGENERATED, PICASSO_OPT_TRUNC_SELECT, PICASSO_PLACE_MEAN, PICASSO_PLACE_INVERSE,
    PICASSO_POOL_AVG, PICASSO_POOL_MAX, PICASSO_POOL_WEIGHTED, PICASSO_POOL_SUM,
    PICASSO_KERNEL_SORT, PICASSO_KERNEL_UNIQUE_COST, PICASSO_KERNEL_SUBROUND0, PICASSO_KERNEL_FACET_INSERT,
    PICASSO_KERNEL_QUADRIC_ROWS, PICASSO_KERNEL_SORT_INCIDENCE, PICASSO_KERNEL_COUNT,
)
