"""S-STE 2:4 sparse linear-layer hot path for AMD MI355X (gfx950): Python binding of libsste.so.

The functions here have the names of the C entry points declared in ``include/sste.h`` and only
marshal arguments (pointers, sizes, strides, the current HIP stream); every step of the path runs in
the library's HIP kernels.  PyTorch provides device memory and streams, nothing else.  Importing
this package does not load the library; the first call does, and it fails loudly if the library
cannot be loaded.
"""
from .binding import (  # noqa: F401
    BF16,
    F8E4M3,
    F8E5M2,
    F32,
    PackBatch,
    SsteError,
    cast_fp8,
    UpdateBatch,
    compute_beta,
    BETA_MSE,
    BETA_L1,
    flip_count,
    library,
    linear_dgrad,
    linear_fwd,
    linear_fwd_ex,
    linear_fwd_act,
    linear_dgrad_act,
    ACT_GELU_TANH,
    ACT_NONE,
    AmaxHistory,
    linear_wgrad,
    linear_wgrad_noalloc,
    mvue_materialize,
    packed_buffers,
    project_pack,
    sgd_project_pack,
    timing_begin,
    timing_end,
    wgrad_plan_override,
    wgrad_workspace_bytes,
)
