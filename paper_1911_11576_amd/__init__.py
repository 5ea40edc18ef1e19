"""Stitched fusion-group kernels for MI355X (gfx950) behind a small C ABI.

`binding` mirrors include/fs.h; `build` compiles the HIP sources into
libfusionstitch.so in this directory.  Importing the package loads nothing: the
library is opened on the first call and that call fails loudly if it is missing.
"""
from .binding import (BoundArgs, FsError, FusedProgram, FusionPlan, Plan, fs_destroy, fs_last_error, fs_launch, fs_launch_static, fs_plan_create,  # noqa: F401
                      fs_plan_describe, fs_plan_info, fs_plan_tune, fs_shared_plan, fs_stream_copy, fs_group_key,
                      fs_tune_cache_clear, fs_tune_cache_load, fs_tune_cache_save, fs_tune_cache_size,
                      fs_kernel_cache_dir, fs_kernel_cache_drop_memory, fs_kernel_cache_stats)
