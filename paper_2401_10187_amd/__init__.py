"""Kron-Matmul for AMD MI355X: Y = X (F_1 (x) ... (x) F_N) by fused sliced multiplies in HIP.

The computation lives in libkronmatmul.so (C-ABI in include/kronmatmul.h); this package only
marshals arguments.  PyTorch supplies device memory and streams."""
from .binding import (  # noqa: F401
    KM_F32, KM_F64, KM_OK, KM_EINVAL, KM_ENOMEM, KM_ELAUNCH, KM_EUNSUPPORTED,
    KM_KERNEL_GENERIC, KM_KERNEL_FUSED, KM_KERNEL_MFMA, KM_KERNEL_SHUFFLE, KM_KERNEL_ROWS, KM_KERNEL_MFMA_ANY,
    KM_BUF_X, KM_BUF_Y, KM_BUF_WS0, KM_BUF_WS1,
    KM_OPT_KERNELS, KM_OPT_MAX_FUSE, KM_OPT_PROFILE, KM_OPT_PREFER_TILE, KM_OPT_PREFER_THREADS, KM_OPT_TILES_PER_WG, KM_OPT_PAIR_INTERLEAVE, KM_OPT_TILE_ORDER, KM_OPT_PREFER_INSTANCE, KM_OPT_INSTANCE_COUNT, KM_OPT_KEEP_MIB,
    KronMatmulError, kronmatmul, Prepared, workspace_size, prepare, plan, tune, cost, store_column, set_option, get_option,
    last_profile, mean_profile, clock_probe, release, status_string, kernel_name, lib, EXPORTS, LIB_PATH,
    KM_STATIC_SCRATCH_BYTES,
)
