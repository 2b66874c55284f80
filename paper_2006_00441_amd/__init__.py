"""DaSGD (Local SGD with delayed averaging) parameter pipeline for one MI355X.

The work is done by hand-written HIP kernels behind a C ABI (include/dasgd.h and dasgd_diag.h, built into
libdasgd.so); this package is the ctypes binding.  There is no CPU fallback: importing works
anywhere (the context's host-side state machine needs no GPU), but binding device memory and
stepping need the built library and a gfx950 GPU, and fail loudly otherwise.
"""
from .binding import (DaSGD, DasgdError, lib, library_path, choose_delay, average_now, average_now_static, check_work_map, device_extent, DASGD_OK, DASGD_EINVAL, DASGD_ESTATE,
                      DASGD_ENOMEM, DASGD_EHIP, SCHED_OVERLAP, SCHED_SERIAL, SCHED_NO_AVERAGE_TIMING_ONLY, SCHED_OVERLAP_FREE, SCHED_AUTO, SNAPSHOT_AUTO, ADDR_RECORDS, ADDR_ROWS, ADDR_ROWS_XV, MAP_ROWS, MAP_MEAN, MAP_MEAN_RUNS,
                      K_LOCAL_STEP, K_LOCAL_STEP_SNAP, K_MEAN, K_MERGE, K_LOCAL_STEP_TO_SNAP, K_STEP_MERGE, K_STEP_SNAP_MERGE,
                      FUSE_NONE, FUSE_SNAPSHOT, FUSE_STEP_MERGE, FUSE_ALL, FUSE_AUTO, SNAPSHOT_COPY, SNAPSHOT_ZERO_COPY,
                      K_STEP_MEAN, K_STEP_MEAN_MERGE, K_MEAN_RECONSTRUCT, KERNEL_NAMES, EXPORTS)

__all__ = ["DaSGD", "DasgdError", "lib", "library_path", "choose_delay", "average_now", "average_now_static", "check_work_map", "device_extent", "DASGD_OK", "DASGD_EINVAL", "DASGD_ESTATE",
           "DASGD_ENOMEM", "DASGD_EHIP", "SCHED_OVERLAP", "SCHED_SERIAL", "SCHED_NO_AVERAGE_TIMING_ONLY", "SCHED_OVERLAP_FREE", "SCHED_AUTO", "SNAPSHOT_AUTO", "ADDR_RECORDS", "ADDR_ROWS", "ADDR_ROWS_XV", "MAP_ROWS", "MAP_MEAN", "MAP_MEAN_RUNS",
           "K_LOCAL_STEP", "K_LOCAL_STEP_SNAP", "K_MEAN", "K_MERGE", "K_LOCAL_STEP_TO_SNAP", "K_STEP_MERGE", "K_STEP_SNAP_MERGE",
           "FUSE_NONE", "FUSE_SNAPSHOT", "FUSE_STEP_MERGE", "FUSE_ALL", "FUSE_AUTO", "SNAPSHOT_COPY", "SNAPSHOT_ZERO_COPY",
           "K_STEP_MEAN", "K_STEP_MEAN_MERGE", "K_MEAN_RECONSTRUCT", "KERNEL_NAMES", "EXPORTS"]
