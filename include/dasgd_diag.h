/* dasgd_diag.h -- diagnostics, tuning knobs and test hooks of the DaSGD parameter pipeline.
 *
 * Nothing here is part of the method (the paper's update rule and its schedule are in dasgd.h); these
 * calls let tests, the benchmark and curious callers look inside a context, time its kernels and
 * override what it would otherwise measure for itself.  Same conventions and error codes as dasgd.h.
 */
#ifndef DASGD_DIAG_H
#define DASGD_DIAG_H

#include "dasgd.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Addressing in use (dasgd_layout). */
enum {
    DASGD_ADDR_RECORDS = 0,  /* record table for every kernel */
    DASGD_ADDR_ROWS    = 1,  /* row pointers in the kernel arguments (x, v and the current g are rows) */
    DASGD_ADDR_ROWS_XV = 2   /* x and v are rows, the current gradient table is not: the local step goes
                                through the record table, merge and mean use the rows */
};

/* Work maps dasgd_check_work_map knows. */
enum {
    DASGD_MAP_ROWS      = 0, /* columns of one row over the (band, workgroup, lane) grid of the row kernels */
    DASGD_MAP_MEAN      = 1, /* column windows of the mean kernels, plain order */
    DASGD_MAP_MEAN_RUNS = 2  /* ... in runs of eight windows per L2 partition */
};

/* Bind shapes only: every later step call runs the host-side state machine (step counter,
 * pending-average ring, due/overdue checks, error codes) and launches NOTHING on any device.
 * For testing schedules and error handling on machines without a GPU; computes nothing. */
int dasgd_bind_dry_run(dasgd_ctx *ctx, int n_tensors, const int64_t *numel);

/* In the overlap schedules a mean that reads and writes fewer than `bytes` bytes ((W+1) rows of fp32)
 * is launched on main_stream after all: handing work to the side stream and back costs two
 * cross-stream waits of 6-10 us each on MI355X, more than so small a mean takes (at 6 TB/s, 64 MiB are
 * 11 us).  Default 64 MiB; 0 sends every mean to the side stream.  Results do not depend on it.
 * ESTATE while averages are pending or an average is due. */
int dasgd_set_side_stream_threshold(dasgd_ctx *ctx, size_t bytes);

/* A mean that goes to the side stream is held back by about `microseconds` (a one-wavefront kernel in
 * front of it that watches the constant clock), so that the kernel the caller enqueued on main_stream
 * behind the local step is dispatched first.  The order decides how the two share the chip: a kernel
 * already in place keeps its wave slots and the mean fills the rest; a mean dispatched first takes every
 * slot it can use and the caller's kernel starts only as the mean drains (measured on MI355X: a 0.75 ms
 * kernel took 0.96-1.08 ms behind a 0.16 ms mean that won the race by 0.3 us).  Without it the order is
 * a race that depends on how far the host runs ahead.  Default 20; 0 = none; at most 200 (EINVAL above).
 * Results do not depend on it.  May be changed at any time. */
int dasgd_set_side_stream_head_start(dasgd_ctx *ctx, unsigned microseconds);

/* Layout of the library-owned buffers inside the workspace and the addressing chosen at bind:
 * flat_offset[t] (may be NULL) = element offset of tensor t in a snapshot row / an average;
 * *P_padded = floats per such row: P rounded up to 256 when the replicas are rows (a snapshot row
 * mirrors a replica), otherwise every tensor padded to a multiple of 64 elements (rounded up to 256,
 * plus 256); *addressing = DASGD_ADDR_* (-1 for a dry run).  ESTATE if not bound. */
int dasgd_layout(const dasgd_ctx *ctx, int64_t *flat_offset, int64_t *P_padded, int *addressing);

/* Locate pending average number `which` (0 = oldest): its launch step and the byte offset of its
 * P_padded floats from the start of the workspace.  The data is complete once side_stream (or
 * main_stream in the serial schedule) has drained.  EINVAL if which is out of range. */
int dasgd_pending_average(const dasgd_ctx *ctx, int which, int64_t *launch_step, size_t *byte_offset);

/* Per-kernel timing.  every_n >= 1: bracket one launch in every_n of each kernel kind with timing
 * events on its own stream (at most max_records launches are recorded; later ones run untimed);
 * every_n == 0: stop.  An event pair costs a few microseconds on the stream. */
int dasgd_profile(dasgd_ctx *ctx, int every_n, int max_records);

/* Wait for both streams, then return, for kernel `kernel` (DASGD_K_*) since profiling was enabled
 * or last read: the summed duration of the timed launches, how many were timed, and how many were
 * launched in all; then reset the three.  Any output pointer may be NULL. */
int dasgd_profile_read(dasgd_ctx *ctx, int kernel, double *total_ms, int64_t *timed, int64_t *launched);

/* Work order of the kernels that read the average for every replica (folded local step, merge).  Their
 * grid is (8 B, W, bands): workgroups are dispatched x fastest, then y, then z and dealt round-robin to
 * the 8 L2 partitions, so a partition handles B = 2^log_band blocks (1 KiB per array each) of replica
 * 0, the same blocks of replica 1, ..., then the next band, and a band's piece of the average is read
 * from HBM once and from that L2 afterwards.  Which band length is fastest depends on P, W and on what
 * runs around the kernel (measured on MI355X: up to 8 % between lengths, with a different winner for
 * each benchmark shape), so by default the library measures it in place: the first 16 launches of
 * such a kernel rotate through five lengths (2^5, 2^8 ... 2^11, fitted to the row), three launches of
 * each bracketed by timing events on main_stream; finished events are collected without waiting at
 * later launches, and the fastest length is kept from then on.  The order never changes results: every
 * element is computed by the same arithmetic whichever workgroup handles it (bit-identical, tested).
 *   log_band  -1: measure (default);  0..11: use this length (fitted to the row length).
 * May be called at any time.  EINVAL outside -1..11.  A caller that captures the step calls into a HIP
 * graph fixes the length first (the measurement queries events, which a capturing stream forbids) --
 * for instance to the value dasgd_band reported after a few eager steps. */
int dasgd_set_band(dasgd_ctx *ctx, int log_band);

/* Band length in use for kernel `kernel` (DASGD_K_STEP_MERGE, DASGD_K_STEP_SNAP_MERGE or DASGD_K_MERGE):
 * *log_band = the fixed or measured value, -1 while the measurement is still running; *settled = 1
 * once it is final; *trials = timed trial launches issued so far for this kernel (0: it has not run
 * more than once yet).  Looks at finished timing events but never waits.  Any output pointer may be
 * NULL.  ESTATE if not bound. */
int dasgd_band(dasgd_ctx *ctx, int kernel, int *log_band, int *settled, int *trials);

/* What DASGD_SCHED_AUTO is doing: *schedule = the schedule in force (DASGD_SCHED_AUTO itself while the
 * measurement is still running), *settled = 1 once it is final (always 1 for a fixed schedule),
 * *overlap_ms / *serial_ms = the measured totals of the three phases each (0 until settled).  Never
 * waits.  Any output pointer may be NULL. */
int dasgd_schedule_in_use(const dasgd_ctx *ctx, int *schedule, int *settled, double *overlap_ms, double *serial_ms);

/* The six measured phases of DASGD_SCHED_AUTO in the order they ran (OVERLAP, SERIAL, OVERLAP, ...),
 * milliseconds each, written to phase_ms[0..5]; zeros until the measurement has settled. */
int dasgd_schedule_trial(const dasgd_ctx *ctx, float *phase_ms);

/* The extent check of dasgd_bind, for callers and tests: *bytes_to_end = number of bytes from p to the
 * end of the device allocation that holds it, as the HIP runtime knows it (a framework's caching
 * allocator may have carved p out of a larger allocation: the figure is an upper bound on what belongs
 * to the caller).  EINVAL if p is NULL or not inside an allocation the runtime knows. */
int dasgd_device_extent(const void *p, size_t *bytes_to_end);

/* Host-only self-check of the index arithmetic that decides which workgroup and lane touch which
 * kilobyte, with the very functions the kernels call.
 *   DASGD_MAP_ROWS: a row of row4 128-bit columns whose first column lies `head` (0..63) columns behind
 *     a 1 KiB boundary, over the grid the library would launch for band length 2^log_band (0..11): every
 *     column must be handled by exactly one lane, the one that keeps each wave on one aligned kilobyte.
 *     (row4 <= 2^27: the check itself needs a byte per column.)
 *   DASGD_MAP_MEAN, DASGD_MAP_MEAN_RUNS: the column windows of the mean kernels over their rounded-up
 *     grid must be a permutation that covers every window of the row (head, log_band ignored).
 * Returns 0 if so, 1..4 naming the violated property (past the end, wrong lane, handled twice, never
 * handled); EINVAL for arguments outside those ranges. */
int dasgd_check_work_map(int kind, int64_t row4, int head, int log_band);

#ifdef __cplusplus
}
#endif
#endif /* DASGD_DIAG_H */
