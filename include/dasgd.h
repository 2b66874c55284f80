/* dasgd.h -- C ABI of the DaSGD per-step parameter pipeline for one MI355X (gfx950).
 *
 * DaSGD = Local SGD with delayed averaging.  W worker replicas of one model (the paper's M
 * workers) live in the HBM of one GPU.  Every iteration k each replica takes a local
 * optimiser step; every tau iterations the replicas' weights are averaged in the
 * background; d iterations after an average was launched it is folded into every replica's
 * current weights (paper, Section 3.3.1, Eq. 2):
 *
 *     x_{k+1}^(m) = x_k^(m) - eta g(x_k^(m))                                   otherwise
 *     x_{k+1}^(m) = xi (x_k^(m) - eta g(x_k^(m)))
 *                   + (1 - xi) (1/M) sum_j [ x_{k-d}^(j) - eta g(x_{k-d}^(j)) ]    if (k+1-d) mod tau == 0
 *
 * The averaging (a network all-reduce in the paper) is an on-device W-way mean here, run on a
 * side stream so that it overlaps the following local steps (paper, Fig. 2 and Fig. 4).
 *
 * Conventions
 *   - All pointers named "device" point to GPU memory owned by the CALLER (allocated e.g. by
 *     PyTorch); the library allocates no device memory.  All pointer ARRAYS are host memory.
 *   - Streams are raw hipStream_t handles passed as void*; the caller owns them.
 *   - Every step call only enqueues work and returns; only dasgd_bind (set-up copies) and
 *     dasgd_destroy block the host (and dasgd_local_step when the gradient pointer table has changed
 *     four times while the GPU still works on the oldest of them).
 *   - The library touches no byte outside the tensors, gradient buffers and workspace it is given.
 *   - A context is not thread-safe.  Functions return DASGD_OK or a negative error code and
 *     leave the context unchanged on error.
 *   - k denotes the 0-based index of the most recently completed local step.
 *
 * Canonical caller loop (one iteration of Eq. 2):
 *     dasgd_local_step(ctx, g);
 *     dasgd_query(ctx, &k, &n_pending, &begin_due, &merge_due);
 *     if (begin_due) dasgd_average_begin(ctx);     // (k+1) mod tau == 0
 *     if (merge_due) dasgd_merge(ctx);             // an average launched at k-d is pending
 *
 * Accuracy.  Results agree with a double-precision evaluation of Eq. 2 to within 1e-5 of the weight
 * scale (per tensor: the larger of the rms of the weights and of their initial values) over runs of up
 * to 3000 steps with the default settings.  Single-precision rounding accumulates like the square root
 * of the step count (about 1.3e-7 sqrt(K) measured), so no fp32 implementation holds that bound much
 * beyond 5000 steps; see DASGD_SNAPSHOT_* for the one setting that spends part of this budget.
 *
 * Diagnostics, tuning knobs and test hooks (profiling, band lengths, layout inspection, dry runs) are
 * declared in dasgd_diag.h.
 */
#ifndef DASGD_H
#define DASGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dasgd_ctx dasgd_ctx;

enum {
    DASGD_OK     = 0,
    DASGD_EINVAL = -1,  /* bad argument: W<1, P<1, d<0, tau<1, non-finite or negative lr, momentum
                           outside [0,1), wd<0, xi outside [0,1], null pointer, sizes that do not add up */
    DASGD_ESTATE = -2,  /* call not legal in the current state (see each function) */
    DASGD_ENOMEM = -3,  /* workspace too small / host allocation failed */
    DASGD_EHIP   = -4   /* a HIP runtime call failed; code via dasgd_last_hip_error */
};

/* Schedules (dasgd_set_schedule).  All use the same kernels. */
enum {
    DASGD_SCHED_OVERLAP = 0, /* the W-way mean runs on the side stream, event-ordered, beside
                                whatever the caller enqueues on the main stream after this step's calls
                                (the next forward/backward pass -- the paper's point: averaging hidden
                                behind local work, Fig. 2 and Fig. 4).  The library's own kernels, which
                                all saturate HBM, wait for a mean in flight instead of competing with it.
                                The mean is dispatched about 20 us behind the caller's next kernel, so
                                that it fills the wave slots that kernel leaves free instead of taking
                                them first (dasgd_set_side_stream_head_start in dasgd_diag.h) */
    DASGD_SCHED_SERIAL  = 1, /* everything on the main stream in program order (no overlap) */
    DASGD_SCHED_NO_AVERAGE_TIMING_ONLY = 2, /* timing floor: no snapshot and no mean are run, the
                                merge reads whatever the slot holds.  RESULTS ARE MEANINGLESS. */
    DASGD_SCHED_OVERLAP_FREE = 3, /* side-stream mean with the full d local steps of slack: main-stream
                                kernels wait only for the average they read, so a mean may also run
                                beside the library's own local steps and merges */
    DASGD_SCHED_AUTO = 4     /* default: OVERLAP or SERIAL, whichever is faster in the caller's own loop.
                                Whether the side stream pays depends on what runs between two steps:
                                behind work that leaves wave slots free the mean disappears; beside
                                nothing, or beside a kernel that fills every SIMD (one large GEMM), the
                                two cross-stream hand-overs per step only cost time (measured on MI355X:
                                1-2 % of the step).  After a warm-up of 16 steps (rounded to whole
                                averaging periods, like the phases; longer while band lengths are still
                                being measured, see dasgd_diag.h) the library alternates the two
                                schedules in six phases of 8 steps, marks the phase boundaries with
                                events on main_stream -- so the caller's own work is inside the
                                measurement; each mark is recorded after main_stream has been made to
                                wait for the means still on the side stream, so that a mean counts in
                                the phase that launched it -- and keeps the schedule with the smaller total once the
                                marks have completed (seen by a non-blocking query at a later step).
                                Results do not depend on the choice.  A caller that captures the step
                                calls into a HIP graph sets a fixed schedule first (event queries are
                                illegal while capturing) */
};

/* How much of one iteration is fused into the local-step kernel (dasgd_set_fusion).  Results are the
 * same at every level up to floating-point rounding of the same operations; only traffic differs. */
enum {
    DASGD_FUSE_NONE       = 0, /* the local step stores x, v (and the snapshot when an average follows);
                                  the merge reads x, writes x */
    DASGD_FUSE_SNAPSHOT   = 1, /* when a snapshot AND a merge fall on the same step, the local step stores
                                  the new weights only into the snapshot and the merge reads them there */
    DASGD_FUSE_STEP_MERGE = 2, /* when a merge is due at the step being taken (and d > 0), the local
                                  step applies it in the same pass (Eq. 2, both branches at once) and
                                  dasgd_merge only retires the average; otherwise as DASGD_FUSE_SNAPSHOT */
    DASGD_FUSE_ALL        = 3, /* the mean is computed by the local-step kernel too (a workgroup updates a
                                  window of columns of all W replicas and sums the new values through
                                  LDS): no snapshot, no mean kernel, nothing on the side stream;
                                  dasgd_average_begin and dasgd_merge only keep the books.  What one GPU
                                  can do when the average need not be a separate, overlappable operation.
                                  Needs d > 0 and either W = 2, 4, 8 or 16 (any memory layout) or the rows
                                  layout (see dasgd_local_step) for x, v and g (any W <= 32); otherwise
                                  behaves as DASGD_FUSE_STEP_MERGE */
    DASGD_FUSE_AUTO       = 4  /* default: DASGD_FUSE_STEP_MERGE, with the mean a kernel of its own that the
                                  overlap schedule can put on the side stream -- except on steps where a
                                  snapshot would have to be STORED (DASGD_SNAPSHOT_COPY, or
                                  DASGD_SNAPSHOT_AUTO after its step budget or below its xi limit) while the
                                  schedule in force is DASGD_SCHED_SERIAL (set, or chosen by
                                  DASGD_SCHED_AUTO): the mean would run in line anyway, so those steps take
                                  the DASGD_FUSE_ALL kernel (W = 2, 4, 8 or 16, d > 0; any memory layout), which
                                  gives the same bits as snapshot store + mean for 20+8/W instead of 28+8/W
                                  bytes per replica-parameter.  Results never depend on it */
};

/* Where the average finds the weights it averages (dasgd_set_snapshot). */
enum {
    DASGD_SNAPSHOT_COPY      = 0, /* the local-step kernel stores them into a snapshot buffer (an extra
                                     4 bytes per element); the mean may then take its full d steps */
    DASGD_SNAPSHOT_ZERO_COPY = 1, /* the live weights are the snapshot.  The mean reads x itself and the
                                     next kernel that writes x waits for it.  On a step that also merges
                                     an older average A (folded into the local step, so that x already
                                     holds x' = xi y + (1 - xi) A), the mean of the y is recovered as
                                     (mean x' - (1 - xi) A) / xi: same quantity, but the fp32 rounding of
                                     the x' enters it amplified by 1/xi.  RUN-LENGTH LIMIT: measured
                                     against a double-precision run the deviation grows like 2.2e-7
                                     sqrt(K) of the weight scale at xi = 0.25 (1.3e-7 sqrt(K) with stored
                                     snapshots) and reaches 1e-5 near K = 2000 steps; the extra term
                                     scales with 1/xi.  The library's own kernels wait for the mean; a
                                     caller whose OWN kernels write x between two steps (clipping,
                                     loading a checkpoint) must first wait for side_stream, or use the
                                     copy mode.  Taken when: schedule OVERLAP, SERIAL or AUTO; fusion level 2 or AUTO;
                                     and either no merge falls on the step or xi >= 1/8 (any memory
                                     layout: the mean finds the live weights through row pointers or through
                                     the record table).  Otherwise the copy is made */
    DASGD_SNAPSHOT_AUTO      = 2  /* default: zero-copy for the first 500 min(1, (xi / 0.25)^2) steps of
                                     the context (none for xi < 1/8), stored snapshots from then on, so
                                     that the accuracy statement at the top of this file holds whatever
                                     the run length: the reconstruction's extra rounding is spent while
                                     the accumulated error is still small.  (With DASGD_FUSE_AUTO and the
                                     serial schedule "stored snapshots" become the one-kernel step, which
                                     gives the same bits and stores none) */
};

/* Kernel kinds, for dasgd_profile_read and dasgd_band (dasgd_diag.h). */
enum {
    DASGD_K_LOCAL_STEP         = 0, /* local step storing x, v                      (20 B per element) */
    DASGD_K_LOCAL_STEP_SNAP    = 1, /* local step storing x, v and the snapshot     (24 B per element) */
    DASGD_K_MEAN               = 2, /* W-way replica mean                            (4 + 4/W)         */
    DASGD_K_MERGE              = 3, /* delayed merge                                 (8 + 4/W)         */
    DASGD_K_LOCAL_STEP_TO_SNAP = 4, /* local step storing v and the snapshot only   (20 B per element) */
    DASGD_K_STEP_MERGE         = 5, /* local step with the merge folded in          (20 + 4/W)        */
    DASGD_K_STEP_SNAP_MERGE    = 6, /* ... that also stores the snapshot             (24 + 4/W)        */
    DASGD_K_STEP_MEAN          = 7, /* local step that also computes the mean        (20 + 4/W)        */
    DASGD_K_STEP_MEAN_MERGE    = 8, /* local step with mean and merge folded in      (20 + 8/W)        */
    DASGD_K_MEAN_RECONSTRUCT   = 9, /* W-way mean of the live weights, merge undone  (4 + 8/W)         */
    DASGD_K_COUNT              = 10
};

/* Create a context for W replicas of P fp32 parameters each.
 *   d    delay in local steps between launching an average and merging it (d >= 0; the paper
 *        analyses d < tau, Section 4.3; any d is accepted: floor(d/tau)+1 averages in flight)
 *   tau  local steps between two averages (tau >= 1)
 *   lr, momentum, wd   learning rate eta (>= 0, finite), heavy-ball momentum in [0,1), coupled
 *        L2 weight decay (>= 0)  (Section 4.1 gives the constants 0.9 and 0.01)
 * xi, the local update proportion of Eq. 2, starts at 0.25 (the only value the paper prints,
 * Section 4.3); change it with dasgd_set_xi.  Host-only: needs no GPU.
 * Returns NULL on invalid arguments or allocation failure. */
dasgd_ctx *dasgd_create(int W, int64_t P, int d, int tau, float lr, float momentum, float wd);

/* Set xi in [0,1] (Eq. 2: weight of the local value at a merge).  Takes effect from the next local
 * step (whose kernel may already apply that step's merge); call it between whole iterations. */
int dasgd_set_xi(dasgd_ctx *ctx, float xi);

/* Set the learning rate (caller-side schedules; the paper's runs use a one-cycle policy,
 * Section 4.1).  Takes effect from the next local step. */
int dasgd_set_lr(dasgd_ctx *ctx, float lr);

/* Choose the schedule (DASGD_SCHED_*).  Only legal while no average is pending. */
int dasgd_set_schedule(dasgd_ctx *ctx, int schedule);

/* Choose the fusion level (DASGD_FUSE_*).  Only legal while no average is pending. */
int dasgd_set_fusion(dasgd_ctx *ctx, int fusion);

/* Choose where the average reads the weights (DASGD_SNAPSHOT_*).  Only legal while no average is pending. */
int dasgd_set_snapshot(dasgd_ctx *ctx, int mode);

/* Bytes of device workspace dasgd_bind needs for a model of n_tensors tensors with numel[t]
 * elements each (sum must equal P).  Holds the record and pointer tables, the snapshots
 * (floor(d/tau)+1 slots of W x P' floats) and the averages (same number of slots of P' floats),
 * where P' pads every tensor to a multiple of 64 elements, rounds up to 256 and adds 256.  Returns 0
 * on invalid arguments (also: a tensor of 2^32 elements or more, P' of 2^32 or more). */
size_t dasgd_workspace_bytes(const dasgd_ctx *ctx, int n_tensors, const int64_t *numel);

/* Bind the replicas' storage.
 *   numel      [n_tensors] host array, sum == P
 *   x, v       [W * n_tensors] host arrays of device pointers, replica-major (entry j*n_tensors+t is
 *              tensor t of replica j); each tensor contiguous fp32, at least 4-byte aligned
 *              (16-byte alignment selects the 128-bit path).  x: weights, updated in place.
 *              v: momentum buffers, updated in place; the caller zero-initialises them (v_0 = 0).
 *              All replicas are expected to start from the same weights (paper, Lemma 1); the
 *              library does not check it.
 *   workspace  device memory, 256-byte aligned, at least dasgd_workspace_bytes(...) bytes; its
 *              contents belong to the library until dasgd_destroy
 *   main_stream, side_stream   hipStream_t handles; local step and merge run on main_stream,
 *              the W-way mean on side_stream.  Must be different streams of equal priority.
 * Copies the tables to the device and clears snapshots/averages (blocks until done).
 * Every tensor and the workspace are checked against the extent of the device allocation that holds
 * them, where the HIP runtime knows it: a tensor or workspace that would run past the end of its
 * allocation is EINVAL (a kernel running past a buffer faults the GPU).  So is any overlap among the
 * x tensors, the v tensors and the workspace: all of them are written.
 * Errors: EINVAL, ENOMEM (workspace too small), ESTATE (already bound, or an earlier bind of this
 * context failed with EHIP: destroy it and create a new one), EHIP. */
int dasgd_bind(dasgd_ctx *ctx, int n_tensors, const int64_t *numel,
               float *const *x, float *const *v,
               void *workspace, size_t workspace_bytes,
               void *main_stream, void *side_stream);

/* Local step k -> k+1 on every replica (Eq. 2, first branch, with the optimiser of Section 4.1):
 *     g' = g + wd x ;  v <- momentum v + g' ;  x <- x - lr v
 * one fused kernel over all replicas and tensors on main_stream.  What else that kernel does depends
 * on the step and on the settings (DASGD_FUSE_*, DASGD_SNAPSHOT_*): when (k+1) mod tau == 0 it may
 * store the new weights into a snapshot slot for the average that dasgd_average_begin will launch;
 * when a merge is due at this same step (and d > 0) it applies that merge in the same pass, after a
 * device-side wait for the average, with the xi in effect now -- dasgd_merge then only retires the
 * average; at lower fusion levels it may leave the new weights only in the snapshot for
 * dasgd_merge to pick up.  What is guaranteed: x holds x_{k+1} once all calls of the canonical loop
 * for this step have been issued (in stream order), and not necessarily between them.
 *   g   [W * n_tensors] host array of device pointers (same order and shapes as x), read only;
 *       the buffers must stay valid and unchanged until the kernel has run.  NULL re-uses the
 *       pointers of the previous call (the table is re-uploaded only when it changes; four device
 *       copies are used in rotation, so a caller that changes it at every step can run at most three
 *       changes ahead of the GPU before this call waits).
 * Layout.  Rows: when every replica's tensors lie back to back in the order given, so that replica j
 * is ONE contiguous run of P floats starting at a 16-byte aligned address -- the rows of a W x ld
 * matrix with any row stride ld >= P, or one arena per replica at any addresses -- and P is a multiple of
 * 4 and W <= 32, the kernels take the W row addresses of x, v and g as arguments and need no table in
 * memory (fastest; a little faster still when the rows start on 1 KiB boundaries of the same phase for
 * x, v and g).  Only the P floats of each row are touched: padding between rows stays the caller's.
 * Records: any other arrangement (one allocation per tensor, odd sizes, unaligned tensors, W > 32) goes
 * through a table with one record per replica and 4096-float piece of a tensor; 128-bit accesses where
 * the piece's addresses are 16-byte aligned, 32-bit accesses otherwise.  x and v select the addressing
 * at dasgd_bind, g whenever its table changes (rows for x and v with any g is fine).  Results are
 * identical, bit for bit.
 * A changed gradient table is checked against its allocations like the tensors at dasgd_bind, and
 * against x, v and the workspace for shared bytes (EINVAL); gradient buffers may alias each other.
 * ESTATE: not bound; an average or a merge that fell due at the previous step was not issued. */
int dasgd_local_step(dasgd_ctx *ctx, const float *const *g);

/* Launch the average of the weights as they were right after the latest local step and before any
 * merge (Eq. 2's summand x - eta g; matrix form (X - eta G) J in the appendix): A = (1/W) sum_j y_j,
 * on side_stream after main_stream's local step, occupying a ring slot until merged.  The y_j are
 * read from the snapshot, or from the live weights (DASGD_SNAPSHOT_ZERO_COPY).  When a merge of
 * an older average is due at this same step, the launch is held back until that merge has been
 * enqueued (the mean has d steps of slack, the merge none), so that the mean runs beside the
 * caller's next forward/backward pass rather than beside the merge.
 * ESTATE: not due (legal exactly once after a local step k with (k+1) mod tau == 0). */
int dasgd_average_begin(dasgd_ctx *ctx);

/* Fold the oldest pending average into every replica (Eq. 2, second branch):
 *     x_j <- xi x_j + (1 - xi) A        computed as x_j + (1 - xi)(A - x_j)
 * on main_stream, after a device-side wait for that average; frees its slot.  If this step's own
 * average is still to be launched (see dasgd_average_begin) it is launched right behind the merge.
 * ESTATE: no pending average, or the oldest one was not launched at step k - d. */
int dasgd_merge(dasgd_ctx *ctx);

/* One whole iteration of Eq. 2, the canonical loop in a single call:
 *     dasgd_local_step(ctx, g); if begin due: dasgd_average_begin(ctx); if merge due: dasgd_merge(ctx);
 * *began / *merged (may be NULL) tell whether an average was launched / retired.  Errors as the three
 * calls; on an error of the second or third call the earlier ones have taken effect. */
int dasgd_step(dasgd_ctx *ctx, const float *const *g, int *began, int *merged);

/* Mean over the replicas of a W x P row-major matrix of gradients, out[i] = (1/W) sum_j G[j*P + i], on
 * main_stream with the W-way mean kernel: the reduction step of synchronous Mini-batch SGD in its
 * per-worker form, x_{k+1} = x_k - (eta/M) sum_j g_j (Section 2.1, Eq. 1), provided so that the
 * paper's comparison schedules (Mini-batch SGD, Local SGD as d = 0) can be timed on the same kernels.
 *   G    device, W*P floats, rows back to back, 16-byte aligned, read only;  P must be a multiple of 4
 *        (the sum is taken pairwise over the replicas for W <= 32, four rows at a time above)
 *   out  device, P floats, 16-byte aligned; may then be passed as every replica's gradient
 * EINVAL: null / misaligned pointer or P % 4 != 0.  ESTATE: not bound. */
int dasgd_gradient_average(dasgd_ctx *ctx, const float *G, float *out);

/* The blocking average in one call, without a context: A = (1/W) sum_j x_j, then x_j <- xi x_j + (1 - xi) A
 * for every replica -- Local SGD's averaging step (Section 2.3.3; "delay 0" in Section 4.3), for callers who
 * take their local steps with an optimiser of their own; with xi = 0 every replica becomes the averaged
 * model that the paper's analysis follows (Section 3.3.1), e.g. before evaluation or a checkpoint.  Two
 * kernels on `stream` (the W-way mean into the workspace, the merge out of it); returns without waiting.
 *   x_rows     host array of W device pointers; replica j is the P contiguous floats at x_rows[j]
 *              (16-byte aligned, P a multiple of 4, W <= 32), updated in place
 *   workspace  device, 256-byte aligned, at least P floats; holds A afterwards
 * Same arithmetic as dasgd_average_begin + dasgd_merge with d = 0 (pairwise sum over the replicas).
 * EINVAL: bad sizes, null / misaligned pointers, rows that overlap each other or the workspace, a row or
 * the workspace running past its allocation.  ENOMEM: workspace smaller than P floats.  EHIP: a launch
 * failed (code via dasgd_last_hip_error(NULL)). */
int dasgd_average_now(int W, int64_t P, float *const *x_rows, float xi, void *workspace, size_t workspace_bytes, void *stream);

/* dasgd_average_now for callers that cannot allocate device memory or hand any over -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc: the average goes to a scratch array that
 * is part of the library's device code (128 MiB per GPU, held from the first use of the library on that
 * GPU until the process ends) instead of a workspace.  The call allocates nothing and calls no allocating
 * routine; inputs, outputs, arithmetic and errors are those of dasgd_average_now, plus
 *   ENOMEM  P > 33,554,432 floats (the scratch array's size): use dasgd_average_now with a workspace.
 * All calls on one GPU share that GPU's scratch array: two calls whose kernels may run at the same time
 * (different streams, different threads) race; calls on one stream are ordered and safe.  Nothing in the
 * array needs clearing between calls: each call writes the P floats it then reads. */
int dasgd_average_now_static(int W, int64_t P, float *const *x_rows, float xi, void *stream);

/* The paper's guideline for the delay (Section 3.4, Eq. 3: the communication must fit into d local
 * iterations, t_c < d t_p) and for the period (Section 6.4: tau = d + 1): returns the smallest integer
 * d >= 1 with t_c < d * t_p, and tau = d + 1.  t_c: time of one weight averaging (>= 0), t_p: time of
 * one local iteration (> 0), any common unit.  Host-only.  EINVAL on non-finite or out-of-range input. */
int dasgd_choose_delay(double t_c, double t_p, int *d, int *tau);

/* Report the state: k (index of the last completed local step, -1 before the first), number of
 * pending averages, and whether dasgd_average_begin / dasgd_merge are due now.  Any output
 * pointer may be NULL. */
int dasgd_query(const dasgd_ctx *ctx, int64_t *step_k, int *n_pending, int *begin_due, int *merge_due);

/* HIP error code of the most recent DASGD_EHIP of this context (0 if none); with ctx == NULL: of the calling
 * thread's latest context-free call. */
int dasgd_last_hip_error(const dasgd_ctx *ctx);

/* Wait for both streams, drop pending averages, release events and host state.  NULL is a no-op. */
void dasgd_destroy(dasgd_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* DASGD_H */
