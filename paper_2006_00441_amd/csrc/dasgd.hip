// Host side of the DaSGD parameter pipeline: the C ABI declared in include/dasgd.h and
// include/dasgd_diag.h, the pending-average ring, and the stream/event schedule that lets the W-way
// mean run behind the following local steps (paper, Section 3 and Fig. 2: a worker hands its weights to
// the averaging and immediately continues; the result is applied d local steps later).
#include "context.hpp"
#include "tuning.hpp"
#include "launch.hpp"


// ------------------------------------------------------------------------------------------------
extern "C" {

dasgd_ctx *dasgd_create(int W, int64_t P, int d, int tau, float lr, float momentum, float wd)
{
    if (W < 1 || W > 65535 || P < 1 || d < 0 || tau < 1) return nullptr;
    if (!std::isfinite(lr) || lr < 0.f) return nullptr;
    if (!(momentum >= 0.f && momentum < 1.f)) return nullptr;
    if (!std::isfinite(wd) || wd < 0.f) return nullptr;
    dasgd_ctx *c = new (std::nothrow) dasgd_ctx();
    if (!c) return nullptr;
    c->W = W; c->P = P; c->d = d; c->tau = tau;
    c->lr = lr; c->momentum = momentum; c->wd = wd;
    c->slots = d / tau + 1;
    c->sched_tuner.phase_len = (std::max(8, 2 * tau) + tau - 1) / tau * tau;      // whole averaging periods
    return c;
}

int dasgd_set_xi(dasgd_ctx *c, float xi)
{
    if (!c || !(xi >= 0.f && xi <= 1.f)) return DASGD_EINVAL;
    c->xi = xi;
    return DASGD_OK;
}

int dasgd_set_lr(dasgd_ctx *c, float lr)
{
    if (!c || !std::isfinite(lr) || lr < 0.f) return DASGD_EINVAL;
    c->lr = lr;
    return DASGD_OK;
}

int dasgd_set_schedule(dasgd_ctx *c, int schedule)
{
    if (!c || schedule < DASGD_SCHED_OVERLAP || schedule > DASGD_SCHED_AUTO) return DASGD_EINVAL;
    if (!c->pending.empty() || begin_due(c)) return DASGD_ESTATE;
    c->schedule = schedule;
    return DASGD_OK;
}

int dasgd_set_side_stream_head_start(dasgd_ctx *c, unsigned microseconds)
{
    if (!c || microseconds > 200) return DASGD_EINVAL;
    c->head_start_us = microseconds;
    return DASGD_OK;
}

int dasgd_set_side_stream_threshold(dasgd_ctx *c, size_t bytes)
{
    if (!c) return DASGD_EINVAL;
    if (!c->pending.empty() || begin_due(c)) return DASGD_ESTATE;
    c->side_min_bytes = bytes;
    return DASGD_OK;
}

int dasgd_set_fusion(dasgd_ctx *c, int fusion)
{
    if (!c || fusion < DASGD_FUSE_NONE || fusion > DASGD_FUSE_AUTO) return DASGD_EINVAL;
    if (!c->pending.empty() || begin_due(c)) return DASGD_ESTATE;
    c->fusion = fusion;
    return DASGD_OK;
}

int dasgd_set_snapshot(dasgd_ctx *c, int mode)
{
    if (!c || mode < DASGD_SNAPSHOT_COPY || mode > DASGD_SNAPSHOT_AUTO) return DASGD_EINVAL;
    if (!c->pending.empty() || begin_due(c)) return DASGD_ESTATE;
    c->snapshot = mode;
    return DASGD_OK;
}

size_t dasgd_workspace_bytes(const dasgd_ctx *c, int n_tensors, const int64_t *numel)
{
    if (!shapes_ok(c, n_tensors, numel)) return 0;
    const Layout L = make_layout(c, n_tensors, numel);
    if (L.P_pad >= (1ll << 32)) return 0;
    return L.total;
}

static int bind_common(dasgd_ctx *c, int n_tensors, const int64_t *numel)
{
    if (!shapes_ok(c, n_tensors, numel)) return DASGD_EINVAL;
    if (make_layout(c, n_tensors, numel).P_pad >= (1ll << 32)) return DASGD_EINVAL;    // record offsets are 32-bit
    if (c->bound) return DASGD_ESTATE;
    if (c->g_pinned || !c->snap_done.empty()) return DASGD_ESTATE;     // an earlier bind failed half-way
    return DASGD_OK;
}

int dasgd_bind_dry_run(dasgd_ctx *c, int n_tensors, const int64_t *numel)
{
    int rc = bind_common(c, n_tensors, numel);
    if (rc != DASGD_OK) return rc;
    c->n_tensors = n_tensors;
    c->numel.assign(numel, numel + n_tensors);
    c->lay = make_layout(c, n_tensors, numel);
    c->dry = true;
    c->bound = true;
    return DASGD_OK;
}

int dasgd_bind(dasgd_ctx *c, int n_tensors, const int64_t *numel, float *const *x, float *const *v,
               void *workspace, size_t workspace_bytes, void *main_stream, void *side_stream)
{
    int rc = bind_common(c, n_tensors, numel);
    if (rc != DASGD_OK) return rc;
    if (!x || !v || !workspace) return DASGD_EINVAL;
    if (main_stream == side_stream) return DASGD_EINVAL;
    if (reinterpret_cast<uintptr_t>(workspace) % kAlign) return DASGD_EINVAL;
    const size_t rows = (size_t)c->W * (size_t)n_tensors;
    for (size_t r = 0; r < rows; ++r) {
        if (!x[r] || !v[r]) return DASGD_EINVAL;
        if ((reinterpret_cast<uintptr_t>(x[r]) | reinterpret_cast<uintptr_t>(v[r])) & 3u) return DASGD_EINVAL;
    }
    {
        DeviceRange lx, lv;
        for (size_t r = 0; r < rows; ++r) {
            const size_t bytes = sizeof(float) * (size_t)numel[r % (size_t)n_tensors];
            if (!range_ok(x[r], bytes, &lx) || !range_ok(v[r], bytes, &lv)) return DASGD_EINVAL;
        }
    }
    {   // x, v and the workspace are all written: none of them may share a byte with another.  (No kernel
        // touches a byte outside these ranges: what lies between or behind the caller's tensors is not ours.)
        std::vector<std::pair<uintptr_t, size_t>> iv;
        iv.reserve(2 * rows + 1);
        for (size_t r = 0; r < rows; ++r) {
            const size_t bytes = sizeof(float) * (size_t)numel[r % (size_t)n_tensors];
            iv.emplace_back(reinterpret_cast<uintptr_t>(x[r]), bytes);
            iv.emplace_back(reinterpret_cast<uintptr_t>(v[r]), bytes);
        }
        iv.emplace_back(reinterpret_cast<uintptr_t>(workspace), workspace_bytes);
        if (any_overlap(iv)) return DASGD_EINVAL;
        c->owned.swap(iv);                     // sorted by start, pairwise disjoint: gradient buffers are checked against it
    }
    const bool as_rows = is_rows(c, n_tensors, numel, x) && is_rows(c, n_tensors, numel, v);
    Layout L = make_layout(c, n_tensors, numel, as_rows);
    if (workspace_bytes < L.total) return DASGD_ENOMEM;
    if (!range_ok(workspace, L.total)) return DASGD_EINVAL;

    // records: one per replica and piece of a tensor
    std::vector<Rec> recs;
    recs.reserve((size_t)c->W * (size_t)L.n_pieces);
    for (int j = 0; j < c->W; ++j)
        for (int t = 0; t < n_tensors; ++t)
            for (int64_t off = 0; off < numel[t]; off += kPiece) {
                Rec r;
                r.x = x[(size_t)j * n_tensors + t] + off;
                r.v = v[(size_t)j * n_tensors + t] + off;
                r.aoff = (uint32_t)(L.foff[t] + off);
                r.goff = (uint32_t)off;
                r.len = (uint32_t)std::min<int64_t>(numel[t] - off, kPiece);
                r.tensor = (uint32_t)t;
                recs.push_back(r);
            }

    c->n_tensors = n_tensors;
    c->numel.assign(numel, numel + n_tensors);
    c->lay = L;
    c->xv_rows = as_rows;
    c->xr = RowSet{};
    c->vr = RowSet{};
    if (as_rows)
        for (int j = 0; j < c->W; ++j) { c->xr.p[j] = x[(size_t)j * n_tensors]; c->vr.p[j] = v[(size_t)j * n_tensors]; }
    c->ws = static_cast<char *>(workspace);
    c->main_s = static_cast<hipStream_t>(main_stream);
    c->side_s = static_cast<hipStream_t>(side_stream);

    HIPCHK(c, hipMemcpyAsync(c->ws + L.recs, recs.data(), sizeof(Rec) * recs.size(), hipMemcpyHostToDevice, c->main_s));
    // snapshots and averages start at zero (padding elements are averaged too and must stay finite)
    {
        const int64_t n4 = (int64_t)((L.total - L.S) / 16);
        const int64_t want = (n4 + kThreads - 1) / kThreads;
        const unsigned blocks = (unsigned)(want < 8192 ? (want < 1 ? 1 : want) : 8192);
        hipLaunchKernelGGL(k_fill_zero, dim3(blocks), dim3(kThreads), 0, c->main_s,
                           reinterpret_cast<v4f *>(c->ws + L.S), n4);
        HIPCHK(c, hipGetLastError());
    }
    HIPCHK(c, hipStreamSynchronize(c->main_s));

    c->snap_done.assign(c->slots, nullptr);
    c->avg_done.assign(c->slots, nullptr);
    HIPCHK(c, hipHostMalloc(&c->g_pinned, sizeof(void *) * rows * kGTables, hipHostMallocDefault));
    for (int b = 0; b < kGTables; ++b) HIPCHK(c, hipEventCreateWithFlags(&c->g_ev[b], hipEventDisableTiming));
    for (int s = 0; s < c->slots; ++s) {
        HIPCHK(c, hipEventCreateWithFlags(&c->snap_done[s], hipEventDisableTiming));
        HIPCHK(c, hipEventCreateWithFlags(&c->avg_done[s], hipEventDisableTiming));
    }
    c->dry = false;
    c->bound = true;
    return DASGD_OK;
}

// Launch the W-way mean for ring slot `slot`.  In the overlap schedules it goes to the side stream,
// ordered after everything enqueued on the main stream so far.  *on_side tells where it went.
static int launch_average(dasgd_ctx *c, int slot, bool *on_side)
{
    hipStream_t s = c->main_s;
    *on_side = side_stream_mean(c);
    if (*on_side) {
        HIPCHK(c, hipEventRecord(c->snap_done[slot], c->main_s));
        HIPCHK(c, hipStreamWaitEvent(c->side_s, c->snap_done[slot], 0));
        s = c->side_s;
        if (c->head_start_us) {
            hipLaunchKernelGGL(k_head_start, dim3(1), dim3(kWave), 0, s, c->head_start_us * 100u);
            HIPCHK(c, hipGetLastError());
        }
    }
    int rec;
    int rc = prof_open(c, c->zc && c->zc_recon ? DASGD_K_MEAN_RECONSTRUCT : DASGD_K_MEAN, s, &rec);
    if (rc != DASGD_OK) return rc;
    if (c->zc && !c->xv_rows) {
        // the replicas are not rows: the live weights are found through the records
        const Rec *recs = reinterpret_cast<const Rec *>(c->ws + c->lay.recs);
        const unsigned slots = (unsigned)((uint64_t)c->lay.n_pieces << kPieceLog);
        const float om = 1.0f - c->zc_xi, inv_xi = 1.0f / c->zc_xi, inv_w = 1.0f / (float)c->W;
        if (c->zc_recon)
            hipLaunchKernelGGL((k_mean_records<true>), dim3(slots), dim3(kWave), 0, s, recs, (unsigned)c->lay.n_pieces, slots, c->W,
                               avg_ptr(c, c->zc_old_slot), avg_ptr(c, slot), inv_w, om, inv_xi);
        else
            hipLaunchKernelGGL((k_mean_records<false>), dim3(slots), dim3(kWave), 0, s, recs, (unsigned)c->lay.n_pieces, slots, c->W,
                               static_cast<const float *>(nullptr), avg_ptr(c, slot), inv_w, om, inv_xi);
        HIPCHK(c, hipGetLastError());
    } else if (c->zc) {
        ConstRowSet rows = {};
        for (int j = 0; j < c->W; ++j) rows.p[j] = c->xr.p[j];
        if (c->zc_recon) {
            const unsigned row4 = (unsigned)(c->P / 4);
            const v4f *Ao = reinterpret_cast<const v4f *>(avg_ptr(c, c->zc_old_slot));
            v4f *An = reinterpret_cast<v4f *>(avg_ptr(c, slot));
            const float om = 1.0f - c->zc_xi, inv_xi = 1.0f / c->zc_xi, inv_w = 1.0f / (float)c->W;
            const dim3 grid(mean_grid(row4));
            if (rows_share_lines(rows, c->W))
                hipLaunchKernelGGL((k_mean_undo_merge<4, true>), grid, dim3(kWave * 4), 0, s, rows, Ao, An, row4, c->W, inv_w, om, inv_xi);
            else
                hipLaunchKernelGGL((k_mean_undo_merge<4, false>), grid, dim3(kWave * 4), 0, s, rows, Ao, An, row4, c->W, inv_w, om, inv_xi);
            HIPCHK(c, hipGetLastError());
        } else {
            rc = launch_mean(c, s, &rows, nullptr, 0, avg_ptr(c, slot), c->P);
            if (rc != DASGD_OK) return rc;
        }
    } else {
        // snapshot rows: P_pad floats each (tensor padding included: zero, averaged to zero)
        rc = launch_mean(c, s, nullptr, snap_ptr(c, slot), c->lay.P_pad, avg_ptr(c, slot), c->lay.P_pad);
        if (rc != DASGD_OK) return rc;
    }
    rc = prof_close(c, s, rec);
    if (rc != DASGD_OK) return rc;
    if (*on_side) HIPCHK(c, hipEventRecord(c->avg_done[slot], c->side_s));
    return DASGD_OK;
}

int dasgd_local_step(dasgd_ctx *c, const float *const *g)
{
    if (!c) return DASGD_EINVAL;
    if (!c->bound) return DASGD_ESTATE;
    if (begin_due(c) || merge_due(c)) return DASGD_ESTATE;          // unfinished business of step k
    const int64_t k = c->n_done;                                    // the step being taken
    const bool snap_step = ((k + 1) % c->tau) == 0;
    if (snap_step && (int)c->pending.size() >= c->slots) return DASGD_ESTATE;
    // will this very step end with a merge?  (d == 0: of the average it launches itself)
    const bool merge_follows = (c->d == 0) ? snap_step
                                           : (!c->pending.empty() && c->pending.front().launch_step == k - c->d);
    const size_t rows = (size_t)c->W * (size_t)c->n_tensors;

    // A changed gradient table is validated and staged first; the context adopts it only after the
    // kernel that uses it has been launched.
    bool g_changed = false, g_rows_new = c->g_rows;
    int g_buf = c->g_cur;
    ConstRowSet gr_new = c->gr;
    if (!c->dry) {
        if (!g && c->g_cur < 0) return DASGD_EINVAL;
        if (g) {
            for (size_t r = 0; r < rows; ++r)
                if (!g[r] || (reinterpret_cast<uintptr_t>(g[r]) & 3u)) return DASGD_EINVAL;
            g_changed = c->g_cur < 0 || std::memcmp(g, c->g_cached.data(), sizeof(void *) * rows) != 0;
            if (g_changed) {
                DeviceRange lg;
                for (size_t r = 0; r < rows; ++r) {
                    const size_t bytes = sizeof(float) * (size_t)c->numel[r % (size_t)c->n_tensors];
                    if (!range_ok(g[r], bytes, &lg)) return DASGD_EINVAL;
                    // a gradient buffer that shares bytes with x, v or the workspace would be overwritten while it is read
                    const uintptr_t a = reinterpret_cast<uintptr_t>(g[r]);
                    auto it = std::upper_bound(c->owned.begin(), c->owned.end(), std::make_pair(a, ~(size_t)0));
                    if (it != c->owned.end() && it->first < a + bytes) return DASGD_EINVAL;
                    if (it != c->owned.begin() && (it - 1)->first + (it - 1)->second > a) return DASGD_EINVAL;
                }
                g_rows_new = is_rows(c, c->n_tensors, c->numel.data(), g);
                gr_new = ConstRowSet{};
                if (g_rows_new)
                    for (int j = 0; j < c->W; ++j) gr_new.p[j] = g[(size_t)j * c->n_tensors];
                g_buf = (c->g_cur + 1) % kGTables;
            }
        }
    }

    const int sched = effective_schedule(c);
    c->sched_now = sched;
    const bool snap = snap_step && sched != DASGD_SCHED_NO_AVERAGE_TIMING_ONLY;
    // DASGD_FUSE_AUTO is level 2, raised to level 3 on the steps where that changes no bit (see below)
    const int fusion = c->fusion == DASGD_FUSE_AUTO ? DASGD_FUSE_STEP_MERGE : c->fusion;
    // fold the merge into this kernel?  (not for d == 0: that merge needs the mean of this step's own output)
    const bool fold = merge_follows && c->d > 0 && fusion >= DASGD_FUSE_STEP_MERGE;
    int mode = kStoreX;
    if (snap) mode = (merge_follows && !fold && fusion >= DASGD_FUSE_SNAPSHOT) ? kStoreS : kStoreXS;
    // zero-copy snapshot: store none, let the mean read x (see DASGD_SNAPSHOT_*)
    const bool zc_wanted = c->snapshot == DASGD_SNAPSHOT_ZERO_COPY ||
                           (c->snapshot == DASGD_SNAPSHOT_AUTO && k < zero_copy_budget(c->xi));
    const bool zc = snap && zc_wanted && fusion == DASGD_FUSE_STEP_MERGE &&
                    (sched == DASGD_SCHED_OVERLAP || sched == DASGD_SCHED_SERIAL) &&
                    (fold ? c->xi >= 0.125f : !merge_follows);
    if (zc) mode = kStoreX;
    bool all = false;               // everything in one kernel?

    if (!c->dry) {
        hipEvent_t phase_mark = nullptr;
        int rc = schedule_tick(c, &phase_mark);
        if (rc != DASGD_OK) return rc;
        if (g_changed) {
            // retire the table in use (all kernels reading it are already enqueued), take the next
            if (c->g_cur >= 0) {
                HIPCHK(c, hipEventRecord(c->g_ev[c->g_cur], c->main_s));
                c->g_ev_live[c->g_cur] = true;
            }
            if (c->g_ev_live[g_buf]) {
                HIPCHK(c, hipEventSynchronize(c->g_ev[g_buf]));      // its last reader ran kGTables-1 changes ago
                c->g_ev_live[g_buf] = false;
            }
            void *stage = static_cast<char *>(c->g_pinned) + sizeof(void *) * rows * (size_t)g_buf;
            std::memcpy(stage, g, sizeof(void *) * rows);
            HIPCHK(c, hipMemcpyAsync(c->ws + c->lay.gp[g_buf], stage, sizeof(void *) * rows, hipMemcpyHostToDevice, c->main_s));
        }
        const int slot = (int)(c->n_launched % c->slots);
        float *S = mode == kStoreX ? nullptr : snap_ptr(c, slot);
        const float *A = nullptr;
        const float om = 1.0f - c->xi;
        // Default overlap schedule: every kernel of this library saturates HBM, so letting a mean run
        // beside one only makes both slower; the local step therefore waits for the means in flight,
        // which leaves them whatever the caller put on the main stream since the last merge (the
        // forward/backward pass) to hide behind.  The free variant waits only for the average it reads.
        for (size_t p = 0; p < c->pending.size(); ++p) {
            Pending &pe = c->pending[p];
            const bool needed = fold && p == 0;
            if (!pe.on_side || pe.awaited || !(needed || sched != DASGD_SCHED_OVERLAP_FREE)) continue;
            HIPCHK(c, hipStreamWaitEvent(c->main_s, c->avg_done[pe.slot], 0));
            pe.awaited = true;
        }
        if (phase_mark) HIPCHK(c, hipEventRecord(phase_mark, c->main_s));
        if (fold) A = avg_ptr(c, c->pending.front().slot);
        const bool row_kernels = c->xv_rows && g_rows_new;
        // A snapshot that would have to be stored (no zero-copy on this step) under a schedule that runs the
        // mean in line anyway: the all-in-one kernel gives the same bits as store + mean (all fusion levels
        // agree with stored snapshots) for 20+8/W instead of 28+8/W bytes per replica-parameter.
        const bool raise = c->fusion == DASGD_FUSE_AUTO && !zc && sched == DASGD_SCHED_SERIAL &&
                           (c->W == 2 || c->W == 4 || c->W == 8 || c->W == 16);
        const bool pow2_w = c->W == 2 || c->W == 4 || c->W == 8 || c->W == 16;
        const uint64_t rec_blocks = (uint64_t)c->lay.n_pieces << kPieceLog;
        // (through the record table the one-kernel step exists for W = 2, 4, 8, 16 only)
        all = (fusion == DASGD_FUSE_ALL || raise) && c->d > 0 && snap &&
              (row_kernels || (pow2_w && rec_blocks <= 0x7fffffffu));
        const int kid = all ? (fold ? DASGD_K_STEP_MEAN_MERGE : DASGD_K_STEP_MEAN)
                      : fold ? (mode == kStoreX ? DASGD_K_STEP_MERGE : DASGD_K_STEP_SNAP_MERGE)
                      : mode == kStoreX ? DASGD_K_LOCAL_STEP
                      : mode == kStoreXS ? DASGD_K_LOCAL_STEP_SNAP : DASGD_K_LOCAL_STEP_TO_SNAP;
        int rec, trial = -1;
        BandTuner *tuned = nullptr;
        rc = prof_open(c, kid, c->main_s, &rec);
        if (rc != DASGD_OK) return rc;
        const unsigned row4 = (unsigned)(c->P / 4);
        if (all && !row_kernels) {
            const Rec *recs = reinterpret_cast<const Rec *>(c->ws + c->lay.recs);
            const float *const *gp = reinterpret_cast<const float *const *>(c->ws + c->lay.gp[g_buf]);
            const dim3 agrid((unsigned)rec_blocks);
            const float inv_w = 1.0f / (float)c->W;
#define DASGD_LAUNCH_RECORDS(WT)                                                                                \
    do {                                                                                                        \
        if (fold) hipLaunchKernelGGL((k_step_all_records<WT, true>), agrid, dim3(kWave * WT), 0, c->main_s, recs, (unsigned)c->lay.n_pieces, \
                                     (unsigned)rec_blocks, gp, c->n_tensors, A, avg_ptr(c, slot), c->lr, c->momentum, c->wd, om, inv_w); \
        else      hipLaunchKernelGGL((k_step_all_records<WT, false>), agrid, dim3(kWave * WT), 0, c->main_s, recs, (unsigned)c->lay.n_pieces, \
                                     (unsigned)rec_blocks, gp, c->n_tensors, A, avg_ptr(c, slot), c->lr, c->momentum, c->wd, om, inv_w); \
    } while (0)
            switch (c->W) {
            case 2:  DASGD_LAUNCH_RECORDS(2);  break;
            case 4:  DASGD_LAUNCH_RECORDS(4);  break;
            case 8:  DASGD_LAUNCH_RECORDS(8);  break;
            default: DASGD_LAUNCH_RECORDS(16); break;
            }
#undef DASGD_LAUNCH_RECORDS
        } else if (all) {
            const dim3 agrid((row4 + kWave - 1) / kWave);
            const v4f *Ao = reinterpret_cast<const v4f *>(A);
            v4f *An = reinterpret_cast<v4f *>(avg_ptr(c, slot));
            const float inv_w = 1.0f / (float)c->W;
#define DASGD_LAUNCH_ROWS(WT)                                                                                   \
    do {                                                                                                        \
        if (fold) hipLaunchKernelGGL((k_step_all_rows<WT, true>), agrid, dim3(kWave * WT), 0, c->main_s, c->xr, c->vr, gr_new, \
                                     Ao, An, row4, c->lr, c->momentum, c->wd, om, inv_w);                       \
        else      hipLaunchKernelGGL((k_step_all_rows<WT, false>), agrid, dim3(kWave * WT), 0, c->main_s, c->xr, c->vr, gr_new, \
                                     Ao, An, row4, c->lr, c->momentum, c->wd, om, inv_w);                       \
    } while (0)
            switch (c->W) {
            case 2:  DASGD_LAUNCH_ROWS(2);  break;
            case 4:  DASGD_LAUNCH_ROWS(4);  break;
            case 8:  DASGD_LAUNCH_ROWS(8);  break;
            case 16: DASGD_LAUNCH_ROWS(16); break;
            default:
                if (fold) hipLaunchKernelGGL((k_step_all_any<true>), agrid, dim3(kWave), 0, c->main_s, c->xr, c->vr, gr_new,
                                             Ao, An, row4, c->W, c->lr, c->momentum, c->wd, om, inv_w);
                else      hipLaunchKernelGGL((k_step_all_any<false>), agrid, dim3(kWave), 0, c->main_s, c->xr, c->vr, gr_new,
                                             Ao, An, row4, c->W, c->lr, c->momentum, c->wd, om, inv_w);
                break;
            }
#undef DASGD_LAUNCH_ROWS
        } else {
            // workgroups per replica, and their order: replica after replica for a plain step (each
            // replica streams linearly); in bands when the average is re-read for every replica
            const uint64_t blocks = row_kernels ? rows_blocks(row4) : ((uint64_t)c->lay.n_pieces << kPieceLog);
            dim3 grid((unsigned)blocks, (unsigned)c->W, 1);
            if (fold) {
                int lb;
                tuned = &c->tuner[kid];
                rc = band_pick(c, *tuned, blocks, &lb, &trial);
                if (rc != DASGD_OK) return rc;
                grid = band_grid(blocks, c->W, lb).grid;
            }
            v4f *S4 = reinterpret_cast<v4f *>(S);
            const v4f *A4 = reinterpret_cast<const v4f *>(A);
            const int64_t ss = c->lay.P_pad;
            if (row_kernels) {
#define DASGD_LAUNCH_STEP(MODE, MERGE)                                                                          \
    hipLaunchKernelGGL((k_step_rows<MODE, MERGE>), grid, dim3(kWave), 0, c->main_s, c->xr, c->vr, gr_new, S4, ss / 4, A4, row4, \
                       c->lr, c->momentum, c->wd, om)
                if (fold && mode == kStoreX)       DASGD_LAUNCH_STEP(kStoreX, true);
                else if (fold)                     DASGD_LAUNCH_STEP(kStoreXS, true);
                else if (mode == kStoreX)          DASGD_LAUNCH_STEP(kStoreX, false);
                else if (mode == kStoreXS)         DASGD_LAUNCH_STEP(kStoreXS, false);
                else                               DASGD_LAUNCH_STEP(kStoreS, false);
#undef DASGD_LAUNCH_STEP
            } else {
                const Rec *recs = reinterpret_cast<const Rec *>(c->ws + c->lay.recs);
                const float *const *gp = reinterpret_cast<const float *const *>(c->ws + c->lay.gp[g_buf]);
#define DASGD_LAUNCH_STEP(MODE, MERGE)                                                                          \
    hipLaunchKernelGGL((k_step_records<MODE, MERGE>), grid, dim3(kWave), 0, c->main_s, recs, (unsigned)c->lay.n_pieces, (unsigned)blocks, \
                       gp, c->n_tensors, S, ss, A, c->lr, c->momentum, c->wd, om)
                if (fold && mode == kStoreX)       DASGD_LAUNCH_STEP(kStoreX, true);
                else if (fold)                     DASGD_LAUNCH_STEP(kStoreXS, true);
                else if (mode == kStoreX)          DASGD_LAUNCH_STEP(kStoreX, false);
                else if (mode == kStoreXS)         DASGD_LAUNCH_STEP(kStoreXS, false);
                else                               DASGD_LAUNCH_STEP(kStoreS, false);
#undef DASGD_LAUNCH_STEP
            }
        }
        HIPCHK(c, hipGetLastError());
        if (g_changed) {                        // launched with the new table: adopt it
            c->g_cached.assign(g, g + rows);
            c->g_cur = g_buf;
            c->g_rows = g_rows_new;
            c->gr = gr_new;
        }
        if (tuned) {
            rc = band_close(c, *tuned, trial);
            if (rc != DASGD_OK) return rc;
        }
        rc = prof_close(c, c->main_s, rec);
        if (rc != DASGD_OK) return rc;
    }
    c->n_done += 1;
    c->begun_for_k = false;
    c->snap_valid = snap_step;
    c->y_in_snap = (mode == kStoreS);
    c->merged_in_step = fold;
    c->zc = zc && !c->dry;
    c->zc_recon = zc && fold;
    c->zc_old_slot = (zc && fold) ? c->pending.front().slot : 0;
    c->zc_xi = c->xi;
    c->mean_in_step = all;
    c->mean_deferred = false;
    c->snap_slot = (int)(c->n_launched % c->slots);
    return DASGD_OK;
}

int dasgd_average_begin(dasgd_ctx *c)
{
    if (!c) return DASGD_EINVAL;
    if (!c->bound || !begin_due(c) || !c->snap_valid) return DASGD_ESTATE;
    if ((int)c->pending.size() >= c->slots) return DASGD_ESTATE;
    const int slot = c->snap_slot;
    bool on_side = false;
    if (!c->dry && c->sched_now != DASGD_SCHED_NO_AVERAGE_TIMING_ONLY && !c->mean_in_step) {
        // The mean has d local steps of slack, the merge of this step has none: when a merge of an
        // OLDER average is still to come in this step, the mean is launched right behind it, so the
        // two bandwidth-bound kernels do not run against each other and the mean overlaps what the
        // caller enqueues next (the forward/backward pass of the following local step).
        if (c->d > 0 && merge_due(c)) {
            c->mean_deferred = true;
        } else {
            int rc = launch_average(c, slot, &on_side);
            if (rc != DASGD_OK) return rc;
        }
    }
    // (an average computed on the main stream has nothing to wait for)
    c->pending.push_back(Pending{c->n_done - 1, slot, on_side, !on_side && !c->mean_deferred});
    c->mean_in_step = false;
    c->n_launched += 1;
    c->begun_for_k = true;
    return DASGD_OK;
}

int dasgd_merge(dasgd_ctx *c)
{
    if (!c) return DASGD_EINVAL;
    if (!c->bound || !merge_due(c)) return DASGD_ESTATE;
    const int slot = c->pending.front().slot;
    if (!c->dry && !c->merged_in_step) {
        Pending &pe = c->pending.front();
        if (pe.on_side && !pe.awaited) {
            HIPCHK(c, hipStreamWaitEvent(c->main_s, c->avg_done[slot], 0));
            pe.awaited = true;
        }
        const float *Y = c->y_in_snap ? snap_ptr(c, c->snap_slot) : nullptr;
        const float om = 1.0f - c->xi;
        int rec, trial = -1, lb;
        int rc = prof_open(c, DASGD_K_MERGE, c->main_s, &rec);
        if (rc != DASGD_OK) return rc;
        const unsigned row4 = (unsigned)(c->P / 4);
        const uint64_t blocks = c->xv_rows ? rows_blocks(row4) : ((uint64_t)c->lay.n_pieces << kPieceLog);
        rc = band_pick(c, c->tuner[DASGD_K_MERGE], blocks, &lb, &trial);
        if (rc != DASGD_OK) return rc;
        const dim3 grid = band_grid(blocks, c->W, lb).grid;
        if (c->xv_rows) {
            const v4f *Y4 = reinterpret_cast<const v4f *>(Y), *A4 = reinterpret_cast<const v4f *>(avg_ptr(c, slot));
            if (Y) hipLaunchKernelGGL((k_merge_rows<true>), grid, dim3(kWave), 0, c->main_s, c->xr, Y4, c->lay.P_pad / 4, A4, row4, om);
            else   hipLaunchKernelGGL((k_merge_rows<false>), grid, dim3(kWave), 0, c->main_s, c->xr, Y4, c->lay.P_pad / 4, A4, row4, om);
        } else {
            const Rec *recs = reinterpret_cast<const Rec *>(c->ws + c->lay.recs);
            if (Y) hipLaunchKernelGGL((k_merge_records<true>), grid, dim3(kWave), 0, c->main_s, recs, (unsigned)c->lay.n_pieces, (unsigned)blocks,
                                      Y, c->lay.P_pad, avg_ptr(c, slot), om);
            else   hipLaunchKernelGGL((k_merge_records<false>), grid, dim3(kWave), 0, c->main_s, recs, (unsigned)c->lay.n_pieces, (unsigned)blocks,
                                      Y, c->lay.P_pad, avg_ptr(c, slot), om);
        }
        HIPCHK(c, hipGetLastError());
        rc = band_close(c, c->tuner[DASGD_K_MERGE], trial);
        if (rc != DASGD_OK) return rc;
        rc = prof_close(c, c->main_s, rec);
        if (rc != DASGD_OK) return rc;
    }
    if (!c->dry && c->mean_deferred) {
        bool on_side = false;
        const int rc2 = launch_average(c, c->snap_slot, &on_side);
        if (rc2 != DASGD_OK) return rc2;
        Pending &mine = c->pending.back();          // registered by dasgd_average_begin of this step
        mine.on_side = on_side;
        mine.awaited = !on_side;
    }
    c->mean_deferred = false;
    c->y_in_snap = false;
    c->merged_in_step = false;
    c->pending.pop_front();
    return DASGD_OK;
}

int dasgd_step(dasgd_ctx *c, const float *const *g, int *began, int *merged)
{
    if (began) *began = 0;
    if (merged) *merged = 0;
    int rc = dasgd_local_step(c, g);
    if (rc != DASGD_OK) return rc;
    if (begin_due(c)) {
        rc = dasgd_average_begin(c);
        if (rc != DASGD_OK) return rc;
        if (began) *began = 1;
    }
    if (merge_due(c)) {
        rc = dasgd_merge(c);
        if (rc != DASGD_OK) return rc;
        if (merged) *merged = 1;
    }
    return DASGD_OK;
}

int dasgd_gradient_average(dasgd_ctx *c, const float *G, float *out)
{
    if (!c || !G || !out) return DASGD_EINVAL;
    if (!c->bound || c->dry) return DASGD_ESTATE;
    if (c->P % 4 != 0 || c->P / 4 > (1ll << 31) - 256) return DASGD_EINVAL;
    if ((reinterpret_cast<uintptr_t>(G) | reinterpret_cast<uintptr_t>(out)) & 15u) return DASGD_EINVAL;
    if (!range_ok(G, sizeof(float) * (size_t)c->W * (size_t)c->P) || !range_ok(out, sizeof(float) * (size_t)c->P)) return DASGD_EINVAL;
    int rec;
    int rc = prof_open(c, DASGD_K_MEAN, c->main_s, &rec);
    if (rc != DASGD_OK) return rc;
    rc = launch_mean(c, c->main_s, nullptr, G, c->P, out, c->P);
    if (rc != DASGD_OK) return rc;
    return prof_close(c, c->main_s, rec);
}

int dasgd_choose_delay(double t_c, double t_p, int *d, int *tau)
{
    if (!(t_c >= 0.0) || !(t_p > 0.0) || !std::isfinite(t_c) || !std::isfinite(t_p)) return DASGD_EINVAL;
    const double r = std::floor(t_c / t_p);
    if (r > 1.0e6) return DASGD_EINVAL;
    const int dd = (int)r + 1;              // smallest integer d with t_c < d * t_p
    if (d) *d = dd;
    if (tau) *tau = dd + 1;
    return DASGD_OK;
}

int dasgd_query(const dasgd_ctx *c, int64_t *step_k, int *n_pending, int *bdue, int *mdue)
{
    if (!c) return DASGD_EINVAL;
    if (step_k) *step_k = c->n_done - 1;
    if (n_pending) *n_pending = (int)c->pending.size();
    if (bdue) *bdue = c->bound && begin_due(c) ? 1 : 0;
    if (mdue) *mdue = c->bound && merge_due(c) ? 1 : 0;
    return DASGD_OK;
}

int dasgd_last_hip_error(const dasgd_ctx *c) { return c ? c->last_hip : g_last_hip; }

int dasgd_average_now_static(int W, int64_t P, float *const *x_rows, float xi, void *stream)
{
    if (P < 1) return DASGD_EINVAL;
    if (P > kStaticScratchFloats) return DASGD_ENOMEM;      // larger replicas: dasgd_average_now with a workspace
    float *A = nullptr;
    const int rc = static_scratch(&A);
    if (rc != DASGD_OK) return rc;
    return average_now(W, P, x_rows, xi, A, static_cast<hipStream_t>(stream));
}

int dasgd_average_now(int W, int64_t P, float *const *x_rows, float xi, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return DASGD_EINVAL;
    if (P < 1 || workspace_bytes / sizeof(float) < (size_t)P) return DASGD_ENOMEM;
    if (!range_ok(workspace, sizeof(float) * (size_t)P)) return DASGD_EINVAL;
    return average_now(W, P, x_rows, xi, static_cast<float *>(workspace), static_cast<hipStream_t>(stream));
}

void dasgd_destroy(dasgd_ctx *c)
{
    if (!c) return;
    if (!c->dry) {
        if (c->bound) {
            (void)hipStreamSynchronize(c->main_s);
            (void)hipStreamSynchronize(c->side_s);
        }
        // a bind that failed half-way leaves some of these set: release whatever exists
        for (hipEvent_t e : c->snap_done) if (e) (void)hipEventDestroy(e);
        for (hipEvent_t e : c->avg_done) if (e) (void)hipEventDestroy(e);
        for (int b = 0; b < kGTables; ++b) if (c->g_ev[b]) (void)hipEventDestroy(c->g_ev[b]);
        for (const ProfRec &r : c->prof_recs) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
        for (const ProfRec &r : c->prof_pool) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
        for (BandTuner &t : c->tuner) {
            for (const BandTuner::Rec &r : t.inflight) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
            for (hipEvent_t e : t.spare) (void)hipEventDestroy(e);
        }
        for (int i = 0; i < c->sched_tuner.n_ev; ++i) if (c->sched_tuner.ev[i]) (void)hipEventDestroy(c->sched_tuner.ev[i]);
        if (c->g_pinned) (void)hipHostFree(c->g_pinned);
    }
    delete c;
}

// ---- include/dasgd_diag.h ------------------------------------------------------------------------

int dasgd_layout(const dasgd_ctx *c, int64_t *flat_offset, int64_t *P_padded, int *addressing)
{
    if (!c) return DASGD_EINVAL;
    if (!c->bound) return DASGD_ESTATE;
    if (flat_offset) std::memcpy(flat_offset, c->lay.foff.data(), sizeof(int64_t) * (size_t)c->n_tensors);
    if (P_padded) *P_padded = c->lay.P_pad;
    if (addressing) *addressing = c->dry ? -1 : !c->xv_rows ? DASGD_ADDR_RECORDS : (c->g_cur >= 0 && !c->g_rows) ? DASGD_ADDR_ROWS_XV : DASGD_ADDR_ROWS;
    return DASGD_OK;
}

int dasgd_pending_average(const dasgd_ctx *c, int which, int64_t *launch_step, size_t *byte_offset)
{
    if (!c) return DASGD_EINVAL;
    if (!c->bound) return DASGD_ESTATE;
    if (which < 0 || which >= (int)c->pending.size()) return DASGD_EINVAL;
    const Pending &p = c->pending[(size_t)which];
    if (launch_step) *launch_step = p.launch_step;
    if (byte_offset) *byte_offset = c->lay.A + sizeof(float) * (size_t)p.slot * (size_t)c->lay.P_pad;
    return DASGD_OK;
}

int dasgd_profile(dasgd_ctx *c, int every_n, int max_records)
{
    if (!c || every_n < 0 || (every_n > 0 && max_records < 1)) return DASGD_EINVAL;
    if (!c->bound || c->dry) return DASGD_ESTATE;
    c->prof_every = every_n;
    c->prof_max = every_n > 0 ? max_records : 0;
    for (int k = 0; k < DASGD_K_COUNT; ++k) c->prof_seen[k] = 0;
    return DASGD_OK;
}

int dasgd_profile_read(dasgd_ctx *c, int kernel, double *total_ms, int64_t *timed, int64_t *launched)
{
    if (!c || kernel < 0 || kernel >= DASGD_K_COUNT) return DASGD_EINVAL;
    if (!c->bound || c->dry) return DASGD_ESTATE;
    HIPCHK(c, hipStreamSynchronize(c->main_s));
    HIPCHK(c, hipStreamSynchronize(c->side_s));
    double sum = 0.0;
    int64_t n = 0;
    std::vector<ProfRec> keep;
    for (const ProfRec &r : c->prof_recs) {
        if (r.kernel != kernel) { keep.push_back(r); continue; }
        float ms = 0.f;
        HIPCHK(c, hipEventElapsedTime(&ms, r.start, r.stop));
        sum += ms;
        n += 1;
        c->prof_pool.push_back(r);
    }
    c->prof_recs.swap(keep);
    if (total_ms) *total_ms = sum;
    if (timed) *timed = n;
    if (launched) *launched = c->prof_seen[kernel];
    c->prof_seen[kernel] = 0;
    return DASGD_OK;
}

int dasgd_set_band(dasgd_ctx *c, int log_band)
{
    if (!c || log_band < -1 || log_band > 11) return DASGD_EINVAL;
    c->band_fixed = log_band;
    return DASGD_OK;
}

int dasgd_band(dasgd_ctx *c, int kernel, int *log_band, int *settled, int *trials)
{
    if (!c || kernel < 0 || kernel >= DASGD_K_COUNT) return DASGD_EINVAL;
    if (!c->bound || c->dry) return DASGD_ESTATE;
    BandTuner &t = c->tuner[kernel];
    if (c->band_fixed < 0 && t.n_cand > 0 && t.chosen < 0) {     // a decision may be due: look, without waiting
        const int rc = band_decide(c, t);
        if (rc != DASGD_OK) return rc;
    }
    if (log_band) *log_band = c->band_fixed >= 0 ? c->band_fixed : t.chosen >= 0 ? t.cand[t.chosen] : -1;
    if (settled) *settled = (c->band_fixed >= 0 || t.chosen >= 0) ? 1 : 0;
    if (trials) {
        *trials = 0;
        for (int i = 0; i < t.n_cand; ++i) *trials += t.issued[i];
    }
    return DASGD_OK;
}

int dasgd_schedule_in_use(const dasgd_ctx *c, int *schedule, int *settled, double *overlap_ms, double *serial_ms)
{
    if (!c) return DASGD_EINVAL;
    const bool is_auto = c->schedule == DASGD_SCHED_AUTO;
    if (schedule) *schedule = is_auto && c->sched_tuner.chosen < 0 ? DASGD_SCHED_AUTO : effective_schedule(c);
    if (settled) *settled = (!is_auto || c->sched_tuner.chosen >= 0) ? 1 : 0;
    if (overlap_ms) *overlap_ms = c->sched_tuner.overlap_ms;
    if (serial_ms) *serial_ms = c->sched_tuner.serial_ms;
    return DASGD_OK;
}

int dasgd_schedule_trial(const dasgd_ctx *c, float *phase_ms)
{
    if (!c || !phase_ms) return DASGD_EINVAL;
    for (int p = 0; p < ScheduleTuner::kPhases - 1; ++p) phase_ms[p] = c->sched_tuner.phase_ms[p];
    return DASGD_OK;
}

int dasgd_device_extent(const void *p, size_t *bytes_to_end)
{
    if (!p || !bytes_to_end) return DASGD_EINVAL;
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    if (hipMemGetAddressRange(&base, &size, const_cast<void *>(p)) != hipSuccess) {
        (void)hipGetLastError();
        return DASGD_EINVAL;
    }
    *bytes_to_end = size - (size_t)(reinterpret_cast<uintptr_t>(p) - reinterpret_cast<uintptr_t>(base));
    return DASGD_OK;
}

int dasgd_check_work_map(int kind, int64_t row4, int head, int log_band)
{
    if (row4 < 1 || row4 > (1ll << 31) - 256) return DASGD_EINVAL;
    const unsigned r4 = (unsigned)row4;
    if (kind == DASGD_MAP_ROWS) {
        // every column of a row whose first element sits `head` 128-bit elements behind a 1 KiB boundary is
        // handled by exactly one (workgroup, lane) of the grid the library would launch, and by none twice
        if (head < 0 || head > 63 || log_band < 0 || log_band > 11) return DASGD_EINVAL;
        if (row4 > (1ll << 27)) return DASGD_EINVAL;            // (host memory of the check itself)
        const BandGrid g = band_grid(rows_blocks(r4), 1, log_band);
        std::vector<unsigned char> seen(r4, 0);
        for (unsigned z = 0; z < g.grid.z; ++z)
            for (unsigned x = 0; x < g.grid.x; ++x) {
                const unsigned q = z * g.grid.x + x;
                for (unsigned lane = 0; lane < 64; ++lane) {
                    const unsigned col = rows_column(q, lane, (unsigned)head);
                    if (col >= r4) continue;
                    if (seen[col]++) return 3;                  // handled twice
                    if (((col + (unsigned)head) & 63u) != lane) return 2;    // not the lane that keeps the kilobyte aligned
                }
            }
        for (unsigned k = 0; k < r4; ++k)
            if (!seen[k]) return 4;                             // never handled
        return DASGD_OK;
    }
    if (kind == DASGD_MAP_MEAN || kind == DASGD_MAP_MEAN_RUNS) {
        // the windows of the mean kernels: a permutation of [0, grid) that covers every window of the row
        const unsigned grid = mean_grid(r4), windows = (r4 + 63u) / 64u;
        std::vector<unsigned char> seen(grid, 0);
        for (unsigned b = 0; b < grid; ++b) {
            const uint64_t w = kind == DASGD_MAP_MEAN_RUNS ? mean_window<true>(b) : mean_window<false>(b);
            if (w >= grid) return 1;                            // a window past the rounded-up grid
            if (seen[w]++) return 3;
        }
        for (unsigned k = 0; k < windows; ++k)
            if (!seen[k]) return 4;
        return DASGD_OK;
    }
    return DASGD_EINVAL;
}

}  // extern "C"
