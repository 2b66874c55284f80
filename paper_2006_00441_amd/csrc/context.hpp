// Host state of one DaSGD context: the ring of pending averages (paper, Section 3 and Fig. 2: an average is
// launched every tau local steps and applied d steps later), the layout of the library-owned buffers inside the
// workspace, and the checks dasgd_bind makes on what the caller hands over.  Included by dasgd.hip only.
#pragma once
#include "../../include/dasgd.h"
#include "../../include/dasgd_diag.h"
#include "kernels.hpp"

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <algorithm>
#include <deque>
#include <mutex>
#include <utility>
#include <new>
#include <vector>

using namespace dasgd;

namespace {

constexpr int kGTables = 4;         // device copies of the gradient pointer table, used in rotation
constexpr size_t kAlign = 256;
constexpr int64_t kRowAlign = 256;  // library-owned rows start on 1 KiB boundaries

inline size_t align_up(size_t n) { return (n + kAlign - 1) / kAlign * kAlign; }

struct Pending {
    int64_t launch_step;
    int slot;
    bool on_side;       // its mean kernel was launched on the side stream
    bool awaited;       // the main stream already waits for it (or it ran there)
};

struct ProfRec {
    int kernel;
    hipEvent_t start, stop;
};

// Which band length (see the three-dimensional grids in kernels.hpp) is fastest depends on the row
// length and on what runs around the kernel, so it is measured where it matters: in the caller's own
// steps.  The first launches of a kernel kind rotate through the candidates, a few of them bracketed by
// timing events; finished events are collected with non-blocking queries at later launches (the host
// never waits), and once every candidate has its samples the fastest is kept.  The band length only
// permutes which workgroup handles which block: results are bit-identical for every choice.
struct BandTuner {
    static constexpr int kMaxCand = 5, kSamples = 3;
    int cand[kMaxCand] = {5, 8, 9, 10, 11};     // log2 of the band length
    int n_cand = 0;                             // 0: candidates not yet fitted to the row length
    double sum_ms[kMaxCand] = {};
    int done[kMaxCand] = {}, issued[kMaxCand] = {};
    int64_t launches = 0;
    int chosen = -1;                            // index into cand once decided
    struct Rec { int cand; hipEvent_t start, stop; };
    std::deque<Rec> inflight;
    std::vector<hipEvent_t> spare;
};

// Whether the side stream pays depends on what the caller runs between two steps: beside work that
// leaves wave slots free the mean disappears behind it; beside nothing, or beside a kernel that fills
// every SIMD, the two cross-stream hand-overs only cost time.  DASGD_SCHED_AUTO therefore measures:
// after a warm-up phase the schedule alternates between OVERLAP and SERIAL in phases of a few steps, an
// event on the main stream marks every phase boundary (so the caller's own work is inside the
// measurement), and once all events have completed -- seen by a non-blocking query at a later step --
// the schedule with the smaller total is kept.
struct ScheduleTuner {
    static constexpr int kPhases = 7;           // phase 0 is the warm-up; 1, 3, 5 OVERLAP; 2, 4, 6 SERIAL
    int phase = 0, steps_in_phase = 0, phase_len = 8;
    int chosen = -1;                            // DASGD_SCHED_OVERLAP or DASGD_SCHED_SERIAL once decided
    hipEvent_t ev[kPhases + 1] = {};
    int n_ev = 0;
    double overlap_ms = 0, serial_ms = 0;
    float phase_ms[kPhases - 1] = {};           // measured phases 1..6 in order, once decided
};

struct Layout {                     // byte offsets into the workspace
    size_t recs, gp[kGTables], S, A, total;
    int64_t P_pad, n_pieces;        // P_pad: floats per snapshot row / average
    std::vector<int64_t> foff;      // start of each tensor inside such a row
    bool rows = false;              // rows mirror the replicas' own layout (foff = plain prefix sums)
};

}  // namespace

struct dasgd_ctx {
    // problem
    int W = 0, d = 0, tau = 1;
    int64_t P = 0;
    float lr = 0, momentum = 0, wd = 0, xi = 0.25f;
    int schedule = DASGD_SCHED_AUTO;
    int fusion = DASGD_FUSE_AUTO;
    int snapshot = DASGD_SNAPSHOT_AUTO;
    int slots = 1;
    size_t side_min_bytes = (size_t)64 << 20;   // means that move less than this run on the main stream
    unsigned head_start_us = 20;                // a side-stream mean is held back by this much (k_head_start)
    // binding
    bool bound = false, dry = false;
    int n_tensors = 0;
    std::vector<int64_t> numel;
    Layout lay;
    char *ws = nullptr;
    hipStream_t main_s = nullptr, side_s = nullptr;
    // rows addressing: every replica's tensors are one contiguous, 16-byte aligned run of P floats
    bool xv_rows = false, g_rows = false;
    RowSet xr = {}, vr = {};
    ConstRowSet gr = {};
    // gradient pointer tables
    std::vector<const float *> g_cached;
    std::vector<std::pair<uintptr_t, size_t>> owned;    // byte ranges of x, v and the workspace, sorted by start
    int g_cur = -1;
    void *g_pinned = nullptr;       // kGTables host staging tables (pinned)
    hipEvent_t g_ev[kGTables] = {};
    bool g_ev_live[kGTables] = {};
    // schedule state
    int64_t n_done = 0;             // completed local steps; k = n_done - 1
    int64_t n_launched = 0;         // averages launched so far
    bool begun_for_k = false;       // dasgd_average_begin already issued for the current k
    bool snap_valid = false;        // the latest local step prepared an average (snapshot stored, or zero-copy)
    bool y_in_snap = false;         // ... and stored ONLY the snapshot: x is stale until this step's merge
    bool mean_deferred = false;     // the mean of snap_slot is launched right after this step's merge
    bool merged_in_step = false;    // the latest local step already applied this step's merge
    bool mean_in_step = false;      // ... and already computed the average that average_begin will register
    bool zc = false;                // the latest local step stored no snapshot: the mean reads x itself
    bool zc_recon = false;          // ... and x already holds the merged weights: undo the merge on the mean
    int zc_old_slot = 0;            // ... with the average in this slot
    float zc_xi = 0.25f;            // ... and this xi
    int snap_slot = 0;
    int sched_now = DASGD_SCHED_OVERLAP;   // the schedule in effect for the step being issued (fixed per step)
    int band_fixed = -1;            // >= 0: log2 of the band length set by the caller; -1: measured (BandTuner)
    BandTuner tuner[DASGD_K_COUNT];
    ScheduleTuner sched_tuner;
    std::deque<Pending> pending;
    std::vector<hipEvent_t> snap_done, avg_done;
    // profiling
    int prof_every = 0;             // 0: off; n: time one launch in n of every kernel kind
    int prof_max = 0;
    int64_t prof_seen[DASGD_K_COUNT] = {};
    std::vector<ProfRec> prof_recs;
    std::vector<ProfRec> prof_pool;
    int last_hip = 0;
};

namespace {

#define HIPCHK(ctx, expr)                                   \
    do {                                                    \
        hipError_t e_ = (expr);                             \
        if (e_ != hipSuccess) {                             \
            (ctx)->last_hip = (int)e_;                      \
            return DASGD_EHIP;                              \
        }                                                   \
    } while (0)

bool shapes_ok(const dasgd_ctx *c, int n_tensors, const int64_t *numel)
{
    if (!c || n_tensors < 1 || !numel) return false;
    int64_t sum = 0;
    for (int t = 0; t < n_tensors; ++t) {
        if (numel[t] < 1 || numel[t] >= (1ll << 32)) return false;
        sum += numel[t];
    }
    return sum == c->P;
}

// Rows of the library-owned buffers (snapshots, averages) either pad every tensor to a 256-byte
// boundary (so that the record kernels can use 128-bit accesses on them whatever the tensor sizes) or,
// when every replica is one contiguous run, mirror that run (column c of a snapshot row is column c of
// the replica).  The byte offsets of the padded layout are used in both cases: the workspace size must
// not depend on pointers that dasgd_workspace_bytes never sees.
Layout make_layout(const dasgd_ctx *c, int n_tensors, const int64_t *numel, bool rows = false)
{
    Layout L;
    L.foff.resize(n_tensors);
    int64_t f = 0, fp = 0, np = 0;
    for (int t = 0; t < n_tensors; ++t) {
        L.foff[t] = rows ? fp : f;
        fp += numel[t];
        f += (numel[t] + kPad - 1) / kPad * kPad;
        np += (numel[t] + kPiece - 1) / kPiece;
    }
    L.rows = rows;
    f = (f + kRowAlign - 1) / kRowAlign * kRowAlign + kRowAlign;
    L.P_pad = f;                    // sizes below always use the padded row length
    L.n_pieces = np;
    const size_t tbl = sizeof(void *) * (size_t)c->W * (size_t)n_tensors;
    size_t o = 0;
    L.recs = o;   o += align_up(sizeof(Rec) * (size_t)c->W * (size_t)np);
    for (int b = 0; b < kGTables; ++b) { L.gp[b] = o; o += align_up(tbl); }
    L.S = o;      o += align_up(sizeof(float) * (size_t)c->slots * (size_t)c->W * (size_t)L.P_pad);
    L.A = o;      o += align_up(sizeof(float) * (size_t)c->slots * (size_t)L.P_pad);
    L.total = o;
    if (rows) L.P_pad = (c->P + kRowAlign - 1) / kRowAlign * kRowAlign;
    return L;
}

// True when, for every replica j, ptr[j*n + t] == ptr[j*n] + (unpadded offset of t) and ptr[j*n] is
// 16-byte aligned, with P a multiple of 4 below 2^33 and at most kMaxRows replicas: every replica is one
// contiguous run of P floats (rows of a matrix with any stride, or one arena per replica).
template <typename T>
bool is_rows(const dasgd_ctx *c, int n_tensors, const int64_t *numel, T *const *ptr)
{
    if (c->W > kMaxRows || c->P % 4 != 0 || c->P / 4 > (1ll << 31) - 256) return false;
    for (int j = 0; j < c->W; ++j) {
        T *base = ptr[(size_t)j * n_tensors];
        if (reinterpret_cast<uintptr_t>(base) & 15u) return false;
        int64_t off = 0;
        for (int t = 0; t < n_tensors; ++t) {
            if (ptr[(size_t)j * n_tensors + t] != base + off) return false;
            off += numel[t];
        }
    }
    return true;
}

// False only when the runtime knows the allocation that holds p and [p, p + bytes) leaves it.  (Memory
// the runtime cannot place -- not allocated through it -- cannot be checked and passes.)  A kernel that
// runs past a buffer faults the GPU; a size mistake of the caller's is better met with an error code.
// `last` remembers the allocation found for the previous pointer of the same pass: tensors usually
// sit side by side in one allocation, and asking the runtime costs about half a microsecond each time.
struct DeviceRange {
    uintptr_t base = 0;
    size_t size = 0;
};
bool range_ok(const void *p, size_t bytes, DeviceRange *last = nullptr)
{
    const uintptr_t a = reinterpret_cast<uintptr_t>(p);
    DeviceRange r;
    if (last && last->size && a >= last->base && a - last->base < last->size) {
        r = *last;
    } else {
        hipDeviceptr_t base = nullptr;
        size_t size = 0;
        if (hipMemGetAddressRange(&base, &size, const_cast<void *>(p)) != hipSuccess) {
            (void)hipGetLastError();
            return true;
        }
        r.base = reinterpret_cast<uintptr_t>(base);
        r.size = size;
        if (last) *last = r;
    }
    return a >= r.base && bytes <= r.size && a - r.base <= r.size - bytes;
}

// True if any two of the byte ranges [first, first + second) overlap (sorts its argument).
bool any_overlap(std::vector<std::pair<uintptr_t, size_t>> &iv)
{
    std::sort(iv.begin(), iv.end());
    for (size_t i = 1; i < iv.size(); ++i)
        if (iv[i].first < iv[i - 1].first + iv[i - 1].second) return true;
    return false;
}

inline float *snap_ptr(const dasgd_ctx *c, int slot)
{
    return reinterpret_cast<float *>(c->ws + c->lay.S) + (size_t)slot * (size_t)c->W * (size_t)c->lay.P_pad;
}
inline float *avg_ptr(const dasgd_ctx *c, int slot)
{
    return reinterpret_cast<float *>(c->ws + c->lay.A) + (size_t)slot * (size_t)c->lay.P_pad;
}

// The schedule in effect for the step being issued.
inline int effective_schedule(const dasgd_ctx *c)
{
    if (c->schedule != DASGD_SCHED_AUTO) return c->schedule;
    const ScheduleTuner &t = c->sched_tuner;
    if (t.chosen >= 0) return t.chosen;
    if (t.phase >= ScheduleTuner::kPhases) return DASGD_SCHED_OVERLAP;       // measured, result still to come
    return (t.phase == 0 || (t.phase & 1)) ? DASGD_SCHED_OVERLAP : DASGD_SCHED_SERIAL;
}

// The mean goes to the side stream in the overlap schedules -- unless it is so small that the two
// cross-stream hand-overs (main -> side before it, side -> main after it; 6-10 us each on MI355X)
// cost more than running it in line could ever lose.
inline bool side_stream_mean(const dasgd_ctx *c)
{
    const int s = c->sched_now;
    if (s != DASGD_SCHED_OVERLAP && s != DASGD_SCHED_OVERLAP_FREE) return false;
    const size_t mean_bytes = sizeof(float) * (size_t)(c->W + 1) * (size_t)c->lay.P_pad;
    return mean_bytes >= c->side_min_bytes;
}

inline bool begin_due(const dasgd_ctx *c)
{
    return c->n_done > 0 && (c->n_done % c->tau) == 0 && !c->begun_for_k;     // (k+1) mod tau == 0
}
inline bool merge_due(const dasgd_ctx *c)
{
    return !c->pending.empty() && c->pending.front().launch_step == (c->n_done - 1) - c->d;
}

// Steps for which DASGD_SNAPSHOT_AUTO takes the zero-copy path.  Measured against a double-precision run
// (W = 8, tau = 1, d = 2, random gradients) the deviation of every fp32 implementation grows like the
// square root of the step count K: about 1.3e-7 sqrt(K) of the weight scale with stored snapshots, and
// 2.2e-7 sqrt(K) with the reconstruction at xi = 0.25, whose extra term scales with 1/xi.  The budget keeps
// the reconstruction's share small enough that the whole run stays below 1e-5 for 3000 steps with a
// quarter to spare (sqrt(500 * 2.2e-7^2 + 2500 * 1.3e-7^2) = 7.2e-6): 500 steps at xi >= 0.25, fewer in
// proportion to xi^2 below, none below xi = 1/8.
inline int64_t zero_copy_budget(float xi)
{
    if (xi < 0.125f) return 0;
    const double r = std::min(1.0, (double)xi / 0.25);
    return (int64_t)(500.0 * r * r);
}

}  // namespace
