// Host side of the DaSGD parameter pipeline: the C ABI declared in include/dasgd.h, the
// pending-average ring, and the stream/event schedule that lets the W-way mean run behind the
// following local steps (paper, Section 3 and Fig. 2: a worker hands its weights to the averaging
// and immediately continues; the result is applied d local steps later).
#include "../../include/dasgd.h"
#include "kernels.hpp"

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <algorithm>
#include <deque>
#include <utility>
#include <new>
#include <vector>

using namespace dasgd;

namespace {

constexpr int kGTables = 4;         // device copies of the gradient pointer table, used in rotation
constexpr size_t kAlign = 256;

inline size_t align_up(size_t n) { return (n + kAlign - 1) / kAlign * kAlign; }

struct Pending {
    int64_t launch_step;
    int slot;
    bool awaited;       // the main stream already waits for this average's mean kernel
};

struct ProfRec {
    int kernel;
    hipEvent_t start, stop;
};

// Which band length (see decode_block) is fastest depends on the row length and on what runs around
// the kernel, so it is measured where it matters: in the caller's own steps.  The first launches of
// a kernel kind rotate through the candidates, a few of them bracketed by timing events; finished
// events are collected with non-blocking queries at later launches (the host never waits), and once
// every candidate has its samples the fastest is kept.  The band length only permutes which
// workgroup handles which block: results are bit-identical for every choice.
struct BandTuner {
    static constexpr int kMaxCand = 5, kSamples = 3;
    int cand[kMaxCand] = {0, 8, 9, 10, 11};     // log2 of the band length
    int n_cand = 0;                             // 0: candidates not yet fitted to the row length
    double sum_ms[kMaxCand] = {};
    int done[kMaxCand] = {}, issued[kMaxCand] = {};
    int64_t launches = 0;
    int chosen = -1;                            // index into cand once decided
    struct Rec { int cand; hipEvent_t start, stop; };
    std::deque<Rec> inflight;
    std::vector<hipEvent_t> spare;
};

struct Layout {                     // byte offsets into the workspace
    size_t chunks, xp, vp, gp[kGTables], S, A, total;
    int64_t P_pad, n_chunks;        // P_pad: elements per snapshot row / average
    std::vector<int64_t> foff;      // start of each tensor inside such a row
    bool flat = false;              // rows mirror the caller's matrix (foff = plain prefix sums, P_pad = row stride)
};

}  // namespace

struct dasgd_ctx {
    // problem
    int W = 0, d = 0, tau = 1;
    int64_t P = 0;
    float lr = 0, momentum = 0, wd = 0, xi = 0.25f;
    int schedule = DASGD_SCHED_OVERLAP;
    int fusion = DASGD_FUSE_STEP_MERGE;
    int snapshot = DASGD_SNAPSHOT_ZERO_COPY;
    int slots = 1;
    size_t side_min_bytes = (size_t)64 << 20;   // means that move less than this run on the main stream
    // binding
    bool bound = false, dry = false;
    int n_tensors = 0;
    std::vector<int64_t> numel;
    Layout lay;
    char *ws = nullptr;
    hipStream_t main_s = nullptr, side_s = nullptr;
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
    bool snap_valid = false;        // the latest local step stored a snapshot
    bool y_in_snap = false;         // ... and ONLY the snapshot: x is stale until this step's merge
    bool mean_deferred = false;     // the mean of snap_slot is launched right after this step's merge
    bool merged_in_step = false;    // the latest local step already applied this step's merge
    bool mean_in_step = false;      // ... and already computed the average that average_begin will register
    bool zc = false;                // the latest local step stored no snapshot: the mean reads x itself
    bool zc_recon = false;          // ... and x already holds the merged weights: undo the merge on the mean
    int zc_old_slot = 0;            // ... with the average in this slot
    float zc_xi = 0.25f;            // ... and this xi
    int snap_slot = 0;
    // matrix layout: x, v (and g) are W x P row-major matrices with one row stride, 16-byte aligned
    bool xv_matrix = false, g_matrix = false;
    int64_t ld = 0;                 // row stride of that matrix in elements (P <= ld < P + 256)
    float *x0 = nullptr, *v0 = nullptr;
    const float *g0 = nullptr;
    int band_fixed = -1;            // >= 0: log2 of the band length set by the caller; -1: measured (BandTuner)
    BandTuner tuner[DASGD_K_COUNT];
    BandTuner table_tuner[2];       // chunk-table local step with a folded merge (0: no snapshot store, 1: with):
                                    // candidates -1 (replica-major grid) and 0 (replicas of a chunk on one XCD)
    bool idx32 = false;             // 64 <= P/4 and W*P/4 + 64 < 2^31: the column-aware flat kernels apply
                                    // (32-bit indices; a 64-element block spans at most two rows)
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
        if (numel[t] < 1) return false;
        sum += numel[t];
    }
    return sum == c->P;
}

// Rows of the library-owned buffers either pad every tensor to a 256-byte boundary (so the table
// kernels can always use 128-bit accesses on them) or, when the caller's x and v are W x P matrices,
// mirror that layout, row stride included (so one flat index addresses x, v, g and the snapshot
// alike).  The byte offsets of the padded layout are used in both cases: the workspace size must not
// depend on pointers that dasgd_workspace_bytes never sees.
constexpr int64_t kMaxRowPad = 256;  // a matrix row may be followed by fewer than this many padding floats

Layout make_layout(const dasgd_ctx *c, int n_tensors, const int64_t *numel, bool flat = false, int64_t ld = 0)
{
    Layout L;
    L.foff.resize(n_tensors);
    int64_t f = 0, fp = 0, nch = 0;
    for (int t = 0; t < n_tensors; ++t) {
        L.foff[t] = flat ? fp : f;
        fp += numel[t];
        f += (numel[t] + kPad - 1) / kPad * kPad;
        nch += (numel[t] + kChunk - 1) / kChunk;
    }
    L.flat = flat;
    f += kMaxRowPad;                // room for the row padding of the matrix layout
    L.P_pad = f;                    // sizes below always use the padded row length
    L.n_chunks = nch;
    const size_t tbl = sizeof(void *) * (size_t)c->W * (size_t)n_tensors;
    size_t o = 0;
    L.chunks = o; o += align_up(sizeof(Chunk) * (size_t)nch);
    L.xp = o;     o += align_up(tbl);
    L.vp = o;     o += align_up(tbl);
    for (int b = 0; b < kGTables; ++b) { L.gp[b] = o; o += align_up(tbl); }
    L.S = o;      o += align_up(sizeof(float) * (size_t)c->slots * (size_t)c->W * (size_t)L.P_pad);
    L.A = o;      o += align_up(sizeof(float) * (size_t)c->slots * (size_t)L.P_pad);
    L.total = o;
    if (flat) L.P_pad = ld;
    return L;
}

// True when ptr[j*n + t] == ptr[0] + j*ld + (unpadded offset of t) for all j, t with one row stride ld,
// P <= ld < P + kMaxRowPad, ld a multiple of 4, base 16-byte aligned: a W x P row-major matrix whose
// rows are back to back or separated by a little alignment padding (which then belongs to the matrix).
template <typename T>
bool is_matrix(const dasgd_ctx *c, int n_tensors, const int64_t *numel, T *const *ptr, int64_t *ld_out)
{
    if (reinterpret_cast<uintptr_t>(ptr[0]) & 15u) return false;
    int64_t ld = c->P;
    if (c->W > 1) {
        const uintptr_t a = reinterpret_cast<uintptr_t>(ptr[0]), b = reinterpret_cast<uintptr_t>(ptr[n_tensors]);
        if (b <= a || (b - a) % sizeof(float)) return false;
        ld = (int64_t)((b - a) / sizeof(float));
    }                               // (one row: nothing tells a stride, so ld = P)
    if (ld < c->P || ld - c->P >= kMaxRowPad || ld % 4 != 0) return false;
    for (int j = 0; j < c->W; ++j) {
        int64_t off = 0;
        for (int t = 0; t < n_tensors; ++t) {
            if (ptr[(size_t)j * n_tensors + t] != ptr[0] + (int64_t)j * ld + off) return false;
            off += numel[t];
        }
    }
    *ld_out = ld;
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

// The mean goes to the side stream in the overlap schedules -- unless it is so small that the two
// cross-stream hand-overs (main -> side before it, side -> main after it; 6-10 us each on MI355X)
// cost more than running it in line could ever lose.
inline bool side_stream_mean(const dasgd_ctx *c)
{
    if (c->schedule != DASGD_SCHED_OVERLAP && c->schedule != DASGD_SCHED_OVERLAP_FREE) return false;
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

// Timing brackets for one launch (no-ops unless profiling).
int prof_open(dasgd_ctx *c, int kernel, hipStream_t s, int *rec_index)
{
    *rec_index = -1;
    if (c->prof_every <= 0) return DASGD_OK;
    if ((c->prof_seen[kernel]++ % c->prof_every) != 0 || (int)c->prof_recs.size() >= c->prof_max) return DASGD_OK;
    ProfRec r;
    if (!c->prof_pool.empty()) {
        r = c->prof_pool.back();
        c->prof_pool.pop_back();
    } else {
        HIPCHK(c, hipEventCreate(&r.start));
        HIPCHK(c, hipEventCreate(&r.stop));
    }
    r.kernel = kernel;
    HIPCHK(c, hipEventRecord(r.start, s));
    c->prof_recs.push_back(r);
    *rec_index = (int)c->prof_recs.size() - 1;
    return DASGD_OK;
}
int prof_close(dasgd_ctx *c, hipStream_t s, int rec_index)
{
    if (rec_index < 0) return DASGD_OK;
    HIPCHK(c, hipEventRecord(c->prof_recs[rec_index].stop, s));
    return DASGD_OK;
}

// Collect the trials that have finished (never waits).
int band_poll(dasgd_ctx *c, BandTuner &t)
{
    while (!t.inflight.empty()) {
        BandTuner::Rec &r = t.inflight.front();
        const hipError_t q = hipEventQuery(r.stop);
        if (q == hipErrorNotReady) {
            (void)hipGetLastError();            // "not ready" is an answer, not a failure: do not leave it behind
            break;
        }
        HIPCHK(c, q);
        float ms = 0.f;
        HIPCHK(c, hipEventElapsedTime(&ms, r.start, r.stop));
        t.sum_ms[r.cand] += ms;
        t.done[r.cand] += 1;
        t.spare.push_back(r.start);
        t.spare.push_back(r.stop);
        t.inflight.pop_front();
    }
    return DASGD_OK;
}

// Collect, and keep the fastest candidate once every one has its samples.
int band_decide(dasgd_ctx *c, BandTuner &t)
{
    const int rc = band_poll(c, t);
    if (rc != DASGD_OK) return rc;
    for (int i = 0; i < t.n_cand; ++i)
        if (t.done[i] < BandTuner::kSamples) return DASGD_OK;
    int best = 0;
    for (int i = 1; i < t.n_cand; ++i)
        if (t.sum_ms[i] / t.done[i] < t.sum_ms[best] / t.done[best]) best = i;
    t.chosen = best;
    for (hipEvent_t e : t.spare) (void)hipEventDestroy(e);
    t.spare.clear();
    return DASGD_OK;
}

// Choice for the next launch of the kernel that tuner t serves, over rows of row4 128-bit columns: the
// log2 of a band length, or a negative candidate (the caller's other work order).  *trial >= 0: the
// launch is a timed trial, band_close must follow it.
int band_pick(dasgd_ctx *c, BandTuner &t, unsigned row4, int *log_band, int *trial)
{
    *trial = -1;
    if (c->band_fixed >= 0) {
        *log_band = (int)decode_clamp_log_band(row4, (unsigned)c->band_fixed);
        return DASGD_OK;
    }
    if (t.n_cand == 0) {                        // fit the candidates to the row length, drop duplicates
        int n = 0;
        for (int i = 0; i < BandTuner::kMaxCand; ++i) {
            const int lb = t.cand[i] < 0 ? t.cand[i] : (int)decode_clamp_log_band(row4, (unsigned)t.cand[i]);
            bool dup = false;
            for (int k = 0; k < n; ++k) dup = dup || t.cand[k] == lb;
            if (!dup) t.cand[n++] = lb;
        }
        t.n_cand = n;
        if (n == 1) t.chosen = 0;
    }
    if (t.chosen < 0) {
        const int rc = band_decide(c, t);
        if (rc != DASGD_OK) return rc;
    }
    if (t.chosen >= 0) {
        *log_band = t.cand[t.chosen];
        return DASGD_OK;
    }
    const int64_t n = t.launches++;
    int pick = -1;
    if (n > 0)                                  // (the first launch of a kind runs cold: not timed)
        for (int i = 0; i < t.n_cand; ++i)
            if (t.issued[i] < BandTuner::kSamples && (pick < 0 || t.issued[i] < t.issued[pick])) pick = i;
    if (pick < 0) {                             // cold launch, or all trials issued and results still to come
        *log_band = t.cand[0];
        return DASGD_OK;
    }
    BandTuner::Rec r;
    r.cand = pick;
    for (hipEvent_t *e : {&r.start, &r.stop}) {
        if (!t.spare.empty()) { *e = t.spare.back(); t.spare.pop_back(); }
        else HIPCHK(c, hipEventCreate(e));
    }
    HIPCHK(c, hipEventRecord(r.start, c->main_s));
    t.inflight.push_back(r);
    t.issued[pick] += 1;
    *log_band = t.cand[pick];
    *trial = pick;
    return DASGD_OK;
}
int band_close(dasgd_ctx *c, BandTuner &t, int trial)
{
    if (trial < 0) return DASGD_OK;
    HIPCHK(c, hipEventRecord(t.inflight.back().stop, c->main_s));
    return DASGD_OK;
}

int launch_mean(dasgd_ctx *c, hipStream_t s, const float *S, float *A, int64_t row_elems)
{
    const int64_t n4 = row_elems / 4;
    const v4f *S4 = reinterpret_cast<const v4f *>(S);
    v4f *A4 = reinterpret_cast<v4f *>(A);
    const float inv_w = 1.0f / (float)c->W;
    auto grid = [&](int U) { return dim3((unsigned)(((n4 + (int64_t)kWave * U - 1) / ((int64_t)kWave * U) + 63) / 64 * 64)); };
    const bool runs = (row_elems % 32) != 0;         // rows not 128-byte aligned to each other
#define DASGD_LAUNCH_MEAN(WT)                                                                                   \
    do {                                                                                                        \
        if (runs) hipLaunchKernelGGL((k_mean<WT, 1, true, true>), grid(1), dim3(kWave), 0, s, S4, A4, n4, n4, c->W, inv_w); \
        else      hipLaunchKernelGGL((k_mean<WT, 1, true, false>), grid(1), dim3(kWave), 0, s, S4, A4, n4, n4, c->W, inv_w); \
    } while (0)
#define DASGD_LAUNCH_MEAN_LDS(WT, NW)                                                                           \
    do {                                                                                                        \
        if (runs) hipLaunchKernelGGL((k_mean_lds<WT, NW, true>), grid(1), dim3(kWave * NW), 0, s, S4, A4, n4, n4, inv_w); \
        else      hipLaunchKernelGGL((k_mean_lds<WT, NW, false>), grid(1), dim3(kWave * NW), 0, s, S4, A4, n4, n4, inv_w); \
    } while (0)
    switch (c->W) {             // rows split over wavefronts + LDS where that measured faster
    case 1:  DASGD_LAUNCH_MEAN(1);  break;
    case 2:  DASGD_LAUNCH_MEAN(2);  break;
    case 4:  DASGD_LAUNCH_MEAN_LDS(4, 4);  break;
    case 8:  DASGD_LAUNCH_MEAN_LDS(8, 4);  break;
    case 16: DASGD_LAUNCH_MEAN_LDS(16, 8); break;
    default: DASGD_LAUNCH_MEAN(0);  break;
    }
#undef DASGD_LAUNCH_MEAN_LDS
#undef DASGD_LAUNCH_MEAN
    HIPCHK(c, hipGetLastError());
    return DASGD_OK;
}

}  // namespace

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
    for (BandTuner &t : c->table_tuner) {
        const int orders[BandTuner::kMaxCand] = {-1, 0, 0, 0, 0};          // duplicates are dropped when the tuner starts
        for (int i = 0; i < BandTuner::kMaxCand; ++i) t.cand[i] = orders[i];
    }
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
    if (!c || schedule < DASGD_SCHED_OVERLAP || schedule > DASGD_SCHED_OVERLAP_FREE) return DASGD_EINVAL;
    if (!c->pending.empty() || begin_due(c)) return DASGD_ESTATE;
    c->schedule = schedule;
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
    if (!c || fusion < DASGD_FUSE_NONE || fusion > DASGD_FUSE_ALL) return DASGD_EINVAL;
    if (!c->pending.empty() || begin_due(c)) return DASGD_ESTATE;
    c->fusion = fusion;
    return DASGD_OK;
}

int dasgd_set_snapshot(dasgd_ctx *c, int mode)
{
    if (!c || (mode != DASGD_SNAPSHOT_COPY && mode != DASGD_SNAPSHOT_ZERO_COPY)) return DASGD_EINVAL;
    if (!c->pending.empty() || begin_due(c)) return DASGD_ESTATE;
    c->snapshot = mode;
    return DASGD_OK;
}

size_t dasgd_workspace_bytes(const dasgd_ctx *c, int n_tensors, const int64_t *numel)
{
    if (!shapes_ok(c, n_tensors, numel)) return 0;
    return make_layout(c, n_tensors, numel).total;
}

static int bind_common(dasgd_ctx *c, int n_tensors, const int64_t *numel)
{
    if (!shapes_ok(c, n_tensors, numel)) return DASGD_EINVAL;
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
    {   // x, v and the workspace are all written: none of them may share a byte with another
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
    int64_t ldx = 0, ldv = 0;
    bool matrix = is_matrix(c, n_tensors, numel, x, &ldx) && is_matrix(c, n_tensors, numel, v, &ldv) && ldx == ldv;
    // the matrix kernels also touch the padding behind the LAST row: it must exist
    if (matrix) {
        const size_t extent = sizeof(float) * (size_t)c->W * (size_t)ldx;
        matrix = range_ok(x[0], extent) && range_ok(v[0], extent);
    }
    Layout L = make_layout(c, n_tensors, numel, matrix, ldx);
    if (workspace_bytes < L.total) return DASGD_ENOMEM;
    if (!range_ok(workspace, L.total)) return DASGD_EINVAL;

    // chunk table
    std::vector<Chunk> chunks;
    chunks.reserve((size_t)L.n_chunks);
    for (int t = 0; t < n_tensors; ++t)
        for (int64_t off = 0; off < numel[t]; off += kChunk) {
            Chunk ch;
            ch.off = off;
            ch.foff = L.foff[t] + off;
            ch.tensor = t;
            ch.len = (int32_t)((numel[t] - off) < kChunk ? (numel[t] - off) : kChunk);
            chunks.push_back(ch);
        }

    c->n_tensors = n_tensors;
    c->numel.assign(numel, numel + n_tensors);
    c->lay = L;
    c->xv_matrix = matrix;
    c->ld = matrix ? ldx : 0;
    c->x0 = x[0];
    c->v0 = v[0];
    c->idx32 = matrix && c->ld / 4 >= 64 && (int64_t)c->W * c->ld / 4 + 64 < (1ll << 31) && decode_grid((unsigned)c->W, (unsigned)(c->ld / 4), 11) < (1ull << 31);
    c->ws = static_cast<char *>(workspace);
    c->main_s = static_cast<hipStream_t>(main_stream);
    c->side_s = static_cast<hipStream_t>(side_stream);

    HIPCHK(c, hipMemcpyAsync(c->ws + L.chunks, chunks.data(), sizeof(Chunk) * chunks.size(), hipMemcpyHostToDevice, c->main_s));
    HIPCHK(c, hipMemcpyAsync(c->ws + L.xp, x, sizeof(void *) * rows, hipMemcpyHostToDevice, c->main_s));
    HIPCHK(c, hipMemcpyAsync(c->ws + L.vp, v, sizeof(void *) * rows, hipMemcpyHostToDevice, c->main_s));
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

// Launch the W-way mean of snapshot slot `slot`.  In the overlap schedule it goes to the side
// stream, ordered after everything enqueued on the main stream so far.
static int launch_average(dasgd_ctx *c, int slot)
{
    hipStream_t s = c->main_s;
    if (side_stream_mean(c)) {
        HIPCHK(c, hipEventRecord(c->snap_done[slot], c->main_s));
        HIPCHK(c, hipStreamWaitEvent(c->side_s, c->snap_done[slot], 0));
        s = c->side_s;
    }
    int rec;
    int rc = prof_open(c, c->zc && c->zc_recon ? DASGD_K_MEAN_RECONSTRUCT : DASGD_K_MEAN, s, &rec);
    if (rc != DASGD_OK) return rc;
    if (c->zc && c->zc_recon) {
        const int64_t n4 = c->ld / 4;
        const unsigned grid = (unsigned)(((n4 + kWave - 1) / kWave + 63) / 64 * 64);
        const v4f *X4 = reinterpret_cast<const v4f *>(c->x0), *Ao = reinterpret_cast<const v4f *>(avg_ptr(c, c->zc_old_slot));
        v4f *An = reinterpret_cast<v4f *>(avg_ptr(c, slot));
        const double om = (double)(1.0f - c->zc_xi), inv_xi = 1.0 / (double)c->zc_xi, inv_w = 1.0 / (double)c->W;
        if (c->ld % 32)
            hipLaunchKernelGGL((k_mean_reconstruct<4, true>), dim3(grid), dim3(kWave * 4), 0, s, X4, Ao, An, n4, n4, c->W, inv_w, om, inv_xi);
        else
            hipLaunchKernelGGL((k_mean_reconstruct<4, false>), dim3(grid), dim3(kWave * 4), 0, s, X4, Ao, An, n4, n4, c->W, inv_w, om, inv_xi);
        HIPCHK(c, hipGetLastError());
    } else {
        rc = launch_mean(c, s, c->zc ? c->x0 : snap_ptr(c, slot), avg_ptr(c, slot), c->lay.P_pad);
        if (rc != DASGD_OK) return rc;
    }
    rc = prof_close(c, s, rec);
    if (rc != DASGD_OK) return rc;
    if (side_stream_mean(c)) HIPCHK(c, hipEventRecord(c->avg_done[slot], c->side_s));
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
    const bool snap = snap_step && c->schedule != DASGD_SCHED_NO_AVERAGE_TIMING_ONLY;
    // fold the merge into this kernel?  (not for d == 0: that merge needs the mean of this step's own output)
    const bool fold = merge_follows && c->d > 0 && c->fusion >= DASGD_FUSE_STEP_MERGE;
    int mode = kStoreX;
    if (snap) mode = (merge_follows && !fold && c->fusion >= DASGD_FUSE_SNAPSHOT) ? kStoreS : kStoreXS;
    // zero-copy snapshot: store none, let the mean read x (see DASGD_SNAPSHOT_ZERO_COPY)
    const bool zc = snap && c->snapshot == DASGD_SNAPSHOT_ZERO_COPY && c->xv_matrix && c->fusion == DASGD_FUSE_STEP_MERGE &&
                    (c->schedule == DASGD_SCHED_OVERLAP || c->schedule == DASGD_SCHED_SERIAL) &&
                    (fold ? c->xi >= 0.125f : !merge_follows);
    if (zc) mode = kStoreX;
    // everything in one kernel?  (decided below once the gradient layout is known)
    bool all = false;
    const size_t rows = (size_t)c->W * (size_t)c->n_tensors;

    if (!c->dry) {
        if (!g && c->g_cur < 0) return DASGD_EINVAL;
        if (g) {
            for (size_t r = 0; r < rows; ++r)
                if (!g[r] || (reinterpret_cast<uintptr_t>(g[r]) & 3u)) return DASGD_EINVAL;
            const bool changed = c->g_cur < 0 || std::memcmp(g, c->g_cached.data(), sizeof(void *) * rows) != 0;
            if (changed) {
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
                // retire the table in use (all kernels reading it are already enqueued), take the next
                if (c->g_cur >= 0) {
                    HIPCHK(c, hipEventRecord(c->g_ev[c->g_cur], c->main_s));
                    c->g_ev_live[c->g_cur] = true;
                }
                const int b = (c->g_cur + 1) % kGTables;
                if (c->g_ev_live[b]) {
                    HIPCHK(c, hipEventSynchronize(c->g_ev[b]));      // its last reader ran kGTables-1 changes ago
                    c->g_ev_live[b] = false;
                }
                void *stage = static_cast<char *>(c->g_pinned) + sizeof(void *) * rows * (size_t)b;
                std::memcpy(stage, g, sizeof(void *) * rows);
                HIPCHK(c, hipMemcpyAsync(c->ws + c->lay.gp[b], stage, sizeof(void *) * rows, hipMemcpyHostToDevice, c->main_s));
                c->g_cached.assign(g, g + rows);
                c->g_cur = b;
                int64_t ldg = 0;
                c->g_matrix = is_matrix(c, c->n_tensors, c->numel.data(), g, &ldg) && ldg == c->ld &&
                              range_ok(g[0], sizeof(float) * (size_t)c->W * (size_t)ldg);
                c->g0 = g[0];
            }
        }
        const int slot = (int)(c->n_launched % c->slots);
        float *S = mode == kStoreX ? nullptr : snap_ptr(c, slot);
        const float *A = nullptr;
        const float om = 1.0f - c->xi;
        // Default overlap schedule: every kernel of this library saturates HBM, so letting a mean run
        // beside one only makes both slower; the local step therefore waits for the means in flight,
        // which leaves them whatever the caller put on the main stream since the last merge (the
        // forward/backward pass) to hide behind.  The free variant waits only for the average it reads.
        if (side_stream_mean(c)) {
            for (size_t p = 0; p < c->pending.size(); ++p) {
                Pending &pe = c->pending[p];
                const bool needed = fold && p == 0;
                if (pe.awaited || !(needed || c->schedule == DASGD_SCHED_OVERLAP)) continue;
                HIPCHK(c, hipStreamWaitEvent(c->main_s, c->avg_done[pe.slot], 0));
                pe.awaited = true;
            }
        }
        if (fold) A = avg_ptr(c, c->pending.front().slot);
        all = c->fusion == DASGD_FUSE_ALL && c->d > 0 && c->xv_matrix && c->g_matrix &&
              c->schedule != DASGD_SCHED_NO_AVERAGE_TIMING_ONLY && snap;
        const int kid = all ? (fold ? DASGD_K_STEP_MEAN_MERGE : DASGD_K_STEP_MEAN)
                      : fold ? (mode == kStoreX ? DASGD_K_STEP_MERGE : DASGD_K_STEP_SNAP_MERGE)
                      : mode == kStoreX ? DASGD_K_LOCAL_STEP
                      : mode == kStoreXS ? DASGD_K_LOCAL_STEP_SNAP : DASGD_K_LOCAL_STEP_TO_SNAP;
        int rec, trial = -1;
        BandTuner *tuned = nullptr;
        int rc = prof_open(c, kid, c->main_s, &rec);
        if (rc != DASGD_OK) return rc;
        const bool flat = c->xv_matrix && c->g_matrix && (!fold || c->idx32);
        if (all) {
            const int64_t row4 = c->ld / 4;
            const dim3 agrid((unsigned)((row4 + kWave - 1) / kWave));
            v4f *x4 = reinterpret_cast<v4f *>(c->x0), *v4 = reinterpret_cast<v4f *>(c->v0);
            const v4f *g4 = reinterpret_cast<const v4f *>(c->g0);
            const v4f *Ao = reinterpret_cast<const v4f *>(A);
            v4f *An = snap ? reinterpret_cast<v4f *>(avg_ptr(c, slot)) : nullptr;
            const float inv_w = 1.0f / (float)c->W;
#define DASGD_LAUNCH_ALL(WT, MEAN, MERGE)                                                                       \
    hipLaunchKernelGGL((k_step_all_flat<WT, MEAN, MERGE>), agrid, dim3(kWave), 0, c->main_s, x4, v4, g4, Ao, An, \
                       row4, c->W, c->lr, c->momentum, c->wd, om, inv_w)
#define DASGD_LAUNCH_ROWS(WT, MERGE)                                                                            \
    hipLaunchKernelGGL((k_step_all_rows<WT, MERGE>), agrid, dim3(kWave * WT), 0, c->main_s, x4, v4, g4, Ao, An,  \
                       row4, c->lr, c->momentum, c->wd, om, inv_w)
#define DASGD_LAUNCH_ALL_W(MEAN, MERGE)                                                                         \
    switch (c->W) {                                                                                             \
    case 1:  DASGD_LAUNCH_ALL(1, MEAN, MERGE);  break;                                                          \
    case 2:  DASGD_LAUNCH_ROWS(2, MERGE);  break;                                                               \
    case 4:  DASGD_LAUNCH_ROWS(4, MERGE);  break;                                                               \
    case 8:  DASGD_LAUNCH_ROWS(8, MERGE);  break;                                                               \
    case 16: DASGD_LAUNCH_ROWS(16, MERGE); break;                                                               \
    default: DASGD_LAUNCH_ALL(0, MEAN, MERGE);  break;                                                          \
    }
            if (fold) { DASGD_LAUNCH_ALL_W(true, true) } else { DASGD_LAUNCH_ALL_W(true, false) }
#undef DASGD_LAUNCH_ROWS
#undef DASGD_LAUNCH_ALL_W
#undef DASGD_LAUNCH_ALL
        } else if (flat) {
            const int64_t n4 = (int64_t)c->W * c->ld / 4;
            const dim3 grid((unsigned)((n4 + kWave - 1) / kWave));
            v4f *x4 = reinterpret_cast<v4f *>(c->x0), *v4 = reinterpret_cast<v4f *>(c->v0), *s4 = reinterpret_cast<v4f *>(S);
            const v4f *g4 = reinterpret_cast<const v4f *>(c->g0);
            if (fold) {
                const v4f *A4 = reinterpret_cast<const v4f *>(A);
                const unsigned row4 = (unsigned)(c->ld / 4);
                int lbi;
                tuned = &c->tuner[kid];
                rc = band_pick(c, *tuned, row4, &lbi, &trial);
                if (rc != DASGD_OK) return rc;
                const unsigned lb = (unsigned)lbi;
                const dim3 fgrid((unsigned)decode_grid((unsigned)c->W, row4, lb));
#define DASGD_LAUNCH_FOLD(SNAP, WT)                                                                             \
    hipLaunchKernelGGL((k_step_merge_flat<SNAP, WT>), fgrid, dim3(kWave), 0, c->main_s, x4, v4, g4, s4, A4,     \
                       (unsigned)n4, row4, c->W, lb, c->lr, c->momentum, c->wd, om)
#define DASGD_LAUNCH_FOLD_W(SNAP)                                                                               \
    switch (c->W) {                                                                                             \
    case 1:  DASGD_LAUNCH_FOLD(SNAP, 1);  break;                                                                \
    case 2:  DASGD_LAUNCH_FOLD(SNAP, 2);  break;                                                                \
    case 4:  DASGD_LAUNCH_FOLD(SNAP, 4);  break;                                                                \
    case 8:  DASGD_LAUNCH_FOLD(SNAP, 8);  break;                                                                \
    case 16: DASGD_LAUNCH_FOLD(SNAP, 16); break;                                                                \
    default: DASGD_LAUNCH_FOLD(SNAP, 0);  break;                                                                \
    }
                if (mode == kStoreX) { DASGD_LAUNCH_FOLD_W(false) } else { DASGD_LAUNCH_FOLD_W(true) }
#undef DASGD_LAUNCH_FOLD_W
#undef DASGD_LAUNCH_FOLD
            } else if (mode == kStoreX)
                hipLaunchKernelGGL((k_local_step_flat<kStoreX>), grid, dim3(kWave), 0, c->main_s, x4, v4, g4, s4, n4, c->lr, c->momentum, c->wd);
            else if (mode == kStoreXS)
                hipLaunchKernelGGL((k_local_step_flat<kStoreXS>), grid, dim3(kWave), 0, c->main_s, x4, v4, g4, s4, n4, c->lr, c->momentum, c->wd);
            else
                hipLaunchKernelGGL((k_local_step_flat<kStoreS>), grid, dim3(kWave), 0, c->main_s, x4, v4, g4, s4, n4, c->lr, c->momentum, c->wd);
        } else {
            const Chunk *chunks = reinterpret_cast<const Chunk *>(c->ws + c->lay.chunks);
            float *const *xp = reinterpret_cast<float *const *>(c->ws + c->lay.xp);
            float *const *vp = reinterpret_cast<float *const *>(c->ws + c->lay.vp);
            const float *const *gp = reinterpret_cast<const float *const *>(c->ws + c->lay.gp[c->g_cur]);
            // Folded merge: either replica-major (all chunks of replica 0, then of replica 1, ...: each
            // replica streams linearly and A is re-read W times, which is cheap while A fits the Infinity
            // Cache), or the W replicas of a chunk back to back on one XCD (A from HBM once).  Which is
            // faster depends on the size of A and on how the allocations lie in memory: measured in place.
            int xcd_order = 0;
            if (fold) {
                tuned = &c->table_tuner[mode == kStoreX ? 0 : 1];
                int pick;
                rc = band_pick(c, *tuned, 1u << 20, &pick, &trial);
                if (rc != DASGD_OK) return rc;
                xcd_order = pick >= 0 ? 1 : 0;
            }
            const dim3 grid = xcd_order ? dim3((unsigned)((c->lay.n_chunks + 7) / 8 * 8 * c->W))
                                        : dim3((unsigned)c->lay.n_chunks, (unsigned)c->W);
#define DASGD_LAUNCH_TABLE(MODE, MERGE)                                                                         \
    hipLaunchKernelGGL((k_local_step<MODE, MERGE>), grid, dim3(kThreads), 0, c->main_s, chunks, xp, vp, gp, S, \
                       c->lay.P_pad, c->n_tensors, c->lr, c->momentum, c->wd, A, om, c->W, (int)c->lay.n_chunks, xcd_order)
            if (fold && mode == kStoreX)       DASGD_LAUNCH_TABLE(kStoreX, true);
            else if (fold)                     DASGD_LAUNCH_TABLE(kStoreXS, true);
            else if (mode == kStoreX)          DASGD_LAUNCH_TABLE(kStoreX, false);
            else if (mode == kStoreXS)         DASGD_LAUNCH_TABLE(kStoreXS, false);
            else                               DASGD_LAUNCH_TABLE(kStoreS, false);
#undef DASGD_LAUNCH_TABLE
        }
        HIPCHK(c, hipGetLastError());
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
    if (!c->dry && c->schedule != DASGD_SCHED_NO_AVERAGE_TIMING_ONLY && !c->mean_in_step) {
        // The mean has d local steps of slack, the merge of this step has none: when a merge of an
        // OLDER average is still to come in this step, the mean is launched right behind it, so the
        // two bandwidth-bound kernels do not run against each other and the mean overlaps what the
        // caller enqueues next (the forward/backward pass of the following local step).
        if (c->d > 0 && merge_due(c)) {
            c->mean_deferred = true;
        } else {
            int rc = launch_average(c, slot);
            if (rc != DASGD_OK) return rc;
        }
    }
    c->pending.push_back(Pending{c->n_done - 1, slot, c->mean_in_step});   // computed on the main stream: nothing to wait for
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
        if (side_stream_mean(c) && !c->pending.front().awaited) HIPCHK(c, hipStreamWaitEvent(c->main_s, c->avg_done[slot], 0));
        const float *Y = c->y_in_snap ? snap_ptr(c, c->snap_slot) : nullptr;
        const float om = 1.0f - c->xi;
        int rec, trial = -1;
        int rc = prof_open(c, DASGD_K_MERGE, c->main_s, &rec);
        if (rc != DASGD_OK) return rc;
        if (c->xv_matrix && c->idx32) {
            const int64_t row4 = c->ld / 4;
            v4f *X4 = reinterpret_cast<v4f *>(c->x0);
            const v4f *Y4 = Y ? reinterpret_cast<const v4f *>(Y) : X4;
            const v4f *A4 = reinterpret_cast<const v4f *>(avg_ptr(c, slot));
            const unsigned n4 = (unsigned)(row4 * c->W);
            int lbi;
            rc = band_pick(c, c->tuner[DASGD_K_MERGE], (unsigned)row4, &lbi, &trial);
            if (rc != DASGD_OK) return rc;
            const unsigned lb = (unsigned)lbi;
            const dim3 grid((unsigned)decode_grid((unsigned)c->W, (unsigned)row4, lb));
            switch (c->W) {
            case 1:  hipLaunchKernelGGL((k_merge_flat<1>),  grid, dim3(kWave), 0, c->main_s, X4, Y4, A4, n4, (unsigned)row4, c->W, lb, om); break;
            case 2:  hipLaunchKernelGGL((k_merge_flat<2>),  grid, dim3(kWave), 0, c->main_s, X4, Y4, A4, n4, (unsigned)row4, c->W, lb, om); break;
            case 4:  hipLaunchKernelGGL((k_merge_flat<4>),  grid, dim3(kWave), 0, c->main_s, X4, Y4, A4, n4, (unsigned)row4, c->W, lb, om); break;
            case 8:  hipLaunchKernelGGL((k_merge_flat<8>),  grid, dim3(kWave), 0, c->main_s, X4, Y4, A4, n4, (unsigned)row4, c->W, lb, om); break;
            case 16: hipLaunchKernelGGL((k_merge_flat<16>), grid, dim3(kWave), 0, c->main_s, X4, Y4, A4, n4, (unsigned)row4, c->W, lb, om); break;
            default: hipLaunchKernelGGL((k_merge_flat<0>),  grid, dim3(kWave), 0, c->main_s, X4, Y4, A4, n4, (unsigned)row4, c->W, lb, om); break;
            }
        } else {
            const Chunk *chunks = reinterpret_cast<const Chunk *>(c->ws + c->lay.chunks);
            float *const *xp = reinterpret_cast<float *const *>(c->ws + c->lay.xp);
            const dim3 grid((unsigned)c->lay.n_chunks);
            if (Y)
                hipLaunchKernelGGL((k_merge<true>), grid, dim3(kThreads), 0, c->main_s, chunks, xp, avg_ptr(c, slot), Y, c->lay.P_pad, c->n_tensors, c->W, om);
            else
                hipLaunchKernelGGL((k_merge<false>), grid, dim3(kThreads), 0, c->main_s, chunks, xp, avg_ptr(c, slot), Y, c->lay.P_pad, c->n_tensors, c->W, om);
        }
        HIPCHK(c, hipGetLastError());
        rc = band_close(c, c->tuner[DASGD_K_MERGE], trial);
        if (rc != DASGD_OK) return rc;
        rc = prof_close(c, c->main_s, rec);
        if (rc != DASGD_OK) return rc;
    }
    if (!c->dry) {
        if (c->mean_deferred) {
            const int rc2 = launch_average(c, c->snap_slot);
            if (rc2 != DASGD_OK) return rc2;
        }
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
    if (c->P % 4 != 0) return DASGD_EINVAL;
    if ((reinterpret_cast<uintptr_t>(G) | reinterpret_cast<uintptr_t>(out)) & 15u) return DASGD_EINVAL;
    if (!range_ok(G, sizeof(float) * (size_t)c->W * (size_t)c->P) || !range_ok(out, sizeof(float) * (size_t)c->P)) return DASGD_EINVAL;
    int rec;
    int rc = prof_open(c, DASGD_K_MEAN, c->main_s, &rec);
    if (rc != DASGD_OK) return rc;
    rc = launch_mean(c, c->main_s, G, out, c->P);
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

int dasgd_layout(const dasgd_ctx *c, int64_t *flat_offset, int64_t *P_padded)
{
    if (!c) return DASGD_EINVAL;
    if (!c->bound) return DASGD_ESTATE;
    if (flat_offset) std::memcpy(flat_offset, c->lay.foff.data(), sizeof(int64_t) * (size_t)c->n_tensors);
    if (P_padded) *P_padded = c->lay.P_pad;
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

int dasgd_check_block_map(int W, int64_t row4, int log_band)
{
    if (W < 1 || W > 65535 || row4 < 64 || log_band < 0 || log_band > 11) return DASGD_EINVAL;
    if ((int64_t)W * row4 + 64 >= (1ll << 31)) return DASGD_EINVAL;
    const unsigned w = (unsigned)W, r4 = (unsigned)row4, n4 = w * r4;
    const unsigned lb = decode_clamp_log_band(r4, (unsigned)log_band);
    const uint64_t grid = decode_grid(w, r4, lb);
    if (grid >= (1ull << 31)) return DASGD_EINVAL;
    const unsigned n_blocks = (n4 + 63u) / 64u;
    std::vector<unsigned char> seen(n_blocks, 0);
    for (uint64_t b = 0; b < grid; ++b) {
        unsigned blk, lo, hi;
        if (!decode_owner((unsigned)b, w, r4, lb, blk, lo, hi)) continue;
        if (blk >= n_blocks) return 1;                                  // a workgroup would start past the end
        if (lo / r4 != (unsigned)(((uint64_t)blk * 64u) / r4)) return 2;   // owned by a row that does not hold its first element
        if (seen[blk]++) return 3;                                      // handled twice
    }
    for (unsigned k = 0; k < n_blocks; ++k)
        if (!seen[k]) return 4;                                         // never handled
    return DASGD_OK;
}

int dasgd_last_hip_error(const dasgd_ctx *c) { return c ? c->last_hip : 0; }

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
        for (BandTuner *ts : {c->tuner, c->table_tuner})
            for (int i = 0; i < (ts == c->tuner ? (int)DASGD_K_COUNT : 2); ++i) {
                BandTuner &t = ts[i];
                for (const BandTuner::Rec &r : t.inflight) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
                for (hipEvent_t e : t.spare) (void)hipEventDestroy(e);
            }
        if (c->g_pinned) (void)hipHostFree(c->g_pinned);
    }
    delete c;
}

}  // extern "C"
