// What the library measures for itself while it runs, without ever making the host wait: per-kernel timing
// brackets (dasgd_profile), the band length of the kernels that re-read the average for every replica, and the
// choice between the overlap and the serial schedule (DASGD_SCHED_AUTO; paper, Section 3.4 Eq. 3 and Fig. 4:
// whether the averaging disappears behind the local computation).  Included by dasgd.hip only.
#pragma once
#include "context.hpp"

namespace {

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

// Grid (gx, W, gz) that covers `blocks` workgroups per replica in bands of 2^log_band blocks per L2
// partition.  The band is lengthened until gz fits the 16-bit limit of a grid's z dimension and
// shortened to what the row needs.
struct BandGrid { dim3 grid; int log_band; };
BandGrid band_grid(uint64_t blocks, int W, int log_band)
{
    if (blocks < 1) blocks = 1;
    int lb = log_band < 0 ? 0 : log_band;
    while (lb > 0 && (8ull << (lb - 1)) >= blocks) --lb;               // one band already holds the row
    while ((blocks + (8ull << lb) - 1) / (8ull << lb) > 65535ull) ++lb;
    const uint64_t gx = 8ull << lb, gz = (blocks + gx - 1) / gx;
    BandGrid g;
    g.grid = dim3((unsigned)gx, (unsigned)W, (unsigned)gz);
    g.log_band = lb;
    return g;
}

// Choice for the next launch of the kernel that tuner t serves, over `blocks` workgroups per replica:
// the log2 of a band length.  *trial >= 0: the launch is a timed trial, band_close must follow it.
int band_pick(dasgd_ctx *c, BandTuner &t, uint64_t blocks, int *log_band, int *trial)
{
    *trial = -1;
    if (c->band_fixed >= 0) {
        *log_band = band_grid(blocks, 1, c->band_fixed).log_band;
        return DASGD_OK;
    }
    if (t.n_cand == 0) {                        // fit the candidates to the row length, drop duplicates
        int n = 0;
        for (int i = 0; i < BandTuner::kMaxCand; ++i) {
            const int lb = band_grid(blocks, 1, t.cand[i]).log_band;
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
        *log_band = t.cand[t.n_cand / 2];
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

// DASGD_SCHED_AUTO: one call per local step.  Advances the phases, decides once the marks have completed, and
// returns in *mark the event (or null) that this step must record on the main stream -- AFTER it has made the
// main stream wait for the means still running on the side stream, so that a mean is charged to the phase
// that launched it and not to the next one.
int schedule_tick(dasgd_ctx *c, hipEvent_t *mark)
{
    *mark = nullptr;
    ScheduleTuner &t = c->sched_tuner;
    if (c->schedule != DASGD_SCHED_AUTO || t.chosen >= 0) return DASGD_OK;
    if (t.phase < ScheduleTuner::kPhases) {
        if (t.steps_in_phase == 0 && t.phase >= 1) {            // boundary: start of a measured phase
            const int i = t.phase - 1;
            if (!t.ev[i]) { HIPCHK(c, hipEventCreate(&t.ev[i])); t.n_ev = i + 1; }
            *mark = t.ev[i];
        }
        ++t.steps_in_phase;
        bool over = t.steps_in_phase >= t.phase_len;
        if (t.phase == 0) {
            // the warm-up lasts two phases and as long as band lengths are still being tried (their timing
            // events and slower candidates would fall into some phases and not others), within reason
            bool bands_busy = false;
            for (const BandTuner &b : c->tuner) bands_busy = bands_busy || (b.n_cand > 0 && b.chosen < 0);
            over = t.steps_in_phase >= 2 * t.phase_len && t.steps_in_phase % t.phase_len == 0 &&
                   (!bands_busy || t.steps_in_phase >= 32 * t.phase_len);
        }
        if (over) {
            t.steps_in_phase = 0;
            t.phase += 1;
        }
        return DASGD_OK;
    }
    const int last = ScheduleTuner::kPhases - 1;                // the mark that ends the last measured phase
    if (!t.ev[last]) {
        HIPCHK(c, hipEventCreate(&t.ev[last]));
        t.n_ev = last + 1;
        *mark = t.ev[last];
        return DASGD_OK;
    }
    const hipError_t q = hipEventQuery(t.ev[last]);
    if (q == hipErrorNotReady) {
        (void)hipGetLastError();
        return DASGD_OK;
    }
    HIPCHK(c, q);
    t.overlap_ms = t.serial_ms = 0;
    for (int p = 1; p < ScheduleTuner::kPhases; ++p) {          // phase p lies between marks p-1 and p
        float ms = 0.f;
        HIPCHK(c, hipEventElapsedTime(&ms, t.ev[p - 1], t.ev[p]));
        ((p & 1) ? t.overlap_ms : t.serial_ms) += ms;
        t.phase_ms[p - 1] = ms;
    }
    t.chosen = t.overlap_ms < t.serial_ms ? DASGD_SCHED_OVERLAP : DASGD_SCHED_SERIAL;
    for (int i = 0; i < t.n_ev; ++i) { (void)hipEventDestroy(t.ev[i]); t.ev[i] = nullptr; }
    t.n_ev = 0;
    return DASGD_OK;
}

}  // namespace
