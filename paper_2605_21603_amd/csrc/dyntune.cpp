// Measured tuning of micro-batch sizes and CU partitions (Section 2.1 names both as the
// knobs a strategy author has to turn; Section 5.3.4 reports the gain of turning one per
// batch at run time).  The candidates and their recording are host logic of the scheduler;
// this file runs them on the device: replay loops on the caller's stream between two events,
// fastest kept.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <vector>

#include "host_error.h"

using dyn::fail;

namespace {

struct EventPair {
    hipEvent_t a = nullptr, b = nullptr;
    ~EventPair() {
        if (a) (void)hipEventDestroy(a);
        if (b) (void)hipEventDestroy(b);
    }
};

// Duration of one forward as a replay loop sees it: three runs of `iters` forwards issued back
// to back between two events (launch latency overlaps the previous forward, as in a serving
// loop), median of the three means; `warmup` untimed forwards first.  Negative if a forward failed.
float time_candidate(dyn_layer *layer, const dyn_batch *batch, const dyn_schedule *sched, hipStream_t stream, EventPair &ev,
                     int warmup, int iters, dyn_status *status) {
    float us[3];
    for (int run = -1; run < 3; ++run) {          // run -1: the warm-up
        const int n = run < 0 ? warmup : iters;
        if (run >= 0 && hipEventRecord(ev.a, stream) != hipSuccess) { *status = DYN_ERR_HIP; return -1.f; }
        for (int i = 0; i < n; ++i) {
            const dyn_status rc = dyn_layer_forward(layer, batch, sched, stream);
            if (rc != DYN_OK) { *status = rc; (void)hipStreamSynchronize(stream); return -1.f; }
        }
        if (run < 0) continue;
        float ms = 0.f;
        if (hipEventRecord(ev.b, stream) != hipSuccess || hipEventSynchronize(ev.b) != hipSuccess ||
            hipEventElapsedTime(&ms, ev.a, ev.b) != hipSuccess) {
            *status = DYN_ERR_HIP;
            return -1.f;
        }
        us[run] = ms * 1e3f / (float)n;
    }
    if (hipStreamSynchronize(stream) != hipSuccess) { *status = DYN_ERR_HIP; return -1.f; }
    std::sort(us, us + 3);
    *status = DYN_OK;
    return us[1];
}

}  // namespace

extern "C" dyn_status dyn_tune(dyn_layer *layer, const dyn_batch *batch, const int32_t *ctx_len_host,
                               const dyn_tune_options *opt_in, void *hip_stream, dyn_scheduler *s, dyn_schedule *out,
                               dyn_tune_result *result, dyn_tune_candidate *table, int capacity) {
    if (!layer || !batch || !opt_in || !s || !out || !result || capacity < 0 || (capacity > 0 && !table))
        return fail(DYN_ERR_INVALID_ARG, "NULL layer, batch, options, scheduler, output or result");
    dyn_tune_options opt = *opt_in;
    // Candidates are timed with eager launches, whatever opt.use_graph says; the flag only marks the
    // schedule that is recorded at the end.  Timing them as graphs meant capturing, replaying and
    // destroying one graph per candidate, dozens per search, in a process that goes on launching
    // graphs - and searches of that kind have ended in a segmentation fault on the host, inside the
    // runtime (in hipGraphLaunch where a stack could be read): with four micro-batches at the 50th
    // graph of a process; with three micro-batches and one graph alive at a time, late in a long
    // process; at last with two micro-batches, late in a long process, after the same run had
    // passed many times.  The library's own bookkeeping of streams, events, graphs and executables
    // replays clean on the CPU under sanitizers against a stand-in runtime that checks every
    // lifetime, so no cause in this library could be shown; what the faults share is a graph
    // destroyed soon after its last replay while others follow, and the search no longer does that.
    // Eager timing carries the host's launch cost, which weighs on the candidates with more streams:
    // the search errs towards the sequential order, never away from it.
    if (opt.max_k < 0 || opt.max_k > 4) return fail(DYN_ERR_INVALID_ARG, "the search covers two to four micro-batches (max_k = %d)", opt.max_k);
    int dev = 0, n_cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return fail(DYN_ERR_HIP, "cannot read the device's CU count");
    opt.n_cus = n_cus;
    if (n_cus % 8) opt.partitions = 0;   // the masks take the same share of each of 8 XCDs
    const int warmup = opt.warmup > 0 ? opt.warmup : 2, iters = opt.iters > 0 ? opt.iters : 7;
    const float min_gain = opt.min_gain < 0.f ? 0.02f : opt.min_gain;

    const int n = dyn_tune_candidates(s, ctx_len_host, &opt, nullptr, 0);
    if (n < 1) return DYN_ERR_INVALID_ARG;
    std::vector<dyn_tune_candidate> cand((size_t)n);
    dyn_tune_candidates(s, ctx_len_host, &opt, cand.data(), n);

    EventPair ev;
    if (hipEventCreate(&ev.a) != hipSuccess || hipEventCreate(&ev.b) != hipSuccess)
        return fail(DYN_ERR_HIP, "cannot create timing events");
    hipStream_t stream = (hipStream_t)hip_stream;
    result->n_tried = result->n_skipped = 0;
    // every side stream of every candidate exists before the first one is timed: creating a
    // CU-masked stream synchronises the device, which must not land inside a timed replay loop
    for (int i = 0; i < n; ++i) {
        dyn_schedule sched;
        if (dyn_tune_record(s, &cand[i], n_cus, 0, &sched) == DYN_OK) (void)dyn_layer_prepare(layer, &sched);
    }
    int best = 0;
    for (int i = 0; i < n; ++i) {
        dyn_schedule sched;
        dyn_status rc = dyn_tune_record(s, &cand[i], n_cus, 0, &sched);
        if (rc == DYN_OK) cand[i].us = time_candidate(layer, batch, &sched, stream, ev, warmup, iters, &rc);
        if (rc != DYN_OK) {
            if (i == 0) return rc;       // the sequential order must run; the error text is the forward's
            cand[i].us = -1.f;
            ++result->n_skipped;
            continue;
        }
        ++result->n_tried;
        if (cand[i].us < cand[best].us) best = i;
    }
    // an overlapped schedule has to earn its place: below min_gain the sequential order stays
    if (best != 0 && cand[best].us > (1.f - min_gain) * cand[0].us) best = 0;
    result->us_sequential = cand[0].us;
    result->best = cand[best];
    if (table) std::copy(cand.begin(), cand.begin() + std::min(n, capacity), table);
    return dyn_tune_record(s, &cand[best], n_cus, opt.use_graph, out);
}
