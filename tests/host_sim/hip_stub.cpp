// A host-only stand-in for the HIP runtime calls libdynlayer makes, so that the library's whole
// host side (schedule expansion, stream / event choreography, graph capture, cache, eviction,
// retirement, the tuner's loops, every launcher's grid arithmetic) can run on a CPU under
// AddressSanitizer and UndefinedBehaviorSanitizer.  TEST INFRASTRUCTURE: nothing here computes
// anything; a kernel launch is a counted node.
//
// Streams, events, graphs and executables are host objects that are never freed, only marked
// destroyed, so that any later use is seen.  The model of the device is the most adversarial
// one the API allows: nothing that was submitted completes until the host waits for it
// (hipStreamSynchronize, hipEventSynchronize, hipDeviceSynchronize).  Every rule below that the
// library breaks is a "violation": it is printed, counted, and the call returns an error.
//
//   * use of a destroyed or unknown stream / event / graph / executable; destroying one twice
//   * hipStreamWaitEvent on an event that was never recorded
//   * a wait, from any stream, on an event whose last record belongs to a capture that has ended
//   * a capturing stream waiting on an event recorded outside its capture, or inside another
//   * hipStreamEndCapture with work on a joined stream that the origin stream does not depend on
//   * hipEventQuery / hipEventSynchronize / hipEventElapsedTime on an event recorded in a capture
//   * hipGraphExecDestroy while a launch of that executable has not completed
//   * hipGraphLaunch into a capturing stream; begin / end capture on the wrong stream
//   * hipStreamSynchronize / hipDeviceSynchronize / stream creation with a CU mask while a capture is open
//     on the calling thread's stream, and CU-masked stream creation while submitted work is pending
//   * a kernel launch with an empty or oversized grid / block or more dynamic LDS than a CU has
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <set>
#include <string>
#include <vector>

#include "hip_stub.h"

namespace {

struct Graph;

struct Dep { struct Stream *stream; uint64_t pos; };

struct Stream {
    int id;
    bool destroyed = false, masked = false;
    Graph *capture = nullptr;             // the capture this stream currently belongs to
    std::vector<int> frontier;            // capture: nodes the stream's next node depends on
    bool launched_in_capture = false;
    uint64_t submitted = 0, completed = 0;   // eager timeline: operations issued / known complete
    std::vector<std::pair<uint64_t, Dep>> waits;   // operation index -> what it waits for
};

struct Event {
    int id;
    bool destroyed = false, recorded = false;
    Graph *capture = nullptr;             // last record was inside this capture
    std::vector<int> nodes;
    Stream *stream = nullptr;             // last record was eager: on this stream, after `pos` operations
    uint64_t pos = 0;
    uint64_t launches_at_record = 0;      // for the fake clock
};

struct Node { std::vector<int> deps; int stream_id; };

struct Graph {
    int id;
    bool destroyed = false, ended = false;
    Stream *origin = nullptr;
    std::vector<Stream *> joined;
    std::vector<Node> nodes;
    int side_branches = 0;
};

struct Exec {
    int id;
    bool destroyed = false;
    Graph *graph;
    int n_nodes, side_branches;
    std::vector<Dep> launches;            // (stream, operation index) of every launch
};

// the registries are never destroyed (not even at exit), so their objects stay reachable for the leak checker
std::set<Stream *> &g_streams = *new std::set<Stream *>();
std::set<Event *> &g_events = *new std::set<Event *>();
std::set<Graph *> &g_graphs = *new std::set<Graph *>();
std::set<Exec *> &g_execs = *new std::set<Exec *>();
Stream g_null_stream{0};
int g_next_id = 1;
hipstub_stats g_stats{};
std::vector<std::string> g_violations;
hipError_t g_last_error = hipSuccess;
uint64_t g_launch_clock = 0;

struct CallConfig { dim3 grid, block; size_t shmem; hipStream_t stream; };
std::vector<CallConfig> g_call_stack;

hipError_t violation(hipError_t err, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    fprintf(stderr, "hip_stub VIOLATION: %s\n", buf);
    g_violations.push_back(buf);
    ++g_stats.violations;
    g_last_error = err;
    return err;
}

Stream *as_stream(hipStream_t s, const char *who, bool *ok) {
    *ok = true;
    if (!s) return &g_null_stream;
    Stream *p = reinterpret_cast<Stream *>(s);
    if (!g_streams.count(p)) { violation(hipErrorInvalidHandle, "%s: unknown stream %p", who, (void *)s); *ok = false; return nullptr; }
    if (p->destroyed) { violation(hipErrorInvalidHandle, "%s: stream %d was destroyed", who, p->id); *ok = false; return nullptr; }
    return p;
}

Event *as_event(hipEvent_t e, const char *who) {
    Event *p = reinterpret_cast<Event *>(e);
    if (!e || !g_events.count(p)) { violation(hipErrorInvalidHandle, "%s: unknown event %p", who, (void *)e); return nullptr; }
    if (p->destroyed) { violation(hipErrorInvalidHandle, "%s: event %d was destroyed", who, p->id); return nullptr; }
    return p;
}

void complete(Stream *s, uint64_t upto) {
    if (upto <= s->completed) return;
    const uint64_t from = s->completed;
    s->completed = upto;
    for (auto &w : s->waits)
        if (w.first > from && w.first <= upto) complete(w.second.stream, w.second.pos);
}

bool any_pending() {
    if (g_null_stream.completed < g_null_stream.submitted) return true;
    for (Stream *s : g_streams)
        if (!s->destroyed && s->completed < s->submitted) return true;
    return false;
}

void submit_eager(Stream *s) { ++s->submitted; }

void add_capture_node(Stream *s) {
    Graph *g = s->capture;
    g->nodes.push_back(Node{s->frontier, s->id});
    s->frontier.assign(1, (int)g->nodes.size() - 1);
    s->launched_in_capture = true;
}

bool reaches(const Graph *g, const std::vector<int> &from, int target) {
    std::vector<char> seen(g->nodes.size(), 0);
    std::vector<int> stack(from);
    while (!stack.empty()) {
        const int n = stack.back();
        stack.pop_back();
        if (n == target) return true;
        if (seen[n]) continue;
        seen[n] = 1;
        for (int d : g->nodes[n].deps) stack.push_back(d);
    }
    return false;
}

void count_live() {
    int execs = 0, branches = 0;
    for (Exec *e : g_execs)
        if (!e->destroyed) { ++execs; branches += e->side_branches; }
    g_stats.max_live_execs = std::max(g_stats.max_live_execs, execs);
    g_stats.max_live_side_branches = std::max(g_stats.max_live_side_branches, branches);
}

}  // namespace

extern "C" {

const hipstub_stats *hipstub_get_stats(void) {
    g_stats.live_streams = g_stats.live_events = g_stats.live_graphs = g_stats.live_execs = 0;
    for (Stream *s : g_streams) g_stats.live_streams += !s->destroyed;
    for (Event *e : g_events) g_stats.live_events += !e->destroyed;
    for (Graph *g : g_graphs) g_stats.live_graphs += !g->destroyed;
    for (Exec *e : g_execs) g_stats.live_execs += !e->destroyed;
    return &g_stats;
}

const char *hipstub_violation(int i) { return i >= 0 && i < (int)g_violations.size() ? g_violations[i].c_str() : ""; }

// ---- registration calls emitted by the compiler for the host side of a HIP source
void **__hipRegisterFatBinary(const void *) { static void *handle = nullptr; return &handle; }
void __hipUnregisterFatBinary(void **) {}
void __hipRegisterFunction(void **, const void *, char *, const char *, unsigned, void *, void *, void *, void *, int *) {}
void __hipRegisterVar(void **, void *, char *, char *, int, size_t, int, int) {}
hipError_t __hipPushCallConfiguration(dim3 grid, dim3 block, size_t shmem, hipStream_t stream) {
    g_call_stack.push_back(CallConfig{grid, block, shmem, stream});
    return hipSuccess;
}
hipError_t __hipPopCallConfiguration(dim3 *grid, dim3 *block, size_t *shmem, hipStream_t *stream) {
    if (g_call_stack.empty()) return hipErrorInvalidValue;
    const CallConfig c = g_call_stack.back();
    g_call_stack.pop_back();
    *grid = c.grid; *block = c.block; *shmem = c.shmem; *stream = c.stream;
    return hipSuccess;
}

}  // extern "C"

// ---- the runtime API (C++ linkage is irrelevant: the HIP headers declare these extern "C")

hipError_t hipGetLastError(void) { const hipError_t e = g_last_error; g_last_error = hipSuccess; return e; }
const char *hipGetErrorString(hipError_t e) {
    switch (e) {
        case hipSuccess: return "no error";
        case hipErrorNotReady: return "not ready";
        case hipErrorInvalidHandle: return "invalid handle (stub: object misuse)";
        case hipErrorInvalidValue: return "invalid value";
        default: return "stub error";
    }
}
hipError_t hipGetDevice(int *dev) { *dev = 0; return hipSuccess; }
hipError_t hipDeviceGetAttribute(int *v, hipDeviceAttribute_t attr, int) {
    *v = attr == hipDeviceAttributeMultiprocessorCount ? 256 : 0;
    return hipSuccess;
}
hipError_t hipFuncSetAttribute(const void *, hipFuncAttribute, int value) {
    if (value > 160 * 1024) return violation(hipErrorInvalidValue, "hipFuncSetAttribute: %d bytes of LDS", value);
    return hipSuccess;
}
hipError_t hipGetSymbolAddress(void **ptr, const void *) {
    *ptr = reinterpret_cast<void *>((uintptr_t)0x7f0000000000ull);     // never dereferenced: kernels do not run
    return hipSuccess;
}

hipError_t hipDeviceSynchronize(void) {
    for (Stream *s : g_streams)
        if (!s->destroyed && s->capture) return violation(hipErrorStreamCaptureUnsupported, "hipDeviceSynchronize while stream %d is capturing", s->id);
    g_null_stream.completed = g_null_stream.submitted;
    for (Stream *s : g_streams) s->completed = s->submitted;
    ++g_stats.device_syncs;
    return hipSuccess;
}

static hipError_t new_stream(hipStream_t *out, bool masked) {
    for (Stream *s : g_streams)
        if (!s->destroyed && s->capture && masked)
            return violation(hipErrorStreamCaptureUnsupported, "CU-masked stream created while stream %d is capturing", s->id);
    if (masked && any_pending()) return violation(hipErrorInvalidValue, "CU-masked stream created while submitted work is pending");
    Stream *s = new Stream{g_next_id++};
    s->masked = masked;
    g_streams.insert(s);
    *out = reinterpret_cast<hipStream_t>(s);
    ++g_stats.streams_created;
    return hipSuccess;
}
hipError_t hipStreamCreateWithFlags(hipStream_t *out, unsigned) { return new_stream(out, false); }
hipError_t hipExtStreamCreateWithCUMask(hipStream_t *out, uint32_t words, const uint32_t *mask) {
    uint32_t any = 0;
    for (uint32_t i = 0; i < words; ++i) any |= mask[i];
    if (!words || !any) return violation(hipErrorInvalidValue, "empty CU mask");
    return new_stream(out, true);
}
hipError_t hipStreamDestroy(hipStream_t st) {
    bool ok;
    Stream *s = as_stream(st, "hipStreamDestroy", &ok);
    if (!ok) return hipErrorInvalidHandle;
    if (s == &g_null_stream) return violation(hipErrorInvalidHandle, "hipStreamDestroy of the null stream");
    if (s->capture) return violation(hipErrorStreamCaptureUnsupported, "stream %d destroyed while capturing", s->id);
    if (s->masked) ++g_stats.masked_streams_destroyed;
    s->destroyed = true;
    return hipSuccess;
}
hipError_t hipStreamSynchronize(hipStream_t st) {
    bool ok;
    Stream *s = as_stream(st, "hipStreamSynchronize", &ok);
    if (!ok) return hipErrorInvalidHandle;
    if (s->capture) return violation(hipErrorStreamCaptureUnsupported, "hipStreamSynchronize on capturing stream %d", s->id);
    complete(s, s->submitted);
    return hipSuccess;
}

hipError_t hipEventCreateWithFlags(hipEvent_t *out, unsigned) {
    Event *e = new Event{g_next_id++};
    g_events.insert(e);
    *out = reinterpret_cast<hipEvent_t>(e);
    ++g_stats.events_created;
    return hipSuccess;
}
hipError_t hipEventCreate(hipEvent_t *out) { return hipEventCreateWithFlags(out, 0); }
hipError_t hipEventDestroy(hipEvent_t ev) {
    Event *e = as_event(ev, "hipEventDestroy");
    if (!e) return hipErrorInvalidHandle;
    e->destroyed = true;
    return hipSuccess;
}
hipError_t hipEventRecord(hipEvent_t ev, hipStream_t st) {
    Event *e = as_event(ev, "hipEventRecord");
    bool ok;
    Stream *s = as_stream(st, "hipEventRecord", &ok);
    if (!e || !ok) return hipErrorInvalidHandle;
    e->recorded = true;
    e->launches_at_record = g_launch_clock;
    if (s->capture) {
        e->capture = s->capture;
        e->nodes = s->frontier;
        e->stream = nullptr;
    } else {
        e->capture = nullptr;
        e->nodes.clear();
        e->stream = s;
        e->pos = s->submitted;
    }
    return hipSuccess;
}
hipError_t hipStreamWaitEvent(hipStream_t st, hipEvent_t ev, unsigned) {
    Event *e = as_event(ev, "hipStreamWaitEvent");
    bool ok;
    Stream *s = as_stream(st, "hipStreamWaitEvent", &ok);
    if (!e || !ok) return hipErrorInvalidHandle;
    if (!e->recorded) return violation(hipErrorInvalidHandle, "stream %d waits on event %d, which was never recorded", s->id, e->id);
    if (e->capture) {
        Graph *g = e->capture;
        if (g->ended || g->destroyed)
            return violation(hipErrorStreamCaptureIsolation, "stream %d waits on event %d whose last record belongs to capture %d, which has ended",
                             s->id, e->id, g->id);
        if (s->capture && s->capture != g)
            return violation(hipErrorStreamCaptureIsolation, "stream %d of capture %d waits on event %d of capture %d", s->id, s->capture->id, e->id, g->id);
        if (!s->capture) {                       // the stream joins the capture
            s->capture = g;
            s->frontier.clear();
            s->launched_in_capture = false;
            g->joined.push_back(s);
        }
        for (int n : e->nodes)
            if (std::find(s->frontier.begin(), s->frontier.end(), n) == s->frontier.end()) s->frontier.push_back(n);
        return hipSuccess;
    }
    if (s->capture)
        return violation(hipErrorStreamCaptureIsolation, "capturing stream %d waits on event %d, recorded outside the capture", s->id, e->id);
    if (e->stream != s) {                    // the wait is an operation of the stream: whoever waits for the stream waits for it
        ++s->submitted;
        s->waits.push_back({s->submitted, Dep{e->stream, e->pos}});
    }
    return hipSuccess;
}
hipError_t hipEventQuery(hipEvent_t ev) {
    Event *e = as_event(ev, "hipEventQuery");
    if (!e) return hipErrorInvalidHandle;
    if (!e->recorded) return hipSuccess;
    if (e->capture) return violation(hipErrorInvalidHandle, "hipEventQuery of event %d, recorded in a capture", e->id);
    return e->stream->completed >= e->pos ? hipSuccess : hipErrorNotReady;
}
hipError_t hipEventSynchronize(hipEvent_t ev) {
    Event *e = as_event(ev, "hipEventSynchronize");
    if (!e) return hipErrorInvalidHandle;
    if (!e->recorded) return hipSuccess;
    if (e->capture) return violation(hipErrorInvalidHandle, "hipEventSynchronize on event %d, recorded in a capture", e->id);
    complete(e->stream, e->pos);
    return hipSuccess;
}
hipError_t hipEventElapsedTime(float *ms, hipEvent_t a, hipEvent_t b) {
    Event *ea = as_event(a, "hipEventElapsedTime"), *eb = as_event(b, "hipEventElapsedTime");
    if (!ea || !eb) return hipErrorInvalidHandle;
    if (!ea->recorded || !eb->recorded || ea->capture || eb->capture)
        return violation(hipErrorInvalidHandle, "hipEventElapsedTime between events %d and %d: not recorded eagerly", ea->id, eb->id);
    if (ea->stream->completed < ea->pos || eb->stream->completed < eb->pos) return hipErrorNotReady;
    // a fake clock: a microsecond per kernel launched (eagerly or inside replayed graphs) between the two records
    *ms = (float)(eb->launches_at_record - ea->launches_at_record) * 1e-3f + 1e-3f;
    return hipSuccess;
}

hipError_t hipLaunchKernel(const void *func, dim3 grid, dim3 block, void **, size_t shmem, hipStream_t st) {
    bool ok;
    Stream *s = as_stream(st, "hipLaunchKernel", &ok);
    if (!ok) return hipErrorInvalidHandle;
    if (!func) return violation(hipErrorInvalidDeviceFunction, "kernel launch without a function");
    const uint64_t threads = (uint64_t)block.x * block.y * block.z;
    if (!grid.x || !grid.y || !grid.z || !threads || threads > 1024 || grid.y > 65535 || grid.z > 65535)
        return violation(hipErrorInvalidConfiguration, "kernel launch with grid (%u, %u, %u) block (%u, %u, %u)", grid.x, grid.y, grid.z,
                         block.x, block.y, block.z);
    if (shmem > 160 * 1024) return violation(hipErrorInvalidValue, "kernel launch with %zu bytes of dynamic LDS", shmem);
    ++g_stats.kernel_launches;
    if (s->capture) {
        add_capture_node(s);
    } else {
        submit_eager(s);
        ++g_launch_clock;
    }
    return hipSuccess;
}

hipError_t hipStreamBeginCapture(hipStream_t st, hipStreamCaptureMode) {
    bool ok;
    Stream *s = as_stream(st, "hipStreamBeginCapture", &ok);
    if (!ok) return hipErrorInvalidHandle;
    if (s == &g_null_stream) return violation(hipErrorStreamCaptureUnsupported, "capture on the null stream");
    if (s->capture) return violation(hipErrorIllegalState, "stream %d is already capturing", s->id);
    Graph *g = new Graph{g_next_id++};
    g_graphs.insert(g);
    g->origin = s;
    s->capture = g;
    s->frontier.clear();
    s->launched_in_capture = false;
    ++g_stats.captures;
    return hipSuccess;
}
hipError_t hipStreamEndCapture(hipStream_t st, hipGraph_t *out) {
    bool ok;
    Stream *s = as_stream(st, "hipStreamEndCapture", &ok);
    *out = nullptr;
    if (!ok) return hipErrorInvalidHandle;
    Graph *g = s->capture;
    if (!g) return violation(hipErrorIllegalState, "hipStreamEndCapture on stream %d, which is not capturing", s->id);
    if (g->origin != s) return violation(hipErrorStreamCaptureUnmatched, "hipStreamEndCapture on stream %d, capture %d began elsewhere", s->id, g->id);
    hipError_t rc = hipSuccess;
    for (Stream *j : g->joined) {
        for (int n : j->frontier)
            if (!reaches(g, s->frontier, n))
                rc = violation(hipErrorStreamCaptureUnjoined, "capture %d ends with node %d of stream %d not joined into the origin stream", g->id, n, j->id);
        if (!j->launched_in_capture) ++g_stats.empty_branches;     // forked, nothing launched: a branch without a node
        else ++g->side_branches;
        j->capture = nullptr;
        j->frontier.clear();
    }
    s->capture = nullptr;
    s->frontier.clear();
    g->ended = true;
    if (rc != hipSuccess) { g->destroyed = true; return rc; }
    g_stats.max_graph_nodes = std::max(g_stats.max_graph_nodes, (int)g->nodes.size());
    *out = reinterpret_cast<hipGraph_t>(g);
    return hipSuccess;
}
hipError_t hipGraphInstantiate(hipGraphExec_t *out, hipGraph_t gr, hipGraphNode_t *, char *, size_t) {
    Graph *g = reinterpret_cast<Graph *>(gr);
    if (!gr || !g_graphs.count(g) || g->destroyed || !g->ended) return violation(hipErrorInvalidHandle, "hipGraphInstantiate of a bad graph %p", (void *)gr);
    Exec *e = new Exec{g_next_id++};
    e->graph = g;
    e->n_nodes = (int)g->nodes.size();
    e->side_branches = g->side_branches;
    g_execs.insert(e);
    *out = reinterpret_cast<hipGraphExec_t>(e);
    ++g_stats.instantiations;
    count_live();
    return hipSuccess;
}
hipError_t hipGraphDestroy(hipGraph_t gr) {
    Graph *g = reinterpret_cast<Graph *>(gr);
    if (!gr || !g_graphs.count(g)) return violation(hipErrorInvalidHandle, "hipGraphDestroy of unknown graph %p", (void *)gr);
    if (g->destroyed) return violation(hipErrorInvalidHandle, "graph %d destroyed twice", g->id);
    g->destroyed = true;
    return hipSuccess;
}
hipError_t hipGraphExecDestroy(hipGraphExec_t ex) {
    Exec *e = reinterpret_cast<Exec *>(ex);
    if (!ex || !g_execs.count(e)) return violation(hipErrorInvalidHandle, "hipGraphExecDestroy of unknown executable %p", (void *)ex);
    if (e->destroyed) return violation(hipErrorInvalidHandle, "executable %d destroyed twice", e->id);
    for (const Dep &l : e->launches)
        if (l.stream->completed < l.pos)
            return violation(hipErrorInvalidHandle, "executable %d destroyed while its launch (operation %llu of stream %d) may still be running",
                             e->id, (unsigned long long)l.pos, l.stream->id);
    e->destroyed = true;
    ++g_stats.execs_destroyed;
    return hipSuccess;
}
hipError_t hipGraphLaunch(hipGraphExec_t ex, hipStream_t st) {
    Exec *e = reinterpret_cast<Exec *>(ex);
    bool ok;
    Stream *s = as_stream(st, "hipGraphLaunch", &ok);
    if (!ok) return hipErrorInvalidHandle;
    if (!ex || !g_execs.count(e)) return violation(hipErrorInvalidHandle, "hipGraphLaunch of unknown executable %p", (void *)ex);
    if (e->destroyed) return violation(hipErrorInvalidHandle, "hipGraphLaunch of destroyed executable %d", e->id);
    if (s->capture) return violation(hipErrorStreamCaptureUnsupported, "hipGraphLaunch into capturing stream %d", s->id);
    submit_eager(s);
    e->launches.erase(std::remove_if(e->launches.begin(), e->launches.end(), [](const Dep &l) { return l.stream->completed >= l.pos; }),
                      e->launches.end());
    e->launches.push_back(Dep{s, s->submitted});
    g_launch_clock += (uint64_t)e->n_nodes;
    ++g_stats.graph_launches;
    count_live();
    return hipSuccess;
}
