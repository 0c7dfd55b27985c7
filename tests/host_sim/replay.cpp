// Replays, on the CPU against the HIP stand-in (hip_stub.cpp), the host-side call sequences of
// libdynlayer that matter for object lifetimes: a tuning run (with four micro-batches too, which
// the device search itself refuses), a run that overflows the graph cache back to back without
// host waits, eager and profiled forwards, CU-masked schedules, the allocation-free entry point.
// TEST INFRASTRUCTURE.  Prints the stand-in's counters as one JSON object; exit status 1 if the
// stand-in saw a violation, a forward failed, or objects were left alive after dyn_layer_destroy.
//
//   replay <shape file> tune <max_k> <partitions> <warmup> <iters>
//   replay <shape file> evict
//   replay <shape file> mixed
//   replay <shape file> opclass <k> <stagger> <memory CUs> <use_graph>
// shape file: "dtype n_layers hidden n_q n_kv head_dim inter n_experts top_k page_size n_seqs" then "q_len ctx_len" per sequence.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include <hip/hip_runtime.h>

#include "../../include/dynlayer.h"
#include "hip_stub.h"

namespace {

int g_failures = 0;

#define EXPECT_OK(expr)                                                                         \
    do {                                                                                        \
        dyn_status rc_ = (expr);                                                                \
        if (rc_ != DYN_OK) {                                                                    \
            fprintf(stderr, "replay: %s -> %d: %s\n", #expr, (int)rc_, dyn_last_error());      \
            ++g_failures;                                                                       \
        }                                                                                       \
    } while (0)

struct Setup {
    dyn_layer_config cfg{};
    std::vector<int32_t> q_start, ctx;
    int n_tokens = 0, n_seqs = 0, max_pages = 1;
    std::vector<dyn_layer_weights> weights;
    std::vector<void *> k_layers, v_layers;      // the caches named layer by layer (used by every other forward of "mixed")
    dyn_layer *layer = nullptr;
    dyn_batch batch{};
};

// Device pointers are never dereferenced (no kernel runs): distinct, aligned fake addresses.
void *fake(uintptr_t n) { return reinterpret_cast<void *>((uintptr_t)0x100000000000ull + n * 0x100000000ull); }

bool load(const char *path, Setup &s) {
    FILE *f = fopen(path, "r");
    if (!f) return false;
    int vals[11];
    for (int &v : vals)
        if (fscanf(f, "%d", &v) != 1) return false;
    s.cfg.dtype = vals[0]; s.cfg.n_layers = vals[1]; s.cfg.hidden = vals[2]; s.cfg.n_q_heads = vals[3];
    s.cfg.n_kv_heads = vals[4]; s.cfg.head_dim = vals[5]; s.cfg.mlp_inter = vals[6]; s.cfg.n_experts = vals[7];
    s.cfg.top_k = vals[8]; s.cfg.page_size = vals[9]; s.n_seqs = vals[10];
    s.cfg.rms_eps = 1e-6f; s.cfg.rope_base = 10000.f;
    s.q_start.push_back(0);
    for (int i = 0; i < s.n_seqs; ++i) {
        int q, c;
        if (fscanf(f, "%d %d", &q, &c) != 2) return false;
        s.q_start.push_back(s.q_start.back() + q);
        s.ctx.push_back(c);
        s.max_pages = std::max(s.max_pages, (c + s.cfg.page_size - 1) / s.cfg.page_size);
    }
    fclose(f);
    s.n_tokens = s.q_start.back();
    for (int l = 0; l < s.cfg.n_layers; ++l) {
        dyn_layer_weights w{};
        w.w_qkv = fake(10 + 8 * l); w.w_o = fake(11 + 8 * l); w.w_gate_up = fake(12 + 8 * l); w.w_down = fake(13 + 8 * l);
        w.g_norm1 = fake(14 + 8 * l); w.g_norm2 = fake(15 + 8 * l);
        w.w_router = s.cfg.n_experts ? (const float *)fake(16 + 8 * l) : nullptr;
        s.weights.push_back(w);
    }
    EXPECT_OK(dyn_layer_create(&s.cfg, s.weights.data(), &s.layer));
    if (!s.layer) return false;
    dyn_batch &b = s.batch;
    b.n_tokens = s.n_tokens; b.n_seqs = s.n_seqs;
    b.x = fake(1); b.y = fake(2); b.seq_of_token = (const int32_t *)fake(3); b.pos_of_token = (const int32_t *)fake(4);
    b.block_table = (const int32_t *)fake(5); b.max_pages_per_seq = s.max_pages; b.q_start_host = s.q_start.data();
    b.k_cache = fake(6); b.v_cache = fake(7); b.kv_layer_stride = 1 << 20;
    b.workspace = fake(8); b.workspace_bytes = dyn_layer_workspace_bytes(s.layer, s.n_tokens, s.max_pages);
    for (int l = 0; l < s.cfg.n_layers; ++l) {
        s.k_layers.push_back(fake(200 + 2 * (s.cfg.n_layers - l)));
        s.v_layers.push_back(fake(201 + 2 * l));
    }
    return true;
}

// The device search as it once was, step for step, with every candidate a HIP graph (prepare every
// candidate's streams, then per candidate: warm-up forwards, three timed runs between two events, a
// stream synchronisation) - the sequence that died inside the runtime on the GPU - and then dyn_tune
// itself, which times the same candidates with eager launches.
void tune_like(Setup &s, int max_k, int partitions, int warmup, int iters) {
    dyn_scheduler *sch = nullptr;
    EXPECT_OK(dyn_scheduler_create(&s.cfg, s.n_tokens, s.n_seqs, s.q_start.data(), &sch));
    dyn_tune_options opt{};
    opt.max_k = max_k; opt.partitions = partitions; opt.n_cus = 256; opt.use_graph = 1; opt.min_gain = 0.02f;
    const int n = dyn_tune_candidates(sch, s.ctx.data(), &opt, nullptr, 0);
    std::vector<dyn_tune_candidate> cand((size_t)std::max(n, 1));
    dyn_tune_candidates(sch, s.ctx.data(), &opt, cand.data(), n);
    hipStream_t stream;
    hipEvent_t a, b;
    if (hipStreamCreateWithFlags(&stream, hipStreamNonBlocking) != hipSuccess || hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) ++g_failures;
    for (int i = 0; i < n; ++i) {
        dyn_schedule sched;
        EXPECT_OK(dyn_tune_record(sch, &cand[i], 256, 1, &sched));
        EXPECT_OK(dyn_layer_prepare(s.layer, &sched));
    }
    int graphs = 0;
    for (int i = 0; i < n; ++i) {
        dyn_schedule sched;
        EXPECT_OK(dyn_tune_record(sch, &cand[i], 256, 1, &sched));
        for (int run = -1; run < 3; ++run) {
            if (run >= 0 && hipEventRecord(a, stream) != hipSuccess) ++g_failures;
            for (int it = 0; it < (run < 0 ? warmup : iters); ++it) EXPECT_OK(dyn_layer_forward(s.layer, &s.batch, &sched, stream));
            if (run < 0) continue;
            float ms = 0.f;
            if (hipEventRecord(b, stream) != hipSuccess || hipEventSynchronize(b) != hipSuccess || hipEventElapsedTime(&ms, a, b) != hipSuccess) ++g_failures;
        }
        if (hipStreamSynchronize(stream) != hipSuccess) ++g_failures;
        ++graphs;
    }
    fprintf(stderr, "replay: %d candidates, each captured, replayed and timed\n", graphs);
    {                                      // and the library's own search on the same batch (eager launches, no graph)
        dyn_schedule out;
        dyn_tune_result res{};
        opt.warmup = warmup; opt.iters = iters;
        EXPECT_OK(dyn_tune(s.layer, &s.batch, s.ctx.data(), &opt, stream, sch, &out, &res, nullptr, 0));
        EXPECT_OK(dyn_layer_forward(s.layer, &s.batch, &out, stream));
    }
    if (hipDeviceSynchronize() != hipSuccess) ++g_failures;
    dyn_scheduler_destroy(sch);
    dyn_layer_destroy(s.layer);
    if (hipEventDestroy(a) != hipSuccess || hipEventDestroy(b) != hipSuccess || hipStreamDestroy(stream) != hipSuccess) ++g_failures;
}

// More distinct graph schedules than the cache holds, two forwards each, two passes, no host wait
// in between: executables leave the cache while their last replay has not completed.
void evict_like(Setup &s) {
    dyn_scheduler *sch = nullptr;
    EXPECT_OK(dyn_scheduler_create(&s.cfg, s.n_tokens, s.n_seqs, s.q_start.data(), &sch));
    dyn_tune_options opt{};
    opt.max_k = 2; opt.n_cus = 256;
    const int n = dyn_tune_candidates(sch, s.ctx.data(), &opt, nullptr, 0);
    std::vector<dyn_tune_candidate> cand((size_t)std::max(n, 1));
    dyn_tune_candidates(sch, s.ctx.data(), &opt, cand.data(), n);
    hipStream_t stream;
    if (hipStreamCreateWithFlags(&stream, hipStreamNonBlocking) != hipSuccess) ++g_failures;
    int used = 0;
    for (int pass = 0; pass < 3; ++pass) {
        used = 0;
        for (int i = 0; i < n && used < 24; ++i) {
            if (cand[i].cus_first) continue;
            ++used;
            dyn_schedule sched;
            EXPECT_OK(dyn_tune_record(sch, &cand[i], 256, 1, &sched));
            EXPECT_OK(dyn_layer_forward(s.layer, &s.batch, &sched, stream));
            EXPECT_OK(dyn_layer_forward(s.layer, &s.batch, &sched, stream));
        }
        if (pass == 1 && hipStreamSynchronize(stream) != hipSuccess) ++g_failures;   // the third pass retires what the second left
    }
    fprintf(stderr, "replay: %d schedules x 2 forwards x 3 passes\n", used);
    // destroy with work still pending on the stream: dyn_layer_destroy waits for the device itself
    dyn_scheduler_destroy(sch);
    dyn_layer_destroy(s.layer);
    if (hipStreamDestroy(stream) != hipSuccess) ++g_failures;
}

// Eager, profiled, graph and masked forwards interleaved on one handle, the allocation-free entry
// point, an empty micro-batch, error paths that must leave no capture open.
void mixed(Setup &s) {
    hipStream_t stream;
    if (hipStreamCreateWithFlags(&stream, hipStreamNonBlocking) != hipSuccess) ++g_failures;
    dyn_scheduler *sch = nullptr;
    EXPECT_OK(dyn_scheduler_create(&s.cfg, s.n_tokens, s.n_seqs, s.q_start.data(), &sch));
    dyn_tune_options opt{};
    opt.max_k = 4; opt.partitions = 3; opt.n_cus = 256;
    const int n = dyn_tune_candidates(sch, s.ctx.data(), &opt, nullptr, 0);
    std::vector<dyn_tune_candidate> cand((size_t)std::max(n, 1));
    dyn_tune_candidates(sch, s.ctx.data(), &opt, cand.data(), n);
    dyn_schedule seq{};
    seq.mode = DYN_SCHED_SEQUENTIAL;
    for (int round = 0; round < 2; ++round)
        for (int i = 0; i < n; ++i) {
            dyn_schedule sched;
            EXPECT_OK(dyn_tune_record(sch, &cand[i], 256, (i + round) % 2, &sched));   // alternately eager and captured
            if (round == 0 && i % 5 == 0) {
                if (hipDeviceSynchronize() != hipSuccess) ++g_failures;                // masked streams are made on an idle device
                EXPECT_OK(dyn_layer_prepare(s.layer, &sched));
            }                               // other masked candidates: the forward creates the stream itself (and waits for the device first)
            // every other candidate with one cache pointer per layer instead of base + stride (another graph: the key holds them)
            s.batch.k_cache_layers = i % 2 ? s.k_layers.data() : nullptr;
            s.batch.v_cache_layers = i % 2 ? s.v_layers.data() : nullptr;
            EXPECT_OK(dyn_layer_forward(s.layer, &s.batch, &sched, stream));
            if (i % 7 == 0) {
                EXPECT_OK(dyn_layer_set_profiling(s.layer, 1));
                dyn_schedule eager = sched;
                eager.use_graph = 0;
                EXPECT_OK(dyn_layer_forward(s.layer, &s.batch, &eager, stream));
                if (hipStreamSynchronize(stream) != hipSuccess) ++g_failures;
                int n_rec = 0;
                std::vector<dyn_slot_time> recs(4096);
                EXPECT_OK(dyn_layer_get_slot_times(s.layer, recs.data(), (int)recs.size(), &n_rec));
                EXPECT_OK(dyn_layer_set_profiling(s.layer, 0));
            }
            if (i % 3 == 0) EXPECT_OK(dyn_layer_forward_noalloc(s.layer, &s.batch, stream));
            if (i % 11 == 0) {             // a forward that fails validation must not leave anything open
                dyn_batch bad = s.batch;
                bad.workspace_bytes = 16;
                if (dyn_layer_forward(s.layer, &bad, &sched, stream) != DYN_ERR_WORKSPACE) ++g_failures;
            }
            EXPECT_OK(dyn_layer_forward(s.layer, &s.batch, &seq, stream));
        }
    dyn_scheduler_destroy(sch);
    dyn_layer_destroy(s.layer);
    if (hipStreamDestroy(stream) != hipSuccess) ++g_failures;
}

// Partitions by operator class instead of by micro-batch: every micro-batch's attention on a
// "memory" partition (the low `mem_cus` bits of the mask), its other operators on the rest of the
// device, so consecutive operators of one micro-batch change streams.
void opclass(Setup &s, int k, int stagger, int mem_cus, int use_graph) {
    hipStream_t stream;
    if (hipStreamCreateWithFlags(&stream, hipStreamNonBlocking) != hipSuccess) ++g_failures;
    std::vector<int> chain = {DYN_OP_NORM1, DYN_OP_QKV, DYN_OP_ROPE_KV, DYN_OP_ATTN, DYN_OP_OPROJ, DYN_OP_NORM2};
    if (s.cfg.n_experts) chain.push_back(DYN_OP_ROUTE);
    chain.insert(chain.end(), {DYN_OP_GATE_UP, DYN_OP_SILU, DYN_OP_DOWN});
    std::vector<int32_t> rows(k + 1);
    for (int i = 0; i <= k; ++i) rows[i] = s.q_start[(size_t)s.n_seqs * i / k];
    std::vector<uint32_t> masks(16, 0u);
    for (int i = 0; i < 256; ++i) masks[(i < mem_cus ? 0 : 8) + i / 32] |= 1u << (i % 32);
    std::vector<dyn_slot> slots;
    std::vector<int> pos(k, 0);
    for (int tick = 0;; ++tick) {
        bool done = true;
        for (int b = 0; b < k; ++b) done = done && pos[b] >= (int)chain.size();
        if (done) break;
        for (int b = 0; b < k; ++b) {
            if (pos[b] >= (int)chain.size() || tick < b * stagger) continue;
            const int op = chain[pos[b]++];
            slots.push_back(dyn_slot{(uint8_t)op, (uint8_t)b, 1, (uint8_t)b, (uint8_t)(op == DYN_OP_ATTN ? 1 : 2)});
        }
    }
    dyn_schedule sched{};
    sched.mode = DYN_SCHED_EXPLICIT; sched.k = k; sched.nano_rows = rows.data(); sched.n_streams = k;
    sched.n_partitions = 2; sched.cu_masks = masks.data(); sched.cu_mask_words = 8;
    sched.n_slots = (int)slots.size(); sched.slots = slots.data(); sched.use_graph = use_graph;
    EXPECT_OK(dyn_schedule_validate(s.layer, &s.batch, &sched));
    EXPECT_OK(dyn_layer_prepare(s.layer, &sched));
    for (int it = 0; it < 4; ++it) EXPECT_OK(dyn_layer_forward(s.layer, &s.batch, &sched, stream));
    if (hipStreamSynchronize(stream) != hipSuccess) ++g_failures;
    EXPECT_OK(dyn_layer_set_profiling(s.layer, 1));
    dyn_schedule eager = sched;
    eager.use_graph = 0;
    EXPECT_OK(dyn_layer_forward(s.layer, &s.batch, &eager, stream));
    if (hipStreamSynchronize(stream) != hipSuccess) ++g_failures;
    int n_rec = 0;
    std::vector<dyn_slot_time> recs(8192);
    EXPECT_OK(dyn_layer_get_slot_times(s.layer, recs.data(), (int)recs.size(), &n_rec));
    EXPECT_OK(dyn_layer_set_profiling(s.layer, 0));
    dyn_layer_destroy(s.layer);
    if (hipStreamDestroy(stream) != hipSuccess) ++g_failures;
}

// The checker checked: each misuse the stand-in exists to catch is committed against it directly,
// once, and must be counted.  Returns the number of misuses that went unseen.
int selftest() {
    int missed = 0;
    auto expect_violation = [&](const char *what, auto &&fn) {
        const int before = hipstub_get_stats()->violations;
        fn();
        if (hipstub_get_stats()->violations == before) { fprintf(stderr, "selftest: not detected: %s\n", what); ++missed; }
    };
    auto kernel = [](hipStream_t st) { (void)hipLaunchKernel((const void *)&selftest, dim3(1), dim3(64), nullptr, 0, st); };
    hipStream_t a, b, c;
    hipEvent_t e1, e2, never;
    (void)hipStreamCreateWithFlags(&a, 0); (void)hipStreamCreateWithFlags(&b, 0); (void)hipStreamCreateWithFlags(&c, 0);
    (void)hipEventCreate(&e1); (void)hipEventCreate(&e2); (void)hipEventCreate(&never);
    hipGraph_t g = nullptr;
    hipGraphExec_t x = nullptr;
    // a proper fork / join capture first
    (void)hipStreamBeginCapture(a, hipStreamCaptureModeRelaxed);
    kernel(a);
    (void)hipEventRecord(e1, a);
    (void)hipStreamWaitEvent(b, e1, 0);
    kernel(b);
    (void)hipEventRecord(e2, b);
    (void)hipStreamWaitEvent(a, e2, 0);
    (void)hipStreamEndCapture(a, &g);
    (void)hipGraphInstantiate(&x, g, nullptr, nullptr, 0);
    if (hipstub_get_stats()->violations) { fprintf(stderr, "selftest: a legal capture was flagged\n"); ++missed; }
    (void)hipGraphLaunch(x, c);
    expect_violation("executable destroyed while its launch is pending", [&] { (void)hipGraphExecDestroy(x); });
    expect_violation("wait on an event whose capture has ended", [&] { (void)hipStreamWaitEvent(c, e2, 0); });
    expect_violation("wait on an event never recorded", [&] { (void)hipStreamWaitEvent(c, never, 0); });
    expect_violation("query of a capture event", [&] { (void)hipEventQuery(e1); });
    expect_violation("unjoined work at the end of a capture", [&] {
        hipGraph_t g2 = nullptr;
        (void)hipStreamBeginCapture(a, hipStreamCaptureModeRelaxed);
        kernel(a);
        (void)hipEventRecord(e1, a);
        (void)hipStreamWaitEvent(b, e1, 0);
        kernel(b);
        (void)hipStreamEndCapture(a, &g2);
    });
    expect_violation("capturing stream waits on an eager event", [&] {
        hipGraph_t g3 = nullptr;
        (void)hipEventRecord(e2, c);
        (void)hipStreamBeginCapture(a, hipStreamCaptureModeRelaxed);
        (void)hipStreamWaitEvent(a, e2, 0);
        (void)hipStreamEndCapture(a, &g3);
        if (g3) (void)hipGraphDestroy(g3);
    });
    expect_violation("graph launch into a capturing stream", [&] {
        hipGraph_t g4 = nullptr;
        (void)hipStreamBeginCapture(a, hipStreamCaptureModeRelaxed);
        (void)hipGraphLaunch(x, a);
        (void)hipStreamEndCapture(a, &g4);
        if (g4) (void)hipGraphDestroy(g4);
    });
    expect_violation("device synchronisation during a capture", [&] {
        hipGraph_t g5 = nullptr;
        (void)hipStreamBeginCapture(a, hipStreamCaptureModeRelaxed);
        (void)hipDeviceSynchronize();
        (void)hipStreamEndCapture(a, &g5);
        if (g5) (void)hipGraphDestroy(g5);
    });
    expect_violation("CU-masked stream created while work is pending", [&] {
        hipStream_t m;
        const uint32_t mask = 0xffff;
        kernel(c);
        (void)hipExtStreamCreateWithCUMask(&m, 1, &mask);
    });
    (void)hipDeviceSynchronize();
    if (hipGraphExecDestroy(x) != hipSuccess) { fprintf(stderr, "selftest: destroy after completion refused\n"); ++missed; }
    expect_violation("launch of a destroyed executable", [&] { (void)hipGraphLaunch(x, c); });
    expect_violation("executable destroyed twice", [&] { (void)hipGraphExecDestroy(x); });
    (void)hipEventDestroy(e1);
    expect_violation("record of a destroyed event", [&] { (void)hipEventRecord(e1, c); });
    (void)hipStreamDestroy(b);
    expect_violation("launch on a destroyed stream", [&] { kernel(b); });
    expect_violation("empty grid", [&] { (void)hipLaunchKernel((const void *)&selftest, dim3(0), dim3(64), nullptr, 0, c); });
    return missed;
}

}  // namespace

int main(int argc, char **argv) {
    if (argc == 2 && std::string(argv[1]) == "selftest") {
        const int missed = selftest();
        printf("{\"missed\": %d, \"violations\": %d}\n", missed, hipstub_get_stats()->violations);
        return missed ? 1 : 0;
    }
    if (argc < 3) { fprintf(stderr, "usage: replay <shape file> tune <max_k> <partitions> <warmup> <iters> | evict | mixed\n"); return 2; }
    Setup s;
    if (!load(argv[1], s)) { fprintf(stderr, "replay: cannot load %s\n", argv[1]); return 2; }
    const std::string mode = argv[2];
    if (mode == "tune" && argc >= 7) tune_like(s, atoi(argv[3]), atoi(argv[4]), atoi(argv[5]), atoi(argv[6]));
    else if (mode == "evict") evict_like(s);
    else if (mode == "mixed") mixed(s);
    else if (mode == "opclass" && argc >= 7) opclass(s, atoi(argv[3]), atoi(argv[4]), atoi(argv[5]), atoi(argv[6]));
    else { fprintf(stderr, "replay: unknown mode\n"); return 2; }
    const hipstub_stats *st = hipstub_get_stats();
    // CU-masked streams live for the process by design; everything else must be gone
    printf("{\"violations\": %d, \"failures\": %d, \"kernel_launches\": %d, \"graph_launches\": %d, \"captures\": %d, "
           "\"instantiations\": %d, \"execs_destroyed\": %d, \"streams_created\": %d, \"events_created\": %d, "
           "\"masked_streams_destroyed\": %d, \"device_syncs\": %d, \"empty_branches\": %d, \"max_graph_nodes\": %d, "
           "\"max_live_execs\": %d, \"max_live_side_branches\": %d, \"live_streams\": %d, \"live_events\": %d, "
           "\"live_graphs\": %d, \"live_execs\": %d}\n",
           st->violations, g_failures, st->kernel_launches, st->graph_launches, st->captures, st->instantiations,
           st->execs_destroyed, st->streams_created, st->events_created, st->masked_streams_destroyed, st->device_syncs,
           st->empty_branches, st->max_graph_nodes, st->max_live_execs, st->max_live_side_branches, st->live_streams,
           st->live_events, st->live_graphs, st->live_execs);
    return st->violations || g_failures || st->live_events || st->live_graphs || st->live_execs ? 1 : 0;
}
