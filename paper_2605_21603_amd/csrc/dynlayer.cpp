// C-ABI library: layer handle, schedule validation, workspace layout and the overlap
// executor (streams, CU-masked partitions, event dependencies, HIP-graph capture).
//
// The executor realises the paper's backend (Section 3.3, Section 4): the schedule names
// what runs where and in which issue order; the dependency state - which dispatch produced
// the rows another consumes - is derived here and turned into event edges between streams.
// Splitting and merging micro-batches is pointer arithmetic on batch-sized buffers
// (Algorithm 1's pre-allocated merge buffers, with every intermediate pre-allocated).
#include "../../include/dynlayer.h"

#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "kernels.h"

namespace dyn {

thread_local std::string g_err;

dyn_status fail(dyn_status st, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return st;
}

}  // namespace dyn

namespace {

using dyn::fail;
using dyn::g_err;

#define HIP_TRY(expr)                                                                                  \
    do {                                                                                               \
        hipError_t e_ = (expr);                                                                        \
        if (e_ != hipSuccess) return fail(DYN_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));        \
    } while (0)

struct Dispatch {
    int layer, op, nano, n_nano, r0, r1, stream, partition;
    bool any_multi;          // some sequence contributes more than one token to rows r0..r1
    bool noop;               // launches nothing: no rows, or the gate when the projection's epilogue applied it
    std::vector<int> deps;   // dispatches (indices into the plan) whose output rows this one reads
    bool lists_ready = false;   // MoE down projection: the gate/up dispatch of the same rows already built its expert lists
    int key() const { return partition * DYN_MAX_STREAMS + stream; }
};

constexpr int kMaxRetiredGraphs = 8, kMaxRetiredBranches = 8;   // evicted executables still waiting for their last replay

// Where everything lives inside the caller's workspace for one forward.  Row-indexed tensors
// ([tokens, width], a micro-batch is a row range) have one region each; scratch that exists only
// while a dispatch runs (split-K planes, split-KV partials, expert lists) has one region per slot
// of the layer's issue order, the same in every layer.  Regions whose lifetimes never overlap
// under the schedule share bytes (plan_layout).
struct SlotScratch {
    size_t planes, part_o, part_ml, lists, moe_planes;   // byte offsets; unused ones are 0
};

struct WsLayout {
    size_t h, qkv, attn, x2, gu, act, xa, xb, plan, total;
    size_t sel, wgt;             // MoE routing: selected experts and their weights per token
    int ld_h, ld_attn, ld_act;   // padded row strides (elements) of the buffers the projections read
    int max_chunks;
    std::vector<SlotScratch> slot;
};

// One region of the layout, for dyn_schedule_regions and the placement itself.
struct Region {
    int kind, slot;              // DYN_REGION_*; slot of the issue order for scratch, -1 for tensors
    size_t bytes, offset;
    std::vector<char> live;      // per slot of the issue order (lifetimes folded over the layers)
    bool always = false;         // alive for the whole forward
    int stream_key = -1;         // scratch: the stream its dispatch runs on
};

struct GraphEntry {
    std::vector<unsigned char> key;   // everything the captured launches were derived from (graph_key)
    hipGraphExec_t exec;
    hipGraph_t graph;
    hipEvent_t last_launch;   // recorded on the caller's stream after every replay
    int side_streams;         // streams of the schedule besides the caller's: parallel branches of the graph
};

}  // namespace

struct dyn_layer {
    dyn_layer_config cfg;
    std::vector<dyn_layer_weights> w;
    dyn::RopeTable rope;
    int chunk_pages;
    // GPU state, created on first use
    hipStream_t streams[(DYN_MAX_PARTITIONS + 1) * DYN_MAX_STREAMS] = {};
    std::vector<uint32_t> stream_mask[(DYN_MAX_PARTITIONS + 1) * DYN_MAX_STREAMS];
    hipStream_t capture_stream = nullptr;
    std::vector<hipEvent_t> events;          // dependency events, one per dispatch of a forward
    hipEvent_t fork_event = nullptr;
    std::vector<GraphEntry> graphs;
    std::vector<GraphEntry> retired;         // evicted from the cache while their last replay may still run
    bool profiling = false;
    std::vector<hipEvent_t> prof_events;     // timing events: fork, then (start, main start, main stop, stop) per dispatch
    std::vector<Dispatch> prof_plan;
};

namespace {

size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

size_t esize(const dyn_layer_config &c) { return c.dtype == DYN_F32 ? 4 : 2; }

int qkv_width(const dyn_layer_config &c) { return (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim; }

struct Sizes {                  // bytes of each whole-batch tensor, and the row strides
    size_t h, qkv, attn, x2, gu, act, xa, xb, plan, sel, wgt;
    int ld_h, ld_attn, ld_act, max_chunks;
};

Sizes tensor_sizes(const dyn_layer *L, int T, int max_pages) {
    const dyn_layer_config &c = L->cfg;
    const size_t e = esize(c), t = (size_t)std::max(T, 0);
    const int pairs = c.n_experts ? c.top_k : 1;
    Sizes z{};
    // Rows of a GEMM input are read 64 bytes at a time by 16 lanes on 16 different rows; with a
    // power-of-two row pitch those land in one L2 channel.  256 bytes of padding per row walks
    // consecutive rows across the channels.
    const int pad = (int)(256 / e);
    z.ld_h = c.hidden + pad;
    z.ld_attn = c.n_q_heads * c.head_dim + pad;
    z.ld_act = c.mlp_inter + pad;
    z.max_chunks = std::max(1, (std::max(max_pages, 1) + L->chunk_pages - 1) / L->chunk_pages);
    z.h = t * z.ld_h * e;
    z.qkv = t * qkv_width(c) * e;
    z.attn = t * z.ld_attn * e;
    z.x2 = t * c.hidden * e;
    // the [gate | up] intermediate exists only when the SiLU gate is not applied in the projection's epilogue
    z.gu = dyn::gemm_gated_supported(c.dtype, 2 * c.mlp_inter, c.hidden) ? 0 : t * pairs * 2 * c.mlp_inter * e;
    z.act = t * pairs * z.ld_act * e;
    z.xa = c.n_layers > 1 ? t * c.hidden * e : 0;
    z.xb = c.n_layers > 2 ? t * c.hidden * e : 0;
    z.plan = (t * z.max_chunks + 2 * t) * 4 * sizeof(int32_t);   // per dispatch: two lists of 2 header words + 2 per entry, one chunk size per token
    z.sel = c.n_experts ? t * c.top_k * sizeof(int32_t) : 0;
    z.wgt = c.n_experts ? t * c.top_k * sizeof(float) : 0;
    return z;
}

// Scratch a dispatch over `rows` token rows holds while it runs (bytes; 0 = none).
struct ScratchBytes { size_t planes, part_o, part_ml, lists, moe_planes; };

ScratchBytes dispatch_scratch(const dyn_layer *L, const Sizes &z, int op, int rows) {
    const dyn_layer_config &c = L->cfg;
    ScratchBytes k{};
    if (rows <= 0) return k;
    const size_t r = (size_t)rows;
    const int H = c.hidden, I = c.mlp_inter, NQKV = qkv_width(c), NQ = c.n_q_heads * c.head_dim;
    const bool moe = c.n_experts > 0, gated = dyn::gemm_gated_supported(c.dtype, 2 * I, H);
    auto planes = [&](int N, int K) {
        return dyn::gemm_uses_plane_buffer(c.dtype, rows, N, K) ? (size_t)dyn::gemm_split_k(c.dtype, N, K) * r * N * sizeof(float) : 0;
    };
    switch (op) {
        case DYN_OP_QKV: k.planes = planes(NQKV, H); break;
        case DYN_OP_OPROJ: k.planes = planes(H, NQ); break;
        case DYN_OP_ATTN:
            k.part_o = r * c.n_q_heads * z.max_chunks * c.head_dim * sizeof(float);
            k.part_ml = r * c.n_q_heads * z.max_chunks * 2 * sizeof(float);
            break;
        case DYN_OP_GATE_UP:
            if (moe) {
                k.lists = r * c.top_k * 2 * c.n_experts * sizeof(int32_t);   // E counts + E lists of up to rows * top_k pairs
                const int S = dyn::gemm_split_k(c.dtype, 2 * I, H, c.n_experts);
                if (!gated && S > 1) k.planes = (size_t)S * r * c.top_k * 2 * I * sizeof(float);
            } else if (!gated) {
                k.planes = planes(2 * I, H);
            }
            break;
        case DYN_OP_DOWN:
            if (moe) {
                k.lists = r * c.top_k * 2 * c.n_experts * sizeof(int32_t);
                k.moe_planes = (size_t)dyn::gemm_split_k(c.dtype, H, I, c.n_experts) * r * c.top_k * H * sizeof(float);
            } else {
                k.planes = planes(H, I);
            }
            break;
        default: break;
    }
    return k;
}

// Upper bound of the workspace any legal schedule of a batch of T tokens needs: every tensor and,
// for every operator, scratch for all T rows at once (a schedule dispatches each (operator,
// micro-batch) once per layer, so its dispatches' scratch adds up to at most that), nothing shared.
size_t ws_bound(const dyn_layer *L, int T, int max_pages) {
    const dyn_layer_config &c = L->cfg;
    const Sizes z = tensor_sizes(L, T, max_pages);
    const size_t t = (size_t)std::max(T, 0);
    const int pairs = c.n_experts ? c.top_k : 1;
    size_t total = 0;
    for (size_t v : {z.h, z.qkv, z.attn, z.x2, z.gu, z.act, z.xa, z.xb, z.plan, z.sel, z.wgt}) total += align_up(v);
    const int widths[4][2] = {{qkv_width(c), c.hidden}, {c.hidden, c.n_q_heads * c.head_dim},
                              {2 * c.mlp_inter, c.hidden}, {c.hidden, c.mlp_inter}};
    for (int i = 0; i < 4; ++i) {
        const int S = dyn::gemm_split_k(c.dtype, widths[i][0], widths[i][1], i >= 2 && c.n_experts ? c.n_experts : 1);
        const size_t prow = (i == 2 ? (size_t)pairs : 1) * t;     // the MoE gate/up projection has a row per (token, expert)
        total += align_up(S > 1 ? (size_t)S * prow * widths[i][0] * sizeof(float) : 0);
    }
    total += align_up(t * c.n_q_heads * z.max_chunks * c.head_dim * sizeof(float)) + align_up(t * c.n_q_heads * z.max_chunks * 2 * sizeof(float));
    if (c.n_experts) {
        const int Sd = dyn::gemm_split_k(c.dtype, c.hidden, c.mlp_inter, c.n_experts);
        total += 2 * align_up(t * c.top_k * 2 * c.n_experts * sizeof(int32_t)) + align_up((size_t)Sd * t * c.top_k * c.hidden * sizeof(float));
    }
    return total + (size_t)256 * 5 * DYN_N_OPS * DYN_MAX_NANO;      // alignment of per-dispatch scratch regions
}

const int kDenseChain[] = {DYN_OP_NORM1, DYN_OP_QKV, DYN_OP_ROPE_KV, DYN_OP_ATTN, DYN_OP_OPROJ,
                           DYN_OP_NORM2, DYN_OP_GATE_UP, DYN_OP_SILU, DYN_OP_DOWN};
const int kMoeChain[] = {DYN_OP_NORM1, DYN_OP_QKV, DYN_OP_ROPE_KV, DYN_OP_ATTN, DYN_OP_OPROJ,
                         DYN_OP_NORM2, DYN_OP_ROUTE, DYN_OP_GATE_UP, DYN_OP_SILU, DYN_OP_DOWN};

const char *op_name(int op) {
    static const char *n[] = {"norm1", "qkv", "rope_kv", "attn", "oproj", "norm2", "route", "gate_up", "silu", "down"};
    return op >= 0 && op < DYN_N_OPS ? n[op] : "?";
}

// The projections' dispatches also run the operator that follows them on the same rows - where
// split-K planes are reduced, inside the reduce kernel (one pass over the planes instead of a
// kernel per operator): qkv -> rotary + cache append, o -> second norm, down -> the next layer's
// first norm.  The slots of those operators stay in the chain (schedules name them, the
// ready-operator rule covers them) and launch nothing.
bool fused_into_producer(int op, int layer) {
    return op == DYN_OP_ROPE_KV || op == DYN_OP_NORM2 || (op == DYN_OP_NORM1 && layer > 0);
}

// Checks of an explicit schedule that need no batch: counts in range, arrays present, masks not empty.
dyn_status check_schedule_fields(const dyn_schedule *s) {
    if (s->k < 1 || s->k > DYN_MAX_NANO) return fail(DYN_ERR_SCHEDULE, "k = %d outside 1..%d", s->k, DYN_MAX_NANO);
    if (!s->nano_rows || !s->slots || s->n_slots < 1) return fail(DYN_ERR_SCHEDULE, "nano_rows or slots missing");
    if (s->n_streams < 1 || s->n_streams > DYN_MAX_STREAMS)
        return fail(DYN_ERR_SCHEDULE, "n_streams = %d outside 1..%d", s->n_streams, DYN_MAX_STREAMS);
    if (s->n_partitions < 0 || s->n_partitions > DYN_MAX_PARTITIONS)
        return fail(DYN_ERR_SCHEDULE, "n_partitions = %d outside 0..%d", s->n_partitions, DYN_MAX_PARTITIONS);
    if (s->n_partitions > 0 && (!s->cu_masks || s->cu_mask_words < 1 || s->cu_mask_words > 32))
        return fail(DYN_ERR_SCHEDULE, "partitions need cu_masks with 1..32 words each");
    for (int p = 0; p < s->n_partitions; ++p) {
        uint32_t any = 0;
        for (int i = 0; i < s->cu_mask_words; ++i) any |= s->cu_masks[p * s->cu_mask_words + i];
        if (!any) return fail(DYN_ERR_SCHEDULE, "CU mask of partition %d is empty", p + 1);
    }
    return DYN_OK;
}

// Checks batch shapes and the schedule, and expands it into the per-forward dispatch list
// with producer edges.
dyn_status build_plan(const dyn_layer *L, const dyn_batch *b, const dyn_schedule *s, std::vector<Dispatch> &plan) {
    if (!L || !b || !s) return fail(DYN_ERR_INVALID_ARG, "NULL layer, batch or schedule");
    if (b->n_tokens < 0 || b->n_seqs < 0) return fail(DYN_ERR_INVALID_ARG, "negative n_tokens or n_seqs");
    if (b->n_tokens > 0 && b->n_seqs == 0) return fail(DYN_ERR_INVALID_ARG, "tokens without sequences");
    if (!b->q_start_host) return fail(DYN_ERR_INVALID_ARG, "q_start_host is NULL");
    if (b->q_start_host[0] != 0 || b->q_start_host[b->n_seqs] != b->n_tokens)
        return fail(DYN_ERR_INVALID_ARG, "q_start_host must run from 0 to n_tokens");
    for (int i = 0; i < b->n_seqs; ++i)
        if (b->q_start_host[i + 1] <= b->q_start_host[i])
            return fail(DYN_ERR_INVALID_ARG, "sequence %d has no token in this step", i);
    if (b->max_pages_per_seq < 1 && b->n_tokens > 0) return fail(DYN_ERR_INVALID_ARG, "max_pages_per_seq < 1");

    const bool moe = L->cfg.n_experts > 0;
    const int *chain = moe ? kMoeChain : kDenseChain;
    const int n_chain = moe ? 10 : 9;
    const int T = b->n_tokens;

    std::vector<dyn_slot> seq_slots;
    int32_t seq_rows[2] = {0, T};
    int k = 1, n_slots = 0;
    const int32_t *rows = seq_rows;
    const dyn_slot *slots = nullptr;
    if (s->mode == DYN_SCHED_SEQUENTIAL) {
        for (int i = 0; i < n_chain; ++i) seq_slots.push_back(dyn_slot{(uint8_t)chain[i], 0, 1, 0, 0});
        slots = seq_slots.data();
        n_slots = n_chain;
    } else if (s->mode == DYN_SCHED_EXPLICIT) {
        dyn_status rc = check_schedule_fields(s);
        if (rc != DYN_OK) return rc;
        k = s->k;
        rows = s->nano_rows;
        if (rows[0] != 0 || rows[k] != T) return fail(DYN_ERR_SCHEDULE, "nano_rows must run from 0 to n_tokens");
        for (int i = 0; i < k; ++i) {
            if (rows[i + 1] < rows[i]) return fail(DYN_ERR_SCHEDULE, "nano_rows decreases at %d", i);
            if (!std::binary_search(b->q_start_host, b->q_start_host + b->n_seqs + 1, rows[i]))
                return fail(DYN_ERR_SCHEDULE, "cut point %d (row %d) is inside a sequence", i, rows[i]);
        }
        slots = s->slots;
        n_slots = s->n_slots;
    } else {
        return fail(DYN_ERR_SCHEDULE, "unknown schedule mode %d", s->mode);
    }

    // cover[op][nano] = slot index that dispatches it
    int cover[DYN_N_OPS][DYN_MAX_NANO];
    for (auto &r : cover) std::fill(r, r + DYN_MAX_NANO, -1);
    int chain_pos[DYN_N_OPS];
    std::fill(chain_pos, chain_pos + DYN_N_OPS, -1);
    for (int i = 0; i < n_chain; ++i) chain_pos[chain[i]] = i;
    for (int i = 0; i < n_slots; ++i) {
        const dyn_slot &sl = slots[i];
        if (sl.op >= DYN_N_OPS || chain_pos[sl.op] < 0)
            return fail(DYN_ERR_SCHEDULE, "slot %d: operator %d is not part of this layer", i, sl.op);
        if (sl.n_nano < 1 || sl.nano + sl.n_nano > k)
            return fail(DYN_ERR_SCHEDULE, "slot %d: micro-batches %d..%d outside 0..%d", i, sl.nano,
                        sl.nano + sl.n_nano - 1, k - 1);
        if (s->mode == DYN_SCHED_EXPLICIT) {
            if (sl.stream >= s->n_streams) return fail(DYN_ERR_SCHEDULE, "slot %d: stream %d out of range", i, sl.stream);
            if (sl.partition > s->n_partitions)
                return fail(DYN_ERR_SCHEDULE, "slot %d: partition %d out of range", i, sl.partition);
        }
        for (int nb = sl.nano; nb < sl.nano + sl.n_nano; ++nb) {
            if (cover[sl.op][nb] >= 0)
                return fail(DYN_ERR_SCHEDULE, "slot %d: %s of micro-batch %d dispatched twice", i, op_name(sl.op), nb);
            const int pos = chain_pos[sl.op];
            if (pos > 0 && cover[chain[pos - 1]][nb] < 0)
                return fail(DYN_ERR_SCHEDULE, "slot %d: %s of micro-batch %d issued before its producer %s", i,
                            op_name(sl.op), nb, op_name(chain[pos - 1]));
            cover[sl.op][nb] = i;
        }
    }
    for (int i = 0; i < n_chain; ++i)
        for (int nb = 0; nb < k; ++nb)
            if (cover[chain[i]][nb] < 0)
                return fail(DYN_ERR_SCHEDULE, "%s of micro-batch %d is never dispatched", op_name(chain[i]), nb);

    plan.clear();
    plan.reserve((size_t)L->cfg.n_layers * n_slots);
    for (int l = 0; l < L->cfg.n_layers; ++l)
        for (int i = 0; i < n_slots; ++i) {
            const dyn_slot &sl = slots[i];
            Dispatch d{l, sl.op, sl.nano, sl.n_nano, rows[sl.nano], rows[sl.nano + sl.n_nano], sl.stream, sl.partition, false, false, {}};
            // Operators that launch nothing of their own: the SiLU gate where the gate/up projection's epilogue
            // applies it; rotary + cache append, which the qkv projection's dispatch applies to the rows it
            // wrote; the second norm, applied by the o projection's dispatch; and from the second layer on
            // the first norm, applied by the previous layer's down projection (fused_into_producer).
            d.noop = d.r1 <= d.r0 || (sl.op == DYN_OP_SILU && dyn::gemm_gated_supported(L->cfg.dtype, 2 * L->cfg.mlp_inter, L->cfg.hidden)) ||
                     fused_into_producer(sl.op, l);
            {   // sequences inside [r0, r1): cut points are sequence boundaries
                const int32_t *q = b->q_start_host;
                const int s0 = (int)(std::lower_bound(q, q + b->n_seqs + 1, d.r0) - q);
                const int s1 = (int)(std::lower_bound(q, q + b->n_seqs + 1, d.r1) - q);
                d.any_multi = d.r1 - d.r0 > s1 - s0;
            }
            const int pos = chain_pos[sl.op];
            for (int nb = sl.nano; nb < sl.nano + sl.n_nano; ++nb) {
                int dep = -1;
                if (pos > 0) dep = l * n_slots + cover[chain[pos - 1]][nb];
                else if (l > 0) dep = (l - 1) * n_slots + cover[chain[n_chain - 1]][nb];
                if (dep >= 0 && std::find(d.deps.begin(), d.deps.end(), dep) == d.deps.end()) d.deps.push_back(dep);
            }
            plan.push_back(std::move(d));
        }
    // The expert lists of a dispatch depend on its rows' routing only: a down projection over
    // exactly the rows of one gate/up dispatch (which it follows in its micro-batches' chain)
    // reads that dispatch's lists instead of building its own.
    if (L->cfg.n_experts)
        for (size_t i = 0; i < plan.size(); ++i) {
            Dispatch &d = plan[i];
            if (d.op != DYN_OP_DOWN || d.noop) continue;
            const int first = d.layer * n_slots;
            for (int j = first; j < first + n_slots; ++j)
                if (plan[j].op == DYN_OP_GATE_UP && !plan[j].noop && plan[j].r0 == d.r0 && plan[j].r1 == d.r1) d.lists_ready = true;
        }
    return DYN_OK;
}

// Issue order is a timeline only within a stream: what is issued on another stream after
// dispatch i may run beside it.  So whatever dispatch i is the last to touch stays alive until
// the next dispatch on i's own stream is issued (that one cannot start before i ends):
// until[i] = index of the last dispatch issued before that one.
std::vector<int> alive_until(const std::vector<Dispatch> &plan) {
    std::vector<int> until(plan.size());
    int next_on[(DYN_MAX_PARTITIONS + 1) * DYN_MAX_STREAMS];
    std::fill(next_on, next_on + (DYN_MAX_PARTITIONS + 1) * DYN_MAX_STREAMS, (int)plan.size());
    for (int i = (int)plan.size() - 1; i >= 0; --i) {
        until[i] = next_on[plan[i].key()] - 1;
        next_on[plan[i].key()] = i;
    }
    return until;
}

// The workspace layout of one plan (Section 3.3.1, Algorithm 1: the backend knows every
// intermediate's producers and consumers, so it knows when its memory is free again).  Two
// regions may share bytes only if everything that touches one has finished before anything
// touches the other, and what orders dispatches on the device is stream order and events, not
// the order of issue.  Two cases are safe by construction and are the ones used:
//   * All dispatches on one stream (the sequential order, or micro-batches issued on a single
//     stream): issue order is execution order.  Every region gets the set of issue slots during
//     which it is alive - a tensor from its first producer to its last consumer over all
//     micro-batches, a dispatch's scratch while the dispatch runs - folded over the layers, which
//     all issue the same slots, and regions alive at disjoint times share bytes.
//   * Several streams: micro-batches advance independently, so no tensor is ever known to be
//     dead while another micro-batch may still be anywhere in the chain: tensors keep regions
//     of their own.  The scratch of two dispatches on the SAME stream still never exists at the
//     same time, so each stream's dispatches share one scratch arena; different streams' do not.
// Regions are placed largest first at the lowest offset where they overlap no region they
// conflict with.  The more runs side by side, the less can be shared: the peak-memory cost of
// overlapping that Section 2.1 names.
WsLayout plan_layout(const dyn_layer *L, const dyn_batch *b, const std::vector<Dispatch> &plan, std::vector<Region> *regions_out) {
    const dyn_layer_config &c = L->cfg;
    const Sizes z = tensor_sizes(L, b->n_tokens, b->max_pages_per_seq);
    WsLayout w{};
    w.ld_h = z.ld_h; w.ld_attn = z.ld_attn; w.ld_act = z.ld_act; w.max_chunks = z.max_chunks;
    const int P = (int)plan.size(), n_slots = P / std::max(c.n_layers, 1);
    w.slot.assign((size_t)std::max(n_slots, 0), SlotScratch{});
    if (P == 0 || n_slots == 0) return w;
    const std::vector<int> until = alive_until(plan);
    const bool moe = c.n_experts > 0, gated = dyn::gemm_gated_supported(c.dtype, 2 * c.mlp_inter, c.hidden);

    bool single_stream = true;
    {
        int key = -1;
        for (const Dispatch &d : plan) {
            if (d.noop) continue;
            if (key < 0) key = d.key();
            single_stream = single_stream && d.key() == key;
        }
    }
    std::vector<Region> regions;
    auto add = [&](int kind, int slot, size_t bytes, bool always) {
        always = always || (!single_stream && slot < 0);            // several streams: tensors are never known dead
        regions.push_back(Region{kind, slot, bytes, 0, std::vector<char>((size_t)n_slots, always ? 1 : 0), always,
                                 slot >= 0 ? plan[slot].key() : -1});
        return (int)regions.size() - 1;
    };
    auto mark = [&](int region, int from, int to) {           // alive over dispatches from..to (global issue indices)
        Region &r = regions[region];
        if (to - from + 1 >= n_slots) { std::fill(r.live.begin(), r.live.end(), 1); return; }
        for (int t = from; t <= to; ++t) r.live[t % n_slots] = 1;
    };
    // slot that dispatches (operator, micro-batch); the same in every layer
    int slot_of[DYN_N_OPS][DYN_MAX_NANO];
    for (auto &r : slot_of) std::fill(r, r + DYN_MAX_NANO, -1);
    int k = 0;
    for (int j = 0; j < n_slots; ++j)
        for (int nb = plan[j].nano; nb < plan[j].nano + plan[j].n_nano; ++nb) { slot_of[plan[j].op][nb] = j; k = std::max(k, nb + 1); }

    // h holds three generations per layer: the first norm's output (written by the first layer's
    // own norm, from then on by the previous layer's down projection), read by qkv; and the second
    // norm's, written by the o projection's dispatch, read by the router and gate/up
    struct TensorDef { int kind; size_t bytes; int producer, last_consumer; bool present; int producer_layer_offset; };
    const TensorDef defs[] = {
        {DYN_REGION_H, z.h, DYN_OP_NORM1, DYN_OP_QKV, true, 0},
        {DYN_REGION_H, z.h, DYN_OP_DOWN, DYN_OP_QKV, c.n_layers > 1, -1},
        {DYN_REGION_H, z.h, DYN_OP_OPROJ, DYN_OP_GATE_UP, true, 0},
        {DYN_REGION_QKV, z.qkv, DYN_OP_QKV, DYN_OP_ATTN, true, 0},
        {DYN_REGION_ATTN, z.attn, DYN_OP_ATTN, DYN_OP_OPROJ, true, 0},
        {DYN_REGION_X2, z.x2, DYN_OP_OPROJ, DYN_OP_DOWN, true, 0},
        {DYN_REGION_GU, z.gu, DYN_OP_GATE_UP, DYN_OP_SILU, !gated, 0},
        {DYN_REGION_ACT, z.act, gated ? DYN_OP_GATE_UP : DYN_OP_SILU, DYN_OP_DOWN, true, 0},
        {DYN_REGION_ROUTING, align_up(z.sel) + z.wgt, DYN_OP_ROUTE, DYN_OP_DOWN, moe, 0},
    };
    int region_of_kind[DYN_REGION_KINDS];
    std::fill(region_of_kind, region_of_kind + DYN_REGION_KINDS, -1);
    for (const TensorDef &d : defs) {
        if (!d.present || !d.bytes) continue;
        int r = region_of_kind[d.kind];
        if (r < 0) r = region_of_kind[d.kind] = add(d.kind, -1, d.bytes, false);
        for (int l = 0; l < c.n_layers; ++l) {
            const int pl = l + d.producer_layer_offset;           // layer of the producing dispatch
            if (pl < 0) continue;
            int from = P, to = -1;
            for (int nb = 0; nb < k; ++nb) {
                from = std::min(from, pl * n_slots + slot_of[d.producer][nb]);
                to = std::max(to, until[l * n_slots + slot_of[d.last_consumer][nb]]);
            }
            mark(r, from, to);
        }
    }
    // layer outputs that feed the next layer alternate between two buffers; the work lists are built
    // by the first layer and walked by all: alive throughout
    const int r_xa = z.xa ? add(DYN_REGION_XA, -1, z.xa, true) : -1;
    const int r_xb = z.xb ? add(DYN_REGION_XB, -1, z.xb, true) : -1;
    const int r_plan = z.plan ? add(DYN_REGION_PLAN, -1, z.plan, true) : -1;
    // scratch per slot
    struct SlotRegions { int planes = -1, part_o = -1, part_ml = -1, lists = -1, moe_planes = -1; };
    std::vector<SlotRegions> sr((size_t)n_slots);
    for (int j = 0; j < n_slots; ++j) {
        const Dispatch &d = plan[j];
        if (d.noop) continue;
        const ScratchBytes kb = dispatch_scratch(L, z, d.op, d.r1 - d.r0);
        if (kb.planes) sr[j].planes = add(DYN_REGION_PLANES, j, kb.planes, false);
        if (kb.part_o) sr[j].part_o = add(DYN_REGION_PART_O, j, kb.part_o, false);
        if (kb.part_ml) sr[j].part_ml = add(DYN_REGION_PART_ML, j, kb.part_ml, false);
        if (kb.lists && !(d.op == DYN_OP_DOWN && d.lists_ready)) sr[j].lists = add(DYN_REGION_LISTS, j, kb.lists, false);
        if (kb.moe_planes) sr[j].moe_planes = add(DYN_REGION_MOE_PLANES, j, kb.moe_planes, false);
        for (int l = 0; l < c.n_layers; ++l) {
            const int i = l * n_slots + j;
            for (int r : {sr[j].planes, sr[j].part_o, sr[j].part_ml, sr[j].lists, sr[j].moe_planes})
                if (r >= 0) mark(r, i, single_stream ? until[i] : i);
        }
    }
    // a down projection that reads the expert lists of the gate/up dispatch over the same rows keeps them alive
    std::vector<int> lists_from((size_t)n_slots, -1);
    for (int j = 0; j < n_slots; ++j) {
        const Dispatch &d = plan[j];
        if (d.op != DYN_OP_DOWN || !d.lists_ready || d.noop) continue;
        for (int g = 0; g < n_slots; ++g)
            if (plan[g].op == DYN_OP_GATE_UP && !plan[g].noop && plan[g].r0 == d.r0 && plan[g].r1 == d.r1) lists_from[j] = g;
        if (lists_from[j] >= 0 && sr[lists_from[j]].lists >= 0) {
            Region &lr = regions[sr[lists_from[j]].lists];
            if (single_stream) {
                for (int l = 0; l < c.n_layers; ++l) mark(sr[lists_from[j]].lists, l * n_slots + lists_from[j], until[l * n_slots + j]);
            } else {                       // read later by a dispatch that may run on another stream: kept throughout
                lr.always = true;
                std::fill(lr.live.begin(), lr.live.end(), 1);
            }
        }
    }

    // placement: largest first, lowest offset that overlaps no placed region alive at the same time
    std::vector<int> order(regions.size());
    for (size_t i = 0; i < order.size(); ++i) order[i] = (int)i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int bb) { return regions[a].bytes > regions[bb].bytes; });
    std::vector<int> placed;
    size_t total = 0;
    for (int ri : order) {
        Region &r = regions[ri];
        std::vector<std::pair<size_t, size_t>> busy;            // [offset, end) of placed regions that conflict
        for (int pi : placed) {
            const Region &q = regions[pi];
            // scratch of dispatches on different streams may exist at the same time whatever the issue order
            bool conflict = r.always || q.always || (!single_stream && r.stream_key != q.stream_key);
            for (int t = 0; t < n_slots && !conflict; ++t) conflict = r.live[t] && q.live[t];
            if (conflict) busy.push_back({q.offset, q.offset + align_up(q.bytes)});
        }
        std::sort(busy.begin(), busy.end());
        size_t off = 0;
        for (const auto &iv : busy)
            if (iv.first < off + align_up(r.bytes) && iv.second > off) off = iv.second;     // overlaps the candidate: move past it
        r.offset = off;
        total = std::max(total, off + align_up(r.bytes));
        placed.push_back(ri);
    }
    w.total = total;
    auto off_of = [&](int region) { return region >= 0 ? regions[region].offset : (size_t)0; };
    w.h = off_of(region_of_kind[DYN_REGION_H]);
    w.qkv = off_of(region_of_kind[DYN_REGION_QKV]);
    w.attn = off_of(region_of_kind[DYN_REGION_ATTN]);
    w.x2 = off_of(region_of_kind[DYN_REGION_X2]);
    w.gu = off_of(region_of_kind[DYN_REGION_GU]);
    w.act = off_of(region_of_kind[DYN_REGION_ACT]);
    w.sel = off_of(region_of_kind[DYN_REGION_ROUTING]);
    w.wgt = w.sel + align_up(z.sel);
    w.xa = off_of(r_xa);
    w.xb = off_of(r_xb);
    w.plan = off_of(r_plan);
    for (int j = 0; j < n_slots; ++j) {
        const int lists_region = lists_from[j] >= 0 ? sr[lists_from[j]].lists : sr[j].lists;
        w.slot[j] = SlotScratch{off_of(sr[j].planes), off_of(sr[j].part_o), off_of(sr[j].part_ml), off_of(lists_region), off_of(sr[j].moe_planes)};
    }
    if (regions_out) *regions_out = std::move(regions);
    return w;
}

void destroy_graph_entry(GraphEntry &g) {
    (void)hipGraphExecDestroy(g.exec);
    (void)hipGraphDestroy(g.graph);
    (void)hipEventDestroy(g.last_launch);
}

// CU-masked streams are hardware queues whose mask is set through the driver.  They are made
// once per distinct mask and stream id for the whole process, on an idle device, shared by
// every layer handle and never destroyed: creating or destroying such a queue while other
// queues are live has hung the runtime here (once mid-forward, twice in dyn_layer_destroy).
struct MaskedStream {
    int stream_id;
    std::vector<uint32_t> mask;
    hipStream_t stream;
};
std::vector<MaskedStream> g_masked_streams;
std::mutex g_masked_mutex;

dyn_status ensure_stream(dyn_layer *L, const dyn_schedule *s, int key, hipStream_t *out) {
    const int partition = key / DYN_MAX_STREAMS;
    if (partition > 0) {
        std::vector<uint32_t> mask(s->cu_masks + (size_t)(partition - 1) * s->cu_mask_words,
                                   s->cu_masks + (size_t)partition * s->cu_mask_words);
        while (!mask.empty() && mask.back() == 0) mask.pop_back();      // trailing zero words name no CU
        if (!L->streams[key] || L->stream_mask[key] != mask) {
            std::lock_guard<std::mutex> lock(g_masked_mutex);
            hipStream_t found = nullptr;
            for (const MaskedStream &m : g_masked_streams)
                if (m.stream_id == key % DYN_MAX_STREAMS && m.mask == mask) found = m.stream;
            if (!found) {
                HIP_TRY(hipDeviceSynchronize());
                HIP_TRY(hipExtStreamCreateWithCUMask(&found, (uint32_t)mask.size(), mask.data()));
                g_masked_streams.push_back(MaskedStream{key % DYN_MAX_STREAMS, mask, found});
            }
            L->streams[key] = found;
            L->stream_mask[key] = mask;
        }
    } else if (!L->streams[key]) {
        HIP_TRY(hipStreamCreateWithFlags(&L->streams[key], hipStreamNonBlocking));
    }
    *out = L->streams[key];
    return DYN_OK;
}

dyn_status launch_op(const dyn_layer *L, const dyn_batch *b, const dyn_schedule *s, const WsLayout &ws, const Dispatch &d,
                     const SlotScratch &sc, hipStream_t st, hipEvent_t mid, hipEvent_t pre) {
    const dyn_layer_config &c = L->cfg;
    const dyn_layer_weights &w = L->w[d.layer];
    const size_t e = esize(c);
    const int rows = d.r1 - d.r0;
    if (rows <= 0) return DYN_OK;
    char *base = (char *)b->workspace;
    const int H = c.hidden, NQ = c.n_q_heads * c.head_dim, NQKV = qkv_width(c), I = c.mlp_inter;
    const int nl = c.n_layers;
    const char *x_in = d.layer == 0 ? (const char *)b->x : (d.layer % 2 ? base + ws.xa : base + ws.xb);
    char *x_out = d.layer == nl - 1 ? (char *)b->y : (d.layer % 2 ? base + ws.xb : base + ws.xa);
    auto rowp = [&](const char *p, int width) { return p + (size_t)d.r0 * width * e; };
    dyn::AttnShape sh{c.n_q_heads, c.n_kv_heads, c.head_dim, c.page_size, b->max_pages_per_seq, L->chunk_pages, ws.max_chunks, 0};
    if (d.partition > 0 && s->mode == DYN_SCHED_EXPLICIT)
        for (int i = 0; i < s->cu_mask_words; ++i)
            sh.n_cus += __builtin_popcount(s->cu_masks[(d.partition - 1) * s->cu_mask_words + i]);
    char *kc = b->k_cache_layers ? (char *)b->k_cache_layers[d.layer] : (char *)b->k_cache + (size_t)d.layer * b->kv_layer_stride;
    char *vc = b->v_cache_layers ? (char *)b->v_cache_layers[d.layer] : (char *)b->v_cache + (size_t)d.layer * b->kv_layer_stride;
    // the dispatch's own scratch: split-K planes of `rows` rows each
    float *const planes = (float *)(base + sc.planes);
    hipError_t err = hipSuccess;
    switch (d.op) {
        case DYN_OP_NORM1:
            if (fused_into_producer(d.op, d.layer)) break;       // the previous layer's down projection wrote h
            err = dyn::launch_rmsnorm(c.dtype, rowp(x_in, H), w.g_norm1, (void *)rowp(base + ws.h, ws.ld_h), ws.ld_h, rows, H, c.rms_eps, st);
            break;
        case DYN_OP_QKV: {
            dyn::GemmEpilogue ep;                                 // rotary + cache append on the rows just projected
            ep.kind = dyn::GemmEpilogue::ROPE;
            ep.seq_of_token = b->seq_of_token + d.r0;
            ep.pos_of_token = b->pos_of_token + d.r0;
            ep.block_table = b->block_table;
            ep.k_cache = kc;
            ep.v_cache = vc;
            ep.rope = &L->rope;
            ep.shape = &sh;
            err = dyn::launch_gemm(c.dtype, rowp(base + ws.h, ws.ld_h), ws.ld_h, w.w_qkv, nullptr, (void *)rowp(base + ws.qkv, NQKV),
                                   planes, (size_t)rows * NQKV, rows, NQKV, H, st, mid, &ep);
            break;
        }
        case DYN_OP_ROPE_KV:
            break;                                                // applied by the qkv projection's dispatch
        case DYN_OP_ATTN:
            err = dyn::launch_attention(c.dtype, rowp(base + ws.qkv, NQKV), b->seq_of_token + d.r0, b->pos_of_token + d.r0,
                                        b->block_table, kc, vc, (void *)rowp(base + ws.attn, ws.ld_attn), ws.ld_attn,
                                        (float *)(base + sc.part_o), (float *)(base + sc.part_ml),
                                        (int32_t *)(base + ws.plan) + (size_t)d.r0 * (ws.max_chunks + 2) * 4, d.any_multi, sh, rows, st, mid, pre,
                                        d.layer > 0);   // every layer dispatches the same row ranges: layer 0 built the work lists
            break;
        case DYN_OP_OPROJ: {
            dyn::GemmEpilogue ep;                                 // the second norm of the rows just written
            ep.kind = dyn::GemmEpilogue::NORM;
            ep.g = w.g_norm2;
            ep.h_out = (void *)rowp(base + ws.h, ws.ld_h);
            ep.ld_h = ws.ld_h;
            ep.eps = c.rms_eps;
            err = dyn::launch_gemm(c.dtype, rowp(base + ws.attn, ws.ld_attn), ws.ld_attn, w.w_o, rowp(x_in, H), (void *)rowp(base + ws.x2, H),
                                   planes, (size_t)rows * H, rows, H, NQ, st, mid, &ep);
            break;
        }
        case DYN_OP_NORM2:
            break;                                                // applied by the o projection's dispatch
        case DYN_OP_ROUTE:
            err = dyn::launch_route(c.dtype, rowp(base + ws.h, ws.ld_h), ws.ld_h, w.w_router,
                                    (int32_t *)(base + ws.sel) + (size_t)d.r0 * c.top_k,
                                    (float *)(base + ws.wgt) + (size_t)d.r0 * c.top_k, rows, H, c.n_experts, c.top_k, st);
            break;
        case DYN_OP_GATE_UP:
            if (c.n_experts) {
                // rows of the grouped projections are (token, rank) pairs p = t * top_k + rank
                const int n_pairs = rows * c.top_k, pair0 = d.r0 * c.top_k;
                int32_t *counts = (int32_t *)(base + sc.lists);
                int32_t *lists = counts + c.n_experts;
                err = dyn::launch_expert_lists((const int32_t *)(base + ws.sel), n_pairs, pair0, c.n_experts, n_pairs, counts, lists, st);
                if (err != hipSuccess) break;
                dyn::GemmGroups gr{counts, lists, n_pairs, c.top_k, c.n_experts, (size_t)2 * I * H, 0};
                if (dyn::gemm_gated_supported(c.dtype, 2 * I, H)) {   // SiLU gate in the epilogue: DYN_OP_SILU has nothing left to do
                    err = dyn::launch_gemm_gated(base + ws.h, ws.ld_h, w.w_gate_up, base + ws.act, ws.ld_act, gr, rows, 2 * I, H, st, mid);
                    break;
                }
                // the grouped kernels index planes by pair id: the dispatch's planes start at its first pair
                err = dyn::launch_gemm_grouped(c.dtype, base + ws.h, ws.ld_h, w.w_gate_up, base + ws.gu,
                                               planes - (size_t)pair0 * 2 * I, (size_t)n_pairs * 2 * I, gr, rows, pair0,
                                               n_pairs, 2 * I, H, st, mid);
                break;
            }
            if (dyn::gemm_gated_supported(c.dtype, 2 * I, H)) {       // SiLU gate in the epilogue: DYN_OP_SILU has nothing left to do
                err = dyn::launch_gemm_gated(rowp(base + ws.h, ws.ld_h), ws.ld_h, w.w_gate_up, (void *)rowp(base + ws.act, ws.ld_act),
                                             ws.ld_act, dyn::GemmGroups{}, rows, 2 * I, H, st, mid);
                break;
            }
            err = dyn::launch_gemm(c.dtype, rowp(base + ws.h, ws.ld_h), ws.ld_h, w.w_gate_up, nullptr, (void *)rowp(base + ws.gu, 2 * I),
                                   planes, (size_t)rows * 2 * I, rows, 2 * I, H, st, mid);
            break;
        case DYN_OP_SILU:
            if (dyn::gemm_gated_supported(c.dtype, 2 * I, H)) break;   // done in the gate/up projection's epilogue
            if (c.n_experts) {
                const size_t pair0 = (size_t)d.r0 * c.top_k;
                err = dyn::launch_silu_mul(c.dtype, base + ws.gu + pair0 * 2 * I * e, base + ws.act + pair0 * ws.ld_act * e,
                                           ws.ld_act, rows * c.top_k, I, st);
                break;
            }
            err = dyn::launch_silu_mul(c.dtype, rowp(base + ws.gu, 2 * I), (void *)rowp(base + ws.act, ws.ld_act), ws.ld_act, rows, I, st);
            break;
        case DYN_OP_DOWN: {
            if (c.n_experts) {
                const int n_pairs = rows * c.top_k, pair0 = d.r0 * c.top_k;
                int32_t *counts = (int32_t *)(base + sc.lists);     // its own, or the matching gate/up dispatch's (lists_ready)
                int32_t *lists = counts + c.n_experts;
                if (!d.lists_ready) err = dyn::launch_expert_lists((const int32_t *)(base + ws.sel), n_pairs, pair0, c.n_experts, n_pairs, counts, lists, st);
                if (err != hipSuccess) break;
                const int Sd = dyn::gemm_split_k(c.dtype, H, I, c.n_experts);
                const size_t plane = (size_t)n_pairs * H;
                float *const mp = (float *)(base + sc.moe_planes);
                dyn::GemmGroups gr{counts, lists, n_pairs, 1, c.n_experts, (size_t)H * I, 1};
                err = dyn::launch_gemm_grouped(c.dtype, base + ws.act, ws.ld_act, w.w_down, nullptr,
                                               mp - (size_t)pair0 * H, plane, gr, rows, pair0, n_pairs, H, I, st, mid);
                if (err != hipSuccess) break;
                err = dyn::launch_moe_combine(c.dtype, mp, plane, Sd,
                                              (const float *)(base + ws.wgt) + pair0, rowp(base + ws.x2, H), (void *)rowp(x_out, H),
                                              rows, H, c.top_k, st);
                if (err == hipSuccess && d.layer + 1 < nl)        // the next layer's first norm of the rows just written
                    err = dyn::launch_rmsnorm(c.dtype, rowp(x_out, H), L->w[d.layer + 1].g_norm1, (void *)rowp(base + ws.h, ws.ld_h), ws.ld_h,
                                              rows, H, c.rms_eps, st);
                break;
            }
            dyn::GemmEpilogue ep;                                 // the next layer's first norm of the rows just written
            if (d.layer + 1 < nl) {
                ep.kind = dyn::GemmEpilogue::NORM;
                ep.g = L->w[d.layer + 1].g_norm1;
                ep.h_out = (void *)rowp(base + ws.h, ws.ld_h);
                ep.ld_h = ws.ld_h;
                ep.eps = c.rms_eps;
            }
            err = dyn::launch_gemm(c.dtype, rowp(base + ws.act, ws.ld_act), ws.ld_act, w.w_down, rowp(base + ws.x2, H), (void *)rowp(x_out, H),
                                   planes, (size_t)rows * H, rows, H, I, st, mid, &ep);
            break;
        }
        default:
            return fail(DYN_ERR_UNSUPPORTED, "operator %s has no kernel", op_name(d.op));
    }
    if (err != hipSuccess) return fail(DYN_ERR_HIP, "launch of %s failed: %s", op_name(d.op), hipGetErrorString(err));
    return DYN_OK;
}

// Issues the plan: fork side streams from origin, wait on producers that ran on another
// stream, record an event after every dispatch, join everything back into origin.
dyn_status run_plan(dyn_layer *L, const dyn_batch *b, const dyn_schedule *s, const WsLayout &ws,
                    const std::vector<Dispatch> &plan, hipStream_t origin, bool profile) {
    while (L->events.size() < plan.size()) {
        hipEvent_t ev;
        HIP_TRY(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
        L->events.push_back(ev);
    }
    if (!L->fork_event) HIP_TRY(hipEventCreateWithFlags(&L->fork_event, hipEventDisableTiming));
    if (profile) {
        while (L->prof_events.size() < 1 + 4 * plan.size()) {
            hipEvent_t ev;
            HIP_TRY(hipEventCreate(&ev));
            L->prof_events.push_back(ev);
        }
        HIP_TRY(hipEventRecord(L->prof_events[0], origin));
    }
    HIP_TRY(hipEventRecord(L->fork_event, origin));
    bool used[(DYN_MAX_PARTITIONS + 1) * DYN_MAX_STREAMS] = {};
    int last_on[(DYN_MAX_PARTITIONS + 1) * DYN_MAX_STREAMS];
    std::fill(last_on, last_on + (DYN_MAX_PARTITIONS + 1) * DYN_MAX_STREAMS, -1);
    std::vector<hipStream_t> st_of(plan.size());
    // Dispatches that launch nothing take no part in the stream choreography: whoever depends
    // on one depends on what it depended on.  Waiting and recording around them would give a
    // captured graph forked branches without a node and the same edge several times.
    // (Profiling, eager only, keeps them so that every dispatch has its time marks.)
    std::vector<std::vector<int>> real_deps(plan.size());
    for (size_t i = 0; i < plan.size(); ++i) {
        const Dispatch &d = plan[i];
        for (int dep : d.deps) {
            const bool elided = plan[dep].noop && !profile;
            for (int r : elided ? real_deps[dep] : std::vector<int>{dep})
                if (std::find(real_deps[i].begin(), real_deps[i].end(), r) == real_deps[i].end()) real_deps[i].push_back(r);
        }
        if (d.noop && !profile) continue;
        const int key = d.key();
        hipStream_t st = origin;
        if (key != 0) {
            dyn_status rc = ensure_stream(L, s, key, &st);
            if (rc != DYN_OK) return rc;
            if (!used[key]) HIP_TRY(hipStreamWaitEvent(st, L->fork_event, 0));
        }
        used[key] = true;
        st_of[i] = st;
        // one wait per producer stream: a stream's events complete in order, the latest covers the rest
        for (int dep : real_deps[i]) {
            if (st_of[dep] == st) continue;
            bool latest = true;
            for (int other : real_deps[i]) latest = latest && !(st_of[other] == st_of[dep] && other > dep);
            if (latest) HIP_TRY(hipStreamWaitEvent(st, L->events[dep], 0));
        }
        if (profile) {
            // the two middle events stay here unless the operator records them around its main kernel
            for (int j = 1; j <= 3; ++j) HIP_TRY(hipEventRecord(L->prof_events[j + 4 * i], st));
        }
        const bool mark = profile && d.r1 > d.r0;
        dyn_status rc = launch_op(L, b, s, ws, d, ws.slot[i % ws.slot.size()], st, mark ? L->prof_events[3 + 4 * i] : nullptr,
                                  mark ? L->prof_events[2 + 4 * i] : nullptr);
        if (rc != DYN_OK) return rc;
        if (profile) HIP_TRY(hipEventRecord(L->prof_events[4 + 4 * i], st));
        HIP_TRY(hipEventRecord(L->events[i], st));
        last_on[key] = (int)i;
    }
    for (int key = 1; key < (DYN_MAX_PARTITIONS + 1) * DYN_MAX_STREAMS; ++key)
        if (last_on[key] >= 0) HIP_TRY(hipStreamWaitEvent(origin, L->events[last_on[key]], 0));
    return DYN_OK;
}

// Everything a captured forward's launches are derived from on the host: the batch's pointers
// and sizes, the sequence structure (q_start_host decides which attention kernels a dispatch
// launches), every dispatch with the flags that change what it launches, and the CU masks.
// Cached graphs are matched on the whole record, not on a hash of it.  What the kernels read
// from device memory (positions, block table, activations) may change between replays.
std::vector<unsigned char> graph_key(const dyn_batch *b, const dyn_schedule *s, const std::vector<Dispatch> &plan) {
    std::vector<unsigned char> key;
    auto put = [&](const void *p, size_t n) {
        const unsigned char *c = (const unsigned char *)p;
        key.insert(key.end(), c, c + n);
    };
    const void *ptrs[] = {b->x, b->y, b->seq_of_token, b->pos_of_token, b->block_table, b->k_cache, b->v_cache, b->workspace};
    put(ptrs, sizeof ptrs);
    const int64_t dims[] = {b->n_tokens, b->n_seqs, b->max_pages_per_seq, (int64_t)b->kv_layer_stride,
                            (int64_t)b->workspace_bytes, (int64_t)plan.size()};
    put(dims, sizeof dims);
    put(b->q_start_host, sizeof(int32_t) * ((size_t)b->n_seqs + 1));
    if (b->k_cache_layers) {               // caches placed layer by layer: the pointers are the launches' arguments
        const int n_layers = plan.empty() ? 0 : plan.back().layer + 1;
        put(b->k_cache_layers, sizeof(void *) * n_layers);
        put(b->v_cache_layers, sizeof(void *) * n_layers);
    }
    for (const Dispatch &d : plan) {
        const int f[] = {d.layer, d.op, d.r0, d.r1, d.stream, d.partition, d.any_multi, d.noop, d.lists_ready};
        put(f, sizeof f);
    }
    if (s->mode == DYN_SCHED_EXPLICIT && s->n_partitions > 0) {
        const int m[] = {s->n_partitions, s->cu_mask_words};
        put(m, sizeof m);
        put(s->cu_masks, sizeof(uint32_t) * s->n_partitions * s->cu_mask_words);
    }
    return key;
}

// Static data-flow analysis of one plan (Section 3.3.1, Algorithm 1): reference counts and
// lifetimes of the intermediate regions, peak of live bytes in issue order.
void analyse_memory(const dyn_layer *L, const dyn_batch *b, const std::vector<Dispatch> &plan, int k, const int32_t *rows,
                    dyn_memory_report *out, size_t *peak, int *peak_at) {
    const dyn_layer_config &c = L->cfg;
    const size_t e = esize(c);
    const Sizes ws = tensor_sizes(L, b->n_tokens, b->max_pages_per_seq);
    const int n_slots = (int)plan.size() / c.n_layers;
    const bool moe = c.n_experts > 0, gated = dyn::gemm_gated_supported(c.dtype, 2 * c.mlp_inter, c.hidden);
    const int pairs = moe ? c.top_k : 1, H = c.hidden, I = c.mlp_inter, NQKV = qkv_width(c), NQ = c.n_q_heads * c.head_dim;
    int slot_of[DYN_N_OPS][DYN_MAX_NANO];
    for (auto &r : slot_of) std::fill(r, r + DYN_MAX_NANO, -1);
    for (int i = 0; i < n_slots; ++i)
        for (int nb = plan[i].nano; nb < plan[i].nano + plan[i].n_nano; ++nb) slot_of[plan[i].op][nb] = i;
    // Who writes and who reads what (the projections' dispatches also run the operator that follows
    // them: qkv rotates and appends, o and down write the next norm's output).
    struct Tensor { int producer; int consumers[2]; size_t row_bytes; bool from_previous_layer; bool present; bool first_layer_only; };
    const Tensor tensors[] = {
        {DYN_OP_DOWN, {DYN_OP_OPROJ, -1}, H * e, true, true, false},                          // layer input (not the caller's x): the residual
        {DYN_OP_NORM1, {DYN_OP_QKV, -1}, ws.ld_h * e, false, true, true},                     // first norm, first layer
        {DYN_OP_DOWN, {DYN_OP_QKV, -1}, ws.ld_h * e, true, true, false},                      // first norm, later layers
        {DYN_OP_QKV, {DYN_OP_ATTN, -1}, NQKV * e, false, true, false},                        // q rotated by the projection's dispatch
        {DYN_OP_ATTN, {DYN_OP_OPROJ, -1}, ws.ld_attn * e, false, true, false},
        {DYN_OP_OPROJ, {DYN_OP_DOWN, -1}, H * e, false, true, false},                         // x2: the residual of the MLP
        {DYN_OP_OPROJ, {moe ? DYN_OP_ROUTE : DYN_OP_GATE_UP, moe ? DYN_OP_GATE_UP : -1}, ws.ld_h * e, false, true, false},   // second norm
        {DYN_OP_ROUTE, {DYN_OP_GATE_UP, DYN_OP_DOWN}, (size_t)c.top_k * 8, false, moe, false},   // selected experts and their weights
        {DYN_OP_GATE_UP, {DYN_OP_SILU, -1}, (size_t)pairs * 2 * I * e, false, !gated, false},
        {gated ? DYN_OP_GATE_UP : DYN_OP_SILU, {DYN_OP_DOWN, -1}, (size_t)pairs * ws.ld_act * e, false, true, false},
    };
    std::vector<size_t> born(plan.size(), 0), dies(plan.size(), 0), scratch(plan.size(), 0);
    const std::vector<int> until = alive_until(plan);      // stream-aware end of what a dispatch is the last to touch
    out->n_regions = out->max_ref_count = out->n_resharded = 0;
    for (int l = 0; l < c.n_layers; ++l)
        for (const Tensor &t : tensors) {
            if (!t.present || (t.from_previous_layer && l == 0) || (t.first_layer_only && l > 0)) continue;
            for (int nb = 0; nb < k; ++nb) {
                const size_t n_rows = (size_t)(rows[nb + 1] - rows[nb]);
                if (!n_rows) continue;
                const int prod = (t.from_previous_layer ? l - 1 : l) * n_slots + slot_of[t.producer][nb];
                int refs = 0, last = prod, seen[2] = {-1, -1};
                bool resharded = false;
                for (int j = 0; j < 2; ++j) {
                    if (t.consumers[j] < 0) continue;
                    const int cons = l * n_slots + slot_of[t.consumers[j]][nb];
                    if (cons != seen[0]) { seen[refs] = cons; ++refs; }
                    last = std::max(last, cons);
                    resharded = resharded || plan[cons].n_nano != plan[prod].n_nano;
                }
                born[prod] += n_rows * t.row_bytes;
                dies[until[last]] += n_rows * t.row_bytes;
                ++out->n_regions;
                out->max_ref_count = std::max(out->max_ref_count, refs);
                out->n_resharded += resharded;
            }
        }
    for (size_t i = 0; i < plan.size(); ++i) {          // scratch a dispatch holds while it runs
        const Dispatch &d = plan[i];
        const size_t r = (size_t)std::max(d.r1 - d.r0, 0);
        auto planes = [&](int N, int K) {
            return dyn::gemm_uses_plane_buffer(c.dtype, (int)r, N, K) ? (size_t)dyn::gemm_split_k(c.dtype, N, K) * r * N * sizeof(float) : 0;
        };
        const size_t lists = moe ? r * c.top_k * 2 * c.n_experts * sizeof(int32_t) : 0;
        switch (d.op) {
            case DYN_OP_QKV: scratch[i] = planes(NQKV, H); break;
            case DYN_OP_OPROJ: scratch[i] = planes(H, NQ); break;
            case DYN_OP_ATTN:
                scratch[i] = r * c.n_q_heads * ws.max_chunks * (c.head_dim + 2) * sizeof(float) + (r * ws.max_chunks + 2 * r) * 4 * sizeof(int32_t);
                break;
            case DYN_OP_GATE_UP:
                scratch[i] = moe ? lists + (gated ? 0 : (size_t)dyn::gemm_split_k(c.dtype, 2 * I, H, c.n_experts) > 1
                                                            ? (size_t)dyn::gemm_split_k(c.dtype, 2 * I, H, c.n_experts) * r * pairs * 2 * I * sizeof(float) : 0)
                                 : (gated ? 0 : planes(2 * I, H));
                break;
            case DYN_OP_DOWN:
                scratch[i] = moe ? lists + (size_t)dyn::gemm_split_k(c.dtype, H, I, c.n_experts) * r * c.top_k * H * sizeof(float) : planes(H, I);
                break;
            default: break;
        }
    }
    size_t live = 0;
    *peak = 0;
    *peak_at = 0;
    for (size_t i = 0; i < plan.size(); ++i) {
        born[i] += scratch[i];
        dies[until[i]] += scratch[i];
    }
    for (size_t i = 0; i < plan.size(); ++i) {
        live += born[i];
        if (live > *peak) { *peak = live; *peak_at = (int)i; }
        live -= dies[i];
    }
}

dyn_status check_config(const dyn_layer_config *c) {
    if (c->dtype != DYN_F32 && c->dtype != DYN_BF16) return fail(DYN_ERR_INVALID_ARG, "dtype %d", c->dtype);
    if (c->n_layers < 1 || c->hidden < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 1 ||
        c->mlp_inter < 1 || c->page_size < 1)
        return fail(DYN_ERR_INVALID_ARG, "non-positive layer dimension");
    if (c->n_q_heads % c->n_kv_heads) return fail(DYN_ERR_INVALID_ARG, "n_q_heads not a multiple of n_kv_heads");
    if (c->n_experts < 0 || c->top_k < 0 || (c->n_experts == 0) != (c->top_k == 0) || c->top_k > c->n_experts)
        return fail(DYN_ERR_INVALID_ARG, "n_experts / top_k inconsistent");
    if (!(c->rms_eps >= 0.f) || !(c->rope_base > 0.f)) return fail(DYN_ERR_INVALID_ARG, "rms_eps or rope_base");
    const int d = c->head_dim, vec = c->dtype == DYN_F32 ? 4 : 8;
    if (d < 8 || d > 2 * dyn::kMaxHalfDim || (d & (d - 1))) return fail(DYN_ERR_UNSUPPORTED, "head_dim must be a power of two in 8..256");
    if (c->hidden % vec || c->mlp_inter % vec) return fail(DYN_ERR_UNSUPPORTED, "hidden and mlp_inter must be multiples of %d", vec);
    if (c->page_size > 512) return fail(DYN_ERR_UNSUPPORTED, "page_size > 512");
    const int nk[4][2] = {{(c->n_q_heads + 2 * c->n_kv_heads) * d, c->hidden}, {c->hidden, c->n_q_heads * d},
                          {2 * c->mlp_inter, c->hidden}, {c->hidden, c->mlp_inter}};
    for (auto &p : nk)
        if (!dyn::gemm_supported(c->dtype, p[0], p[1]))
            return fail(DYN_ERR_UNSUPPORTED, "projection %d x %d: bf16 needs widths that are multiples of 128 and depths that are multiples of 256", p[0], p[1]);
    if (c->n_experts > 16) return fail(DYN_ERR_UNSUPPORTED, "at most 16 experts");
    if (c->kv_chunk_positions != 0 && (c->kv_chunk_positions < 64 || c->kv_chunk_positions > 65536 || c->kv_chunk_positions % c->page_size))
        return fail(DYN_ERR_INVALID_ARG, "kv_chunk_positions = %d: 0, or a multiple of page_size in 64..65536", c->kv_chunk_positions);
    return DYN_OK;
}

// Workspace of dyn_layer_forward_noalloc: a device array that is part of the library's code
// object, so callers that must not allocate need no workspace of their own.  Each GPU the
// library runs on holds its own copy at its own address until the process ends; the name below
// is only the host-side handle of the symbol, the address comes from hipGetSymbolAddress, once
// per device, and everything (kernel arguments included) uses that pointer.
constexpr size_t kScratchBytes = DYN_NOALLOC_MAX_WORKSPACE;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

dyn_status scratch_pointer(void **out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(DYN_ERR_UNSUPPORTED, "device index %d outside 0..%d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr || ((uintptr_t)ptr & 255)) return fail(DYN_ERR_HIP, "static scratch array resolved to a bad address %p", ptr);
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return DYN_OK;
}

dyn_status check_batch_tensors(const dyn_layer *L, const dyn_batch *b) {
    if (!b->x || !b->y || !b->seq_of_token || !b->pos_of_token || !b->block_table)
        return fail(DYN_ERR_INVALID_ARG, "NULL tensor pointer in batch");
    if (b->x == b->y) return fail(DYN_ERR_INVALID_ARG, "y must not alias x");
    if ((b->k_cache_layers != nullptr) != (b->v_cache_layers != nullptr))
        return fail(DYN_ERR_INVALID_ARG, "k_cache_layers and v_cache_layers go together");
    if (b->k_cache_layers) {
        for (int l = 0; l < L->cfg.n_layers; ++l) {
            if (!b->k_cache_layers[l] || !b->v_cache_layers[l])
                return fail(DYN_ERR_INVALID_ARG, "layer %d: NULL cache pointer in k_cache_layers / v_cache_layers", l);
            if (((uintptr_t)b->k_cache_layers[l] | (uintptr_t)b->v_cache_layers[l]) & 15)
                return fail(DYN_ERR_INVALID_ARG, "layer %d: cache pointer not 16-byte aligned", l);
        }
        return DYN_OK;
    }
    if (!b->k_cache || !b->v_cache) return fail(DYN_ERR_INVALID_ARG, "NULL tensor pointer in batch");
    if (L->cfg.n_layers > 1 && b->kv_layer_stride == 0) return fail(DYN_ERR_INVALID_ARG, "kv_layer_stride is 0 with several layers");
    return DYN_OK;
}

}  // namespace

extern "C" {

const char *dyn_last_error(void) { return g_err.c_str(); }

dyn_status dyn_layer_create(const dyn_layer_config *cfg, const dyn_layer_weights *weights, dyn_layer **out) {
    if (!cfg || !weights || !out) return fail(DYN_ERR_INVALID_ARG, "NULL argument");
    *out = nullptr;
    dyn_status rc = check_config(cfg);
    if (rc != DYN_OK) return rc;
    for (int l = 0; l < cfg->n_layers; ++l) {
        const dyn_layer_weights &w = weights[l];
        if (!w.w_qkv || !w.w_o || !w.w_gate_up || !w.w_down || !w.g_norm1 || !w.g_norm2 || (cfg->n_experts && !w.w_router))
            return fail(DYN_ERR_INVALID_ARG, "layer %d: NULL weight pointer", l);
    }
    dyn_layer *L = new dyn_layer();
    L->cfg = *cfg;
    L->w.assign(weights, weights + cfg->n_layers);
    for (int i = 0; i < cfg->head_dim / 2; ++i)
        L->rope.inv_freq[i] = std::pow((double)cfg->rope_base, -2.0 * i / cfg->head_dim);
    // split-KV chunk: a constant of the handle (256 positions unless the configuration says otherwise)
    L->chunk_pages = std::max(1, (cfg->kv_chunk_positions ? cfg->kv_chunk_positions : 256) / cfg->page_size);
    *out = L;
    return DYN_OK;
}

void dyn_layer_destroy(dyn_layer *L) {
    if (!L) return;
    (void)hipDeviceSynchronize();
    for (auto *list : {&L->graphs, &L->retired})
        for (auto &g : *list) destroy_graph_entry(g);
    for (auto ev : L->events) (void)hipEventDestroy(ev);
    for (auto ev : L->prof_events) (void)hipEventDestroy(ev);
    if (L->fork_event) (void)hipEventDestroy(L->fork_event);
    for (int key = 0; key < DYN_MAX_STREAMS; ++key)          // plain side streams; masked ones are process-wide
        if (L->streams[key]) (void)hipStreamDestroy(L->streams[key]);
    if (L->capture_stream) (void)hipStreamDestroy(L->capture_stream);
    delete L;
}

size_t dyn_layer_workspace_bytes(const dyn_layer *L, int max_tokens, int max_pages_per_seq) {
    if (!L || max_tokens < 0 || max_pages_per_seq < 0) return 0;
    return ws_bound(L, max_tokens, max_pages_per_seq);
}

dyn_status dyn_schedule_validate(const dyn_layer *L, const dyn_batch *b, const dyn_schedule *s) {
    std::vector<Dispatch> plan;
    return build_plan(L, b, s, plan);
}

size_t dyn_schedule_workspace_bytes(const dyn_layer *L, const dyn_batch *b, const dyn_schedule *s) {
    std::vector<Dispatch> plan;
    if (build_plan(L, b, s, plan) != DYN_OK) return 0;
    return plan_layout(L, b, plan, nullptr).total;
}

dyn_status dyn_schedule_regions(const dyn_layer *L, const dyn_batch *b, const dyn_schedule *s, dyn_region *out, int capacity, int *n_out) {
    if (!n_out || capacity < 0 || (capacity > 0 && !out)) return fail(DYN_ERR_INVALID_ARG, "NULL argument");
    std::vector<Dispatch> plan;
    dyn_status rc = build_plan(L, b, s, plan);
    if (rc != DYN_OK) return rc;
    std::vector<Region> regions;
    plan_layout(L, b, plan, &regions);
    *n_out = (int)regions.size();
    for (int i = 0; i < *n_out && i < capacity; ++i) {
        const Region &r = regions[i];
        out[i] = dyn_region{r.kind, r.slot, r.stream_key, r.offset, r.bytes, {0, 0}};
        for (size_t t = 0; t < r.live.size() && t < 128; ++t)
            if (r.live[t]) out[i].live_slots[t / 64] |= 1ull << (t % 64);
    }
    return DYN_OK;
}

dyn_status dyn_schedule_memory(const dyn_layer *L, const dyn_batch *b, const dyn_schedule *s, dyn_memory_report *out) {
    if (!out) return fail(DYN_ERR_INVALID_ARG, "NULL report");
    std::vector<Dispatch> plan;
    dyn_status rc = build_plan(L, b, s, plan);
    if (rc != DYN_OK) return rc;
    *out = dyn_memory_report{};
    out->workspace_bytes = ws_bound(L, b->n_tokens, b->max_pages_per_seq);
    out->workspace_bytes_schedule = plan_layout(L, b, plan, nullptr).total;
    if (b->n_tokens == 0) return DYN_OK;
    const int32_t whole[2] = {0, b->n_tokens};
    dyn_memory_report seq_report{};
    dyn_schedule seq{};
    seq.mode = DYN_SCHED_SEQUENTIAL;
    std::vector<Dispatch> seq_plan;
    if ((rc = build_plan(L, b, &seq, seq_plan)) != DYN_OK) return rc;
    int at = 0;
    analyse_memory(L, b, seq_plan, 1, whole, &seq_report, &out->peak_live_bytes_sequential, &at);
    const bool explicit_mode = s->mode == DYN_SCHED_EXPLICIT;
    analyse_memory(L, b, plan, explicit_mode ? s->k : 1, explicit_mode ? s->nano_rows : whole, out, &out->peak_live_bytes,
                   &out->peak_at_dispatch);
    return DYN_OK;
}

dyn_status dyn_layer_forward(dyn_layer *L, const dyn_batch *b, const dyn_schedule *s, void *hip_stream) {
    std::vector<Dispatch> plan;
    dyn_status rc = build_plan(L, b, s, plan);
    if (rc != DYN_OK) return rc;
    if (b->n_tokens == 0) return DYN_OK;
    if ((rc = check_batch_tensors(L, b)) != DYN_OK) return rc;
    const WsLayout ws = plan_layout(L, b, plan, nullptr);
    if (!b->workspace || ((uintptr_t)b->workspace & 255)) return fail(DYN_ERR_WORKSPACE, "workspace missing or not 256-byte aligned");
    if (b->workspace_bytes < ws.total)
        return fail(DYN_ERR_WORKSPACE, "workspace has %zu bytes, this schedule needs %zu", b->workspace_bytes, ws.total);
    hipStream_t origin = (hipStream_t)hip_stream;

    // every stream the schedule names exists before the first kernel of the forward is issued
    for (const Dispatch &d : plan)
        if (d.key() != 0) {
            hipStream_t tmp;
            rc = ensure_stream(L, s, d.key(), &tmp);
            if (rc != DYN_OK) return rc;
        }
    // A replayed HIP graph runs its kernels on streams of the executable's own, which carry no CU
    // mask: the partition of a captured dispatch is lost (attention alone on a 64-CU partition,
    // one Llama-3-8B layer at batch 256: 2182 us per step issued eagerly, 1435 us replayed, 1110 us
    // on the whole device).  A schedule that places a dispatch on a partition is therefore always
    // issued eagerly, whatever use_graph says.
    bool partitioned = false;
    for (const Dispatch &d : plan) partitioned = partitioned || d.partition > 0;
    if (!s->use_graph || partitioned) {
        rc = run_plan(L, b, s, ws, plan, origin, L->profiling);
        if (rc == DYN_OK && L->profiling) L->prof_plan = plan;
        return rc;
    }
    if (L->profiling) return fail(DYN_ERR_UNSUPPORTED, "profiling records eager schedules only");
    std::vector<unsigned char> key = graph_key(b, s, plan);
    // graphs evicted earlier are destroyed once their last replay has finished
    for (size_t i = 0; i < L->retired.size();) {
        if (hipEventQuery(L->retired[i].last_launch) == hipSuccess) {
            destroy_graph_entry(L->retired[i]);
            L->retired.erase(L->retired.begin() + i);
        } else {
            (void)hipGetLastError();       // "not ready" is an answer, not an error to find later
            ++i;
        }
    }
    // A burst of distinct schedules issued without a host wait can pile evicted executables up
    // behind their last replays.  The number alive at once is bounded: beyond it this call
    // waits for the oldest one's last replay (the only place a graph forward blocks the host).
    auto retired_branches = [&]() {
        int n = 0;
        for (const GraphEntry &g : L->retired) n += g.side_streams;
        return n;
    };
    while (!L->retired.empty() && ((int)L->retired.size() > kMaxRetiredGraphs || retired_branches() > kMaxRetiredBranches)) {
        HIP_TRY(hipEventSynchronize(L->retired.front().last_launch));
        destroy_graph_entry(L->retired.front());
        L->retired.erase(L->retired.begin());
    }
    for (auto &g : L->graphs)
        if (g.key == key) {
            HIP_TRY(hipGraphLaunch(g.exec, origin));
            HIP_TRY(hipEventRecord(g.last_launch, origin));
            return DYN_OK;
        }
    if (!L->capture_stream) HIP_TRY(hipStreamCreateWithFlags(&L->capture_stream, hipStreamNonBlocking));
    // create every event before capture starts (the streams exist already)
    while (L->events.size() < plan.size()) {
        hipEvent_t ev;
        HIP_TRY(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
        L->events.push_back(ev);
    }
    if (!L->fork_event) HIP_TRY(hipEventCreateWithFlags(&L->fork_event, hipEventDisableTiming));
    HIP_TRY(hipStreamBeginCapture(L->capture_stream, hipStreamCaptureModeRelaxed));
    rc = run_plan(L, b, s, ws, plan, L->capture_stream, false);
    hipGraph_t graph = nullptr;
    hipError_t e = hipStreamEndCapture(L->capture_stream, &graph);
    if (rc != DYN_OK) { if (graph) (void)hipGraphDestroy(graph); return rc; }
    if (e != hipSuccess) return fail(DYN_ERR_HIP, "hipStreamEndCapture: %s", hipGetErrorString(e));
    hipGraphExec_t exec = nullptr;
    e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    if (e != hipSuccess) { (void)hipGraphDestroy(graph); return fail(DYN_ERR_HIP, "hipGraphInstantiate: %s", hipGetErrorString(e)); }
    hipEvent_t last_launch = nullptr;
    e = hipEventCreateWithFlags(&last_launch, hipEventDisableTiming);
    if (e != hipSuccess) {
        (void)hipGraphExecDestroy(exec);
        (void)hipGraphDestroy(graph);
        return fail(DYN_ERR_HIP, "hipEventCreateWithFlags: %s", hipGetErrorString(e));
    }
    int side_streams = 0;
    {
        bool seen[(DYN_MAX_PARTITIONS + 1) * DYN_MAX_STREAMS] = {};
        for (const Dispatch &d : plan)
            if (d.key() != 0 && !seen[d.key()]) { seen[d.key()] = true; ++side_streams; }
    }
    // The oldest entries leave the cache at 16 graphs, and earlier when the cached graphs together
    // have many parallel branches: both segmentation faults seen inside hipGraphLaunch came with
    // 26 or more side branches among the instantiated graphs, none with 20 or fewer.  The forward
    // is asynchronous, so an evicted graph's last replay may still be running: destroyed later.
    auto branches = [&]() {
        int n = side_streams;
        for (const GraphEntry &g : L->graphs) n += g.side_streams;
        return n;
    };
    while (!L->graphs.empty() && (L->graphs.size() >= 16 || branches() > 16)) {
        L->retired.push_back(L->graphs.front());
        L->graphs.erase(L->graphs.begin());
    }
    L->graphs.push_back(GraphEntry{std::move(key), exec, graph, last_launch, side_streams});
    HIP_TRY(hipGraphLaunch(exec, origin));
    HIP_TRY(hipEventRecord(last_launch, origin));
    return DYN_OK;
}

dyn_status dyn_layer_release_graphs(dyn_layer *L) {
    if (!L) return fail(DYN_ERR_INVALID_ARG, "NULL layer");
    for (auto *list : {&L->graphs, &L->retired}) {
        for (auto &g : *list) {
            HIP_TRY(hipEventSynchronize(g.last_launch));     // recorded behind its last replay
            destroy_graph_entry(g);
        }
        list->clear();
    }
    return DYN_OK;
}

dyn_status dyn_layer_prepare(dyn_layer *L, const dyn_schedule *s) {
    if (!L) return fail(DYN_ERR_INVALID_ARG, "NULL layer");
    void *unused = nullptr;
    dyn_status rc = scratch_pointer(&unused);      // resolves this device's copy of the static scratch array as part of set-up
    if (rc != DYN_OK) return rc;
    if (!s || s->mode == DYN_SCHED_SEQUENTIAL) return DYN_OK;
    if (s->mode != DYN_SCHED_EXPLICIT) return fail(DYN_ERR_SCHEDULE, "unknown schedule mode %d", s->mode);
    if ((rc = check_schedule_fields(s)) != DYN_OK) return rc;
    for (int i = 0; i < s->n_slots; ++i) {
        const dyn_slot &sl = s->slots[i];
        if (sl.stream >= s->n_streams || sl.partition > s->n_partitions)
            return fail(DYN_ERR_SCHEDULE, "slot %d: stream %d / partition %d out of range", i, sl.stream, sl.partition);
        const int key = sl.partition * DYN_MAX_STREAMS + sl.stream;
        hipStream_t tmp;
        if (key != 0 && (rc = ensure_stream(L, s, key, &tmp)) != DYN_OK) return rc;
    }
    return DYN_OK;
}

dyn_status dyn_layer_forward_noalloc(dyn_layer *L, const dyn_batch *b, void *hip_stream) {
    dyn_schedule seq{};
    seq.mode = DYN_SCHED_SEQUENTIAL;
    std::vector<Dispatch> plan;
    dyn_status rc = build_plan(L, b, &seq, plan);
    if (rc != DYN_OK) return rc;
    if (b->n_tokens == 0) return DYN_OK;
    if ((rc = check_batch_tensors(L, b)) != DYN_OK) return rc;
    const WsLayout ws = plan_layout(L, b, plan, nullptr);
    if (ws.total > kScratchBytes)
        return fail(DYN_ERR_WORKSPACE, "this batch needs %zu bytes of workspace, the static scratch array holds %zu: use dyn_layer_forward with a workspace of the caller's",
                    ws.total, kScratchBytes);
    void *ptr = nullptr;
    if ((rc = scratch_pointer(&ptr)) != DYN_OK) return rc;
    dyn_batch local = *b;
    local.workspace = ptr;                  // the device address of this GPU's copy, never the symbol's name
    local.workspace_bytes = kScratchBytes;
    // Chain order on the caller's stream: no side stream, no event, no graph, nothing created.
    // Nothing in the workspace has to start at zero: every region is written by the operator
    // before the one that reads it, and the work lists' counters are set by the kernel that
    // builds the lists.
    for (const Dispatch &d : plan) {
        if (d.noop) continue;
        if ((rc = launch_op(L, &local, &seq, ws, d, ws.slot[(&d - plan.data()) % ws.slot.size()], (hipStream_t)hip_stream, nullptr, nullptr)) != DYN_OK) return rc;
    }
    return DYN_OK;
}

dyn_status dyn_probe_hbm_read(const void *buf, size_t bytes, void *sink, void *hip_stream) {
    if (!buf || !sink || bytes < 16 || (bytes & 15) || ((uintptr_t)buf & 15) || ((uintptr_t)sink & 3))
        return fail(DYN_ERR_INVALID_ARG, "probe needs a 16-byte aligned buffer of a multiple of 16 bytes and a sink");
    hipError_t e = dyn::launch_stream_read(buf, bytes, (uint32_t *)sink, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail(DYN_ERR_HIP, "launch of the read probe failed: %s", hipGetErrorString(e));
    return DYN_OK;
}

dyn_status dyn_probe_mfma_loop(const void *buf, size_t bytes, int n_stages, void *sink, size_t sink_bytes, void *hip_stream, double *flops) {
    if (!buf || !sink || ((uintptr_t)buf & 15) || ((uintptr_t)sink & 3) || n_stages < 1 || n_stages > (1 << 20))
        return fail(DYN_ERR_INVALID_ARG, "probe needs a 16-byte aligned buffer, a sink and 1 .. 2^20 stages");
    if (bytes < dyn::mfma_probe_bytes() || sink_bytes < (size_t)256 * 512 * sizeof(float))
        return fail(DYN_ERR_INVALID_ARG, "probe needs %zu bytes of operands and %zu bytes of sink", dyn::mfma_probe_bytes(), (size_t)256 * 512 * sizeof(float));
    hipError_t e = dyn::launch_mfma_probe(buf, n_stages, (float *)sink, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail(DYN_ERR_HIP, "launch of the matrix-core probe failed: %s", hipGetErrorString(e));
    if (flops) *flops = dyn::mfma_probe_flops(n_stages);
    return DYN_OK;
}

dyn_status dyn_layer_set_profiling(dyn_layer *L, int on) {
    if (!L) return fail(DYN_ERR_INVALID_ARG, "NULL layer");
    L->profiling = on != 0;
    return DYN_OK;
}

dyn_status dyn_layer_get_slot_times(dyn_layer *L, dyn_slot_time *out, int capacity, int *n_out) {
    if (!L || !n_out || (capacity > 0 && !out)) return fail(DYN_ERR_INVALID_ARG, "NULL argument");
    const int n = (int)L->prof_plan.size();
    *n_out = n;
    for (int i = 0; i < n && i < capacity; ++i) {
        const Dispatch &d = L->prof_plan[i];
        out[i] = dyn_slot_time{d.layer, d.op, d.nano, d.n_nano, d.stream, d.partition, 0.f, 0.f, 0.f, 0.f};
        HIP_TRY(hipEventElapsedTime(&out[i].start_ms, L->prof_events[0], L->prof_events[1 + 4 * i]));
        HIP_TRY(hipEventElapsedTime(&out[i].main_start_ms, L->prof_events[0], L->prof_events[2 + 4 * i]));
        HIP_TRY(hipEventElapsedTime(&out[i].main_stop_ms, L->prof_events[0], L->prof_events[3 + 4 * i]));
        HIP_TRY(hipEventElapsedTime(&out[i].stop_ms, L->prof_events[0], L->prof_events[4 + 4 * i]));
        if (out[i].main_stop_ms <= out[i].main_start_ms) {   // one-kernel operator: no inner marks
            out[i].main_start_ms = out[i].start_ms;
            out[i].main_stop_ms = out[i].stop_ms;
        }
    }
    return DYN_OK;
}

}  // extern "C"
