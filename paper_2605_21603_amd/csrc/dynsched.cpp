// Programmable scheduling on the host: the recorder behind split / get_ready_ops / execute
// (Section 3.2.2, Figure 6), a per-operator cost model, and the built-in policy that chooses
// between the sequential order and a two-micro-batch split (Section 2.1 "Splitting",
// Section 5.3.1).  Nothing here touches the GPU: the product of a recording is a
// dyn_schedule that dyn_layer_forward validates again and runs.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

#include "host_error.h"
#include "kernels.h"

using dyn::fail;

namespace {

const int kDenseChain[] = {DYN_OP_NORM1, DYN_OP_QKV,     DYN_OP_ROPE_KV, DYN_OP_ATTN, DYN_OP_OPROJ,
                           DYN_OP_NORM2, DYN_OP_GATE_UP, DYN_OP_SILU,    DYN_OP_DOWN};
const int kMoeChain[] = {DYN_OP_NORM1, DYN_OP_QKV,   DYN_OP_ROPE_KV, DYN_OP_ATTN, DYN_OP_OPROJ,
                         DYN_OP_NORM2, DYN_OP_ROUTE, DYN_OP_GATE_UP, DYN_OP_SILU, DYN_OP_DOWN};

}  // namespace

struct dyn_scheduler {
    dyn_layer_config cfg;
    int n_tokens, n_seqs;
    std::vector<int32_t> q_start;
    const int *chain;
    int n_chain;
    // recording state
    int k;
    std::vector<int32_t> rows;            // [k + 1] cut points
    int next[DYN_MAX_NANO];               // chain position each micro-batch executes next
    std::vector<dyn_slot> slots;
    int max_stream;
    int n_partitions, mask_words;
    std::vector<uint32_t> masks;
};

namespace {

void reset_recording(dyn_scheduler *s, int k) {
    s->k = k;
    std::fill(s->next, s->next + DYN_MAX_NANO, 0);
    s->slots.clear();
    s->max_stream = 0;
}

// ---------------------------------------------------------------------------------------
// Cost model.  Every operator is priced from its algorithmic bytes and FLOPs with the rates
// this library's kernels reach on an MI355X (per-operator events and kernel traces of the
// benchmark, Llama-3-8B shapes), plus a fixed cost per kernel launch:
//   projections, few rows     weights stream at about 3.8 TB/s
//   projections, more rows    the launcher's own tile and regime (dyn::gemm_path): a launch takes
//                             ceil(workgroups / resident workgroups) rounds of one tile's duration,
//                             a CU working at 1/256 of 0.95 PFLOP/s (1.25 with 256 x 256 tiles);
//                             planes that are not folded in registers are read back at 5 TB/s
//   decode attention          K/V stream at about 5.0 TB/s
//   prefill attention         about 0.45 PFLOP/s
//   element-wise operators    about 2 TB/s
//   a dependent kernel in a replayed graph costs about 2 us before it does anything; the
//   split-K reduce, the split-KV merge and the work-list kernel add their own launches.
// fp32 layers (the correctness configuration) are priced with the same formulas at one
// eighth of the rates; their absolute values are not meaningful.
// ---------------------------------------------------------------------------------------
struct Rates {
    double w_stream = 3.8e12, mfma = 0.95e15, mfma_wide = 1.25e15, kv_stream = 5.0e12, prefill = 0.45e15, elementwise = 2.0e12;
    double launch_us = 2.0;
};

struct OpCost {
    double us[DYN_N_OPS];
    double total() const {
        double t = 0;
        for (double v : us) t += v;
        return t;
    }
};

// Cost of the chain over token rows [r0, r1) of the batch (whole sequences).
OpCost estimate(const dyn_scheduler *s, const int32_t *ctx_len, int r0, int r1) {
    OpCost c{};
    const dyn_layer_config &g = s->cfg;
    const double e = g.dtype == DYN_BF16 ? 2.0 : 4.0;
    Rates R;
    if (g.dtype != DYN_BF16) { R.w_stream /= 8; R.mfma /= 8; R.mfma_wide /= 8; R.kv_stream /= 8; R.prefill /= 8; }
    const double T = r1 - r0;
    if (T <= 0) return c;
    const double H = g.hidden, D = g.head_dim, NQ = g.n_q_heads, NKV = g.n_kv_heads, I = g.mlp_inter;
    auto gemm = [&](double n, double k, double helper_launches) {
        const double bytes = n * k * e + T * (n + k) * e;
        double compute, tail = 0;
        if (g.dtype == DYN_BF16 && dyn::gemm_supported(1, (int)n, (int)k)) {
            // the launcher's own choice of tile and regime: a launch takes ceil(workgroups / resident)
            // rounds, each as long as one workgroup's tile takes at the rate its regime reaches
            const dyn::GemmPath p = dyn::gemm_path(1, (int)T, (int)n, (int)k);
            if (p.tail_rows) {   // the last rows as a launch of their own: at most 256 rows, tall or few-row tiles
                const dyn::GemmPath q = dyn::gemm_path(1, p.tail_rows, (int)n, (int)k);
                const double q_rounds = std::ceil((double)q.workgroups / q.resident);
                tail = std::max(n * k * e / R.w_stream, q_rounds * (5e-6 + 2.0 * q.bn * q.mt * (k / q.split) / (R.mfma / 256))) +
                       (q.split > 1 ? q.split * p.tail_rows * n * 4 / 5e12 : 0) + R.launch_us * 1e-6 * (q.split > 1 ? 2 : 1);
            }
            const double depth = p.folded ? k : k / p.split;
            const double wg_flops = 2.0 * p.bn * p.mt * depth;
            const double rounds = std::ceil((double)p.workgroups / p.resident);
            switch (p.kind) {
                case dyn::GEMM_TALL:    // one workgroup per CU; planes (if any) are read back by the reduce kernel
                    compute = rounds * (5e-6 + wg_flops / (R.mfma / 256)) + (p.split > 1 ? p.split * T * n * 4 / 5e12 : 0);
                    break;
                case dyn::GEMM_WIDE:
                    compute = rounds * (3e-6 + wg_flops / (R.mfma_wide / 256));
                    break;
                case dyn::GEMM_MANY:    // two workgroups share a CU
                    compute = rounds * 2.0 * wg_flops / (R.mfma / 256);
                    break;
                default:
                    compute = 2.0 * std::ceil(T / 128) * 128 * n * k / R.mfma;
            }
        } else {
            compute = 2.0 * std::ceil(T / 128) * 128 * n * k / R.mfma;
        }
        return (std::max(bytes / R.w_stream, compute) + tail) * 1e6 + R.launch_us * (1 + helper_launches);
    };
    auto elementwise = [&](double bytes) { return bytes / R.elementwise * 1e6 + R.launch_us; };
    // attention: decode sequences stream their K/V once per kv head; multi-token sequences are priced by FLOPs
    const int32_t *q = s->q_start.data();
    const int s0 = (int)(std::lower_bound(q, q + s->n_seqs + 1, r0) - q);
    const int s1 = (int)(std::lower_bound(q, q + s->n_seqs + 1, r1) - q);
    double kv_bytes = 0, prefill_flops = 0;
    for (int i = s0; i < s1; ++i) {
        const double ql = q[i + 1] - q[i], ctx = ctx_len[i];
        if (ql == 1) {
            kv_bytes += ctx * 2 * NKV * D * e;
        } else {
            const double pairs = ql * (2 * ctx - ql + 1) / 2;     // (query, key) pairs of a causal chunk ending at ctx
            prefill_flops += 4.0 * NQ * D * pairs;
            kv_bytes += ctx * 2 * NKV * D * e;
        }
    }
    c.us[DYN_OP_NORM1] = elementwise(2 * T * H * e);
    c.us[DYN_OP_QKV] = gemm((NQ + 2 * NKV) * D, H, 1);
    c.us[DYN_OP_ROPE_KV] = elementwise(2 * T * (NQ + 2 * NKV) * D * e);
    c.us[DYN_OP_ATTN] = (kv_bytes / R.kv_stream + prefill_flops / R.prefill) * 1e6 + 3 * R.launch_us;
    c.us[DYN_OP_OPROJ] = gemm(H, NQ * D, 1);
    c.us[DYN_OP_NORM2] = elementwise(2 * T * H * e);
    if (g.n_experts > 0) {
        // every expert that receives a token is read once; with T * top_k pairs spread over E experts
        const double pairs = T * g.top_k, experts_hit = std::min<double>(g.n_experts, pairs);
        c.us[DYN_OP_ROUTE] = elementwise(T * H * e) + 2 * R.launch_us;
        const double fl_gu = 2.0 * pairs * 2 * I * H, fl_d = 2.0 * pairs * H * I;
        c.us[DYN_OP_GATE_UP] = std::max(experts_hit * 2 * I * H * e / R.w_stream, fl_gu / R.mfma) * 1e6 + R.launch_us;
        c.us[DYN_OP_DOWN] = std::max(experts_hit * H * I * e / R.w_stream, fl_d / R.mfma) * 1e6 + 3 * R.launch_us;
        c.us[DYN_OP_SILU] = 0;
    } else {
        c.us[DYN_OP_GATE_UP] = gemm(2 * I, H, 0);
        c.us[DYN_OP_SILU] = 0;                                    // applied in the gate/up epilogue
        c.us[DYN_OP_DOWN] = gemm(H, I, 1);
    }
    return c;
}

// Two streams that run side by side share the CUs' memory pipelines: while a decode-attention
// kernel streams K/V, a co-resident projection kernel advances at a fraction of its own speed
// (its L2 reads queue behind the attention's HBM reads), so the makespan of a prefill
// micro-batch beside a decode micro-batch is the longer stream plus most of the shorter one.
// How much of the shorter one stays unhidden grows with the prefill chunk: small chunks leave
// CUs and launch gaps for the other stream, 2048 tokens and more fill the chip round after
// round.  Fitted to prefill chunks of 256..4096 tokens beside 64..256 decodes at contexts
// 2048..8192 (measured split time = longer + share x shorter, estimates scaled to the measured
// sequential time): 0.58-0.76 at 256 tokens, 0.77-0.81 at 512, 0.71-0.88 at 1024, 0.90-0.99 at 2048.
double unhidden_share(int prefill_tokens) {
    if (prefill_tokens <= 384) return 0.62;
    if (prefill_tokens <= 1536) return 0.80;
    return 0.93;
}

}  // namespace

extern "C" {

dyn_status dyn_scheduler_create(const dyn_layer_config *cfg, int n_tokens, int n_seqs, const int32_t *q_start_host,
                                dyn_scheduler **out) {
    if (!cfg || !out) return fail(DYN_ERR_INVALID_ARG, "NULL config or output pointer");
    *out = nullptr;
    if (n_tokens < 0 || n_seqs < 0 || (n_tokens > 0 && n_seqs == 0))
        return fail(DYN_ERR_INVALID_ARG, "bad n_tokens / n_seqs (%d, %d)", n_tokens, n_seqs);
    if (!q_start_host) return fail(DYN_ERR_INVALID_ARG, "q_start_host is NULL");
    if (q_start_host[0] != 0 || q_start_host[n_seqs] != n_tokens)
        return fail(DYN_ERR_INVALID_ARG, "q_start_host must run from 0 to n_tokens");
    for (int i = 0; i < n_seqs; ++i)
        if (q_start_host[i + 1] <= q_start_host[i])
            return fail(DYN_ERR_INVALID_ARG, "sequence %d has no token in this step", i);
    if ((cfg->n_experts > 0) != (cfg->top_k > 0)) return fail(DYN_ERR_INVALID_ARG, "n_experts and top_k must both be 0 or both positive");
    dyn_scheduler *s = new dyn_scheduler();
    s->cfg = *cfg;
    s->n_tokens = n_tokens;
    s->n_seqs = n_seqs;
    s->q_start.assign(q_start_host, q_start_host + n_seqs + 1);
    s->chain = cfg->n_experts > 0 ? kMoeChain : kDenseChain;
    s->n_chain = cfg->n_experts > 0 ? 10 : 9;
    s->rows = {0, n_tokens};
    s->n_partitions = 0;
    s->mask_words = 0;
    reset_recording(s, 1);
    *out = s;
    return DYN_OK;
}

void dyn_scheduler_destroy(dyn_scheduler *s) { delete s; }

dyn_status dyn_scheduler_split(dyn_scheduler *s, int k, const int32_t *sizes) {
    if (!s || !sizes) return fail(DYN_ERR_INVALID_ARG, "NULL scheduler or sizes");
    if (k < 1 || k > DYN_MAX_NANO) return fail(DYN_ERR_SCHEDULE, "k = %d outside 1..%d", k, DYN_MAX_NANO);
    std::vector<int32_t> rows(k + 1, 0);
    for (int i = 0; i < k; ++i) {
        if (sizes[i] < 0) return fail(DYN_ERR_SCHEDULE, "micro-batch %d has negative size", i);
        rows[i + 1] = rows[i] + sizes[i];
        if (!std::binary_search(s->q_start.begin(), s->q_start.end(), rows[i + 1]))
            return fail(DYN_ERR_SCHEDULE, "micro-batch %d ends at row %d, inside a sequence", i, rows[i + 1]);
    }
    if (rows[k] != s->n_tokens)
        return fail(DYN_ERR_SCHEDULE, "micro-batch sizes add up to %d, the batch has %d tokens", rows[k], s->n_tokens);
    s->rows = rows;
    reset_recording(s, k);
    return DYN_OK;
}

dyn_status dyn_scheduler_set_partitions(dyn_scheduler *s, int n_partitions, const uint32_t *cu_masks, int cu_mask_words) {
    if (!s) return fail(DYN_ERR_INVALID_ARG, "NULL scheduler");
    if (n_partitions < 0 || n_partitions > DYN_MAX_PARTITIONS)
        return fail(DYN_ERR_SCHEDULE, "n_partitions = %d outside 0..%d", n_partitions, DYN_MAX_PARTITIONS);
    if (n_partitions > 0 && (!cu_masks || cu_mask_words < 1 || cu_mask_words > 32))
        return fail(DYN_ERR_SCHEDULE, "partitions need cu_masks with 1..32 words each");
    for (int p = 0; p < n_partitions; ++p) {
        uint32_t any = 0;
        for (int i = 0; i < cu_mask_words; ++i) any |= cu_masks[p * cu_mask_words + i];
        if (!any) return fail(DYN_ERR_SCHEDULE, "CU mask of partition %d is empty", p + 1);
    }
    for (const dyn_slot &sl : s->slots)
        if (sl.partition > n_partitions)
            return fail(DYN_ERR_SCHEDULE, "a recorded dispatch already uses partition %d", sl.partition);
    s->n_partitions = n_partitions;
    s->mask_words = n_partitions ? cu_mask_words : 0;
    s->masks.assign(cu_masks, cu_masks + (size_t)n_partitions * s->mask_words);
    return DYN_OK;
}

int dyn_scheduler_get_ready_ops(const dyn_scheduler *s, int nano, uint8_t *ops, int capacity) {
    if (!s || nano < 0 || nano >= s->k || capacity < 0 || (capacity > 0 && !ops)) {
        fail(DYN_ERR_INVALID_ARG, "bad scheduler, micro-batch index or buffer");
        return -1;
    }
    if (s->next[nano] >= s->n_chain) return 0;
    if (capacity > 0) ops[0] = (uint8_t)s->chain[s->next[nano]];
    return 1;
}

dyn_status dyn_scheduler_execute(dyn_scheduler *s, int n, const uint8_t *ops, const uint8_t *nanos, int stream,
                                 int partition) {
    if (!s || !ops || !nanos) return fail(DYN_ERR_INVALID_ARG, "NULL scheduler, ops or nanos");
    if (n < 1) return fail(DYN_ERR_INVALID_ARG, "execute needs at least one (operator, micro-batch) pair");
    if (stream < 0 || stream >= DYN_MAX_STREAMS) return fail(DYN_ERR_SCHEDULE, "stream %d outside 0..%d", stream, DYN_MAX_STREAMS - 1);
    if (partition < 0 || partition > s->n_partitions)
        return fail(DYN_ERR_SCHEDULE, "partition %d outside 0..%d (set_partitions first)", partition, s->n_partitions);
    // readiness of every pair, in the order given (a pair may depend on an earlier pair of the same call)
    int next[DYN_MAX_NANO];
    std::copy(s->next, s->next + DYN_MAX_NANO, next);
    for (int i = 0; i < n; ++i) {
        const int nb = nanos[i];
        if (nb >= s->k) return fail(DYN_ERR_SCHEDULE, "pair %d: micro-batch %d outside 0..%d", i, nb, s->k - 1);
        if (next[nb] >= s->n_chain)
            return fail(DYN_ERR_SCHEDULE, "pair %d: micro-batch %d has already finished the layer", i, nb);
        if (s->chain[next[nb]] != ops[i])
            return fail(DYN_ERR_SCHEDULE, "pair %d: operator %d of micro-batch %d is not ready (operator %d is next)", i,
                        ops[i], nb, s->chain[next[nb]]);
        ++next[nb];
    }
    // merge form: one operator over adjacent micro-batches in ascending order
    bool merge = n > 1;
    for (int i = 1; i < n && merge; ++i) merge = ops[i] == ops[0] && nanos[i] == nanos[i - 1] + 1;
    if (merge || n == 1) {
        s->slots.push_back(dyn_slot{ops[0], nanos[0], (uint8_t)n, (uint8_t)stream, (uint8_t)partition});
    } else {
        for (int i = 0; i < n; ++i)   // sequential fallback: no fused kernel for different operators
            s->slots.push_back(dyn_slot{ops[i], nanos[i], 1, (uint8_t)stream, (uint8_t)partition});
    }
    std::copy(next, next + DYN_MAX_NANO, s->next);
    s->max_stream = std::max(s->max_stream, stream);
    return DYN_OK;
}

dyn_status dyn_scheduler_finish(dyn_scheduler *s, int use_graph, dyn_schedule *out) {
    if (!s || !out) return fail(DYN_ERR_INVALID_ARG, "NULL scheduler or output");
    for (int nb = 0; nb < s->k; ++nb)
        if (s->next[nb] < s->n_chain)
            return fail(DYN_ERR_SCHEDULE, "micro-batch %d stops before operator %d: the layer is incomplete", nb,
                        s->chain[s->next[nb]]);
    out->mode = DYN_SCHED_EXPLICIT;
    out->k = s->k;
    out->nano_rows = s->rows.data();
    out->n_streams = s->max_stream + 1;
    out->n_partitions = s->n_partitions;
    out->cu_masks = s->n_partitions ? s->masks.data() : nullptr;
    out->cu_mask_words = s->mask_words;
    out->n_slots = (int)s->slots.size();
    out->slots = s->slots.data();
    out->use_graph = use_graph ? 1 : 0;
    return DYN_OK;
}

dyn_status dyn_policy_auto(dyn_scheduler *s, const int32_t *ctx_len_host, int use_graph, dyn_schedule *out,
                           dyn_policy_choice *choice) {
    if (!s || !ctx_len_host || !out) return fail(DYN_ERR_INVALID_ARG, "NULL scheduler, ctx_len_host or output");
    for (int i = 0; i < s->n_seqs; ++i)
        if (ctx_len_host[i] < s->q_start[i + 1] - s->q_start[i])
            return fail(DYN_ERR_INVALID_ARG, "sequence %d attends %d keys but has %d tokens in this step", i, ctx_len_host[i],
                        s->q_start[i + 1] - s->q_start[i]);
    const int T = s->n_tokens;
    // the one cut considered: between a run of multi-token sequences and a run of single-token ones
    int cut = -1;
    {
        int flips = 0, at = -1;
        for (int i = 1; i < s->n_seqs; ++i) {
            const bool a = s->q_start[i] - s->q_start[i - 1] > 1, b = s->q_start[i + 1] - s->q_start[i] > 1;
            if (a != b) { ++flips; at = s->q_start[i]; }
        }
        if (flips == 1) cut = at;
    }
    const double t_seq = estimate(s, ctx_len_host, 0, T).total();
    double t_split = 0;
    if (cut > 0) {
        const double a = estimate(s, ctx_len_host, 0, cut).total(), b = estimate(s, ctx_len_host, cut, T).total();
        const int multi_rows = s->q_start[1] - s->q_start[0] > 1 ? cut : T - cut;     // tokens of the multi-token side of the cut
        t_split = std::max(a, b) + unhidden_share(multi_rows) * std::min(a, b);
    }
    // The model is good to about 5-8 % on mixes of 256..4096 prefill tokens and 64..256 decodes,
    // but its errors on the two orders go the same way.  A predicted gain below 1 % is not worth
    // the extra streams.
    const bool split = cut > 0 && t_split < 0.99 * t_seq;
    if (choice) {
        choice->split = split;
        choice->cut_row = split ? cut : 0;
        choice->est_sequential_us = (float)t_seq;
        choice->est_split_us = (float)t_split;
    }
    dyn_status rc;
    if (!split) {
        const int32_t all = T;
        if ((rc = dyn_scheduler_split(s, 1, &all)) != DYN_OK) return rc;
        for (int i = 0; i < s->n_chain; ++i) {
            const uint8_t op = (uint8_t)s->chain[i], nb = 0;
            if ((rc = dyn_scheduler_execute(s, 1, &op, &nb, 0, 0)) != DYN_OK) return rc;
        }
    } else {
        const int32_t sizes[2] = {cut, T - cut};
        if ((rc = dyn_scheduler_split(s, 2, sizes)) != DYN_OK) return rc;
        // a strategy in the paper's style: each micro-batch on its own stream, issued round-robin
        // one ready operator at a time, so the long stream's GEMMs meet the short one's attention
        for (;;) {
            bool any = false;
            for (uint8_t nb = 0; nb < 2; ++nb) {
                uint8_t op;
                if (dyn_scheduler_get_ready_ops(s, nb, &op, 1) == 1) {
                    if ((rc = dyn_scheduler_execute(s, 1, &op, &nb, nb, 0)) != DYN_OK) return rc;
                    any = true;
                }
            }
            if (!any) break;
        }
    }
    return dyn_scheduler_finish(s, use_graph, out);
}

// ---------------------------------------------------------------------------------------
// Candidates of the measured tuner (Section 2.1: unequal micro-batch sizes, the share of
// compute units per overlapped stream; Section 5.3.4: chosen per batch at run time).

namespace {

// the sequence boundary strictly inside (0, T) nearest to `target`; -1 if there is none
int snap_to_boundary(const dyn_scheduler *s, long target) {
    int best = -1;
    for (int i = 1; i < s->n_seqs; ++i) {
        const int b = s->q_start[i];
        if (b <= 0 || b >= s->n_tokens) continue;
        if (best < 0 || std::labs((long)b - target) < std::labs((long)best - target)) best = b;
    }
    return best;
}

bool op_is_merged(int form, int op) {
    if (form == DYN_FORM_MLP_MERGED) return op >= DYN_OP_ROUTE;
    if (form == DYN_FORM_MLP_SPLIT) return op <= DYN_OP_NORM2;
    if (form == DYN_FORM_ATTN_SPLIT) return op == DYN_OP_QKV || op == DYN_OP_OPROJ || op == DYN_OP_GATE_UP || op == DYN_OP_DOWN;
    return false;
}

}  // namespace

int dyn_tune_candidates(const dyn_scheduler *s, const int32_t *ctx_len_host, const dyn_tune_options *opt,
                        dyn_tune_candidate *table, int capacity) {
    if (!s || !opt || capacity < 0 || (capacity > 0 && !table)) {
        fail(DYN_ERR_INVALID_ARG, "NULL scheduler, options or table");
        return -1;
    }
    const int max_k = opt->max_k ? opt->max_k : 2;
    const int n_cus = opt->n_cus ? opt->n_cus : 256;
    if (max_k < 1 || max_k > 4 || opt->partitions < 0 || opt->partitions > 3 || n_cus < 8 || n_cus % 8) {
        fail(DYN_ERR_INVALID_ARG, "max_k outside 1..4, partitions outside 0..3 or n_cus not a multiple of 8");
        return -1;
    }
    const int T = s->n_tokens;
    int n = 0;
    auto emit = [&](int k, const int32_t *rows, int form, int stagger, int cus_first) {
        if (n < capacity) {
            dyn_tune_candidate &c = table[n];
            std::memset(&c, 0, sizeof c);
            c.k = k;
            std::copy(rows, rows + k + 1, c.rows);
            c.form = form;
            c.stagger = stagger;
            c.cus_first = cus_first;
        }
        ++n;
    };
    const int32_t whole[2] = {0, T};
    emit(1, whole, DYN_FORM_SEQUENTIAL, 0, 0);
    if (max_k < 2 || s->n_seqs < 2) return n;

    // two micro-batches: cut points in ascending order, each once
    std::vector<int> cuts;
    auto add_cut = [&](int c) {
        if (c > 0 && c < T && std::find(cuts.begin(), cuts.end(), c) == cuts.end()) cuts.push_back(c);
    };
    for (int eighths : {2, 3, 4, 5, 6}) add_cut(snap_to_boundary(s, (long)T * eighths / 8));
    if (ctx_len_host) {   // the boundary where the keys to attend (the attention's bytes) are halved
        double total = 0, run = 0;
        for (int i = 0; i < s->n_seqs; ++i) total += ctx_len_host[i];
        for (int i = 0; i + 1 < s->n_seqs; ++i) {
            run += ctx_len_host[i];
            if (run >= total / 2) { add_cut(s->q_start[i + 1]); break; }
        }
    }
    {   // multi-token (prefill) sequences on one side, single-token (decode) ones on the other
        int flips = 0, at = -1;
        for (int i = 1; i < s->n_seqs; ++i) {
            const bool a = s->q_start[i] - s->q_start[i - 1] > 1, b = s->q_start[i + 1] - s->q_start[i] > 1;
            if (a != b) { ++flips; at = s->q_start[i]; }
        }
        if (flips == 1) add_cut(at);
    }
    std::sort(cuts.begin(), cuts.end());
    const int quarter = n_cus / 4;
    const int shares[3] = {2 * quarter, 3 * quarter, quarter};
    for (int c : cuts) {
        const int32_t rows[3] = {0, c, T};
        emit(2, rows, DYN_FORM_SPLIT, 2, 0);
        emit(2, rows, DYN_FORM_MLP_MERGED, 1, 0);
        emit(2, rows, DYN_FORM_MLP_MERGED, 2, 0);
        emit(2, rows, DYN_FORM_ATTN_SPLIT, 1, 0);
        emit(2, rows, DYN_FORM_MLP_SPLIT, 1, 0);
        for (int p = 0; p < opt->partitions; ++p) {
            emit(2, rows, DYN_FORM_SPLIT, 2, shares[p]);
            emit(2, rows, DYN_FORM_MLP_MERGED, 2, shares[p]);
        }
    }
    // three and four micro-batches: equal token counts snapped to boundaries, strictly increasing
    for (int k = 3; k <= max_k; ++k) {
        int32_t rows[DYN_MAX_NANO + 1] = {0};
        bool ok = true;
        for (int i = 1; i < k && ok; ++i) {
            rows[i] = snap_to_boundary(s, (long)T * i / k);
            ok = rows[i] > rows[i - 1];
        }
        rows[k] = T;
        if (!ok || rows[k - 1] >= T) continue;
        emit(k, rows, DYN_FORM_SPLIT, 1, 0);
        emit(k, rows, DYN_FORM_MLP_MERGED, 1, 0);
        emit(k, rows, DYN_FORM_ATTN_SPLIT, 1, 0);
        if (opt->partitions > 0) emit(k, rows, DYN_FORM_MLP_MERGED, 1, shares[0]);
    }
    return n;
}

dyn_status dyn_tune_record(dyn_scheduler *s, const dyn_tune_candidate *c, int n_cus, int use_graph, dyn_schedule *out) {
    if (!s || !c || !out) return fail(DYN_ERR_INVALID_ARG, "NULL scheduler, candidate or output");
    if (c->k < 1 || c->k > DYN_MAX_NANO || c->form < DYN_FORM_SEQUENTIAL || c->form > DYN_FORM_MLP_SPLIT || c->stagger < 0)
        return fail(DYN_ERR_INVALID_ARG, "candidate with k = %d, form = %d, stagger = %d", c->k, c->form, c->stagger);
    if ((c->form == DYN_FORM_SEQUENTIAL) != (c->k == 1))
        return fail(DYN_ERR_INVALID_ARG, "the sequential form has one micro-batch and the others at least two");
    dyn_status rc;
    int32_t sizes[DYN_MAX_NANO];
    for (int i = 0; i < c->k; ++i) sizes[i] = c->rows[i + 1] - c->rows[i];
    if (c->rows[0] != 0) return fail(DYN_ERR_SCHEDULE, "the first micro-batch starts at row %d", c->rows[0]);
    if ((rc = dyn_scheduler_split(s, c->k, sizes)) != DYN_OK) return rc;
    if (c->cus_first) {
        // Partition 1 takes the low `low` bits of every 32-bit mask word, partition 2 the rest.  Bit i
        // of a mask is compute unit i / 8 of XCD i % 8, so every XCD gives the same share whenever
        // `low` is a multiple of 8 (the quarter shares of 256 units: 8, 16 and 24 bits per word).
        if (n_cus <= 0) n_cus = 256;
        const int words = (n_cus + 31) / 32, per_word = n_cus / words;
        const int low = c->cus_first / words;
        if (c->cus_first % words || low < 1 || low >= per_word)
            return fail(DYN_ERR_INVALID_ARG, "cus_first = %d does not divide into %d mask words of %d CUs", c->cus_first, words, per_word);
        std::vector<uint32_t> masks((size_t)2 * words);
        const uint32_t lo = (1u << low) - 1u, all = per_word == 32 ? 0xffffffffu : (1u << per_word) - 1u;
        for (int i = 0; i < words; ++i) {
            masks[i] = lo;
            masks[words + i] = all & ~lo;
        }
        if ((rc = dyn_scheduler_set_partitions(s, 2, masks.data(), words)) != DYN_OK) return rc;
    } else if ((rc = dyn_scheduler_set_partitions(s, 0, nullptr, 0)) != DYN_OK) {
        return rc;
    }
    // Micro-batches advance operator by operator, micro-batch b `stagger` operators behind
    // b-1; an operator of a merged class is dispatched once, when the last micro-batch arrives.
    int pos[DYN_MAX_NANO] = {0};
    const int k = c->k;
    for (int tick = 0;; ++tick) {
        bool done = true;
        for (int b = 0; b < k; ++b) done = done && pos[b] >= s->n_chain;
        if (done) break;
        for (int b = 0; b < k; ++b) {
            if (pos[b] >= s->n_chain || tick < b * c->stagger) continue;
            const uint8_t op = (uint8_t)s->chain[pos[b]];
            if (!op_is_merged(c->form, op)) {
                const uint8_t nb = (uint8_t)b;
                const int part = c->cus_first ? 1 + (b & 1) : 0;
                if ((rc = dyn_scheduler_execute(s, 1, &op, &nb, k == 1 ? 0 : b, part)) != DYN_OK) return rc;
                ++pos[b];
            } else {
                bool all_here = true;
                for (int j = 0; j < k; ++j) all_here = all_here && pos[j] == pos[b];
                if (!all_here) continue;
                uint8_t ops[DYN_MAX_NANO], nbs[DYN_MAX_NANO];
                for (int j = 0; j < k; ++j) { ops[j] = op; nbs[j] = (uint8_t)j; }
                if ((rc = dyn_scheduler_execute(s, k, ops, nbs, 0, 0)) != DYN_OK) return rc;
                for (int j = 0; j < k; ++j) ++pos[j];
            }
        }
    }
    return dyn_scheduler_finish(s, use_graph, out);
}

}  // extern "C"
