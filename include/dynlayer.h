/*
 * dynlayer - transformer decoder-layer forward step for MI355X (gfx950), run either
 * sequentially or as nano-batches whose operators overlap on one GPU.
 *
 * The scheduling contract follows the paper's programmable operator scheduling
 * (Section 3.2.2, Figure 6): a batch is split into k micro-batches of chosen sizes
 * ("split"), each micro-batch advances through a chain of coarse operators in order
 * (the "ready operators" rule), and every dispatch ("execute") names the operator, the
 * micro-batches it covers - one (split form) or several adjacent ones (merge form) -
 * and the stream it runs on.  Data flow between operators is the library's business
 * (Section 3.3.1, Algorithm 1): every intermediate is one contiguous [tokens, width]
 * buffer and a micro-batch is a row range of it, so splitting and merging never copy.
 *
 * All tensor arguments are DEVICE pointers owned by the caller and only borrowed here,
 * unless a field says HOST.  The library owns streams, events, graphs and its handle.
 * No function throws; each returns a dyn_status and dyn_last_error() gives the detail.
 *
 * Tensor layouts (row-major, last index fastest; element type = dyn_layer_config.dtype
 * unless stated):
 *   x, y         [n_tokens, hidden]
 *   w_qkv        [(n_q_heads + 2 n_kv_heads) * head_dim, hidden]  q rows, k rows, v rows
 *   w_o          [hidden, n_q_heads * head_dim]
 *   w_gate_up    [2 * mlp_inter, hidden] gate rows then up rows;  MoE: [E, 2*mlp_inter, hidden]
 *   w_down       [hidden, mlp_inter];                             MoE: [E, hidden, mlp_inter]
 *   w_router     [E, hidden] float32 always (MoE only)
 *   g_norm1/2    [hidden]
 *   k_cache      [n_pages, n_kv_heads, page_size, head_dim]
 *   v_cache      [n_pages, n_kv_heads, head_dim, page_size]   (position fastest in a page)
 *   block_table  [n_seqs, max_pages_per_seq] int32: physical page of a logical page
 * Every weight matrix is output-major: out = in * W^T.
 */
#ifndef DYNLAYER_H
#define DYNLAYER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DYN_OK = 0,
    DYN_ERR_INVALID_ARG = 1, /* NULL pointer, negative size, inconsistent shapes */
    DYN_ERR_UNSUPPORTED = 2, /* a shape or dtype no kernel here handles */
    DYN_ERR_SCHEDULE = 3,    /* descriptor breaks the ready-operator rule or its own bounds */
    DYN_ERR_WORKSPACE = 4,   /* workspace missing, misaligned or too small */
    DYN_ERR_HIP = 5          /* a HIP runtime call failed */
} dyn_status;

enum { DYN_F32 = 0, DYN_BF16 = 1 };

/* The operator chain of one layer, in dependency order.  Granularity is the logical
 * coarse operator (a norm, a projection, attention), as the paper's graph partitioning
 * argues (Section 3.2.1).  DYN_OP_ROUTE exists only in MoE layers. */
enum {
    DYN_OP_NORM1 = 0,   /* h1 = RMSNorm(x) */
    DYN_OP_QKV = 1,     /* [q|k|v] = h1 W_qkv^T */
    DYN_OP_ROPE_KV = 2, /* rotary on q and k; k', v appended to the paged cache */
    DYN_OP_ATTN = 3,    /* causal paged attention of each token over positions 0..pos */
    DYN_OP_OPROJ = 4,   /* x2 = x + o W_o^T */
    DYN_OP_NORM2 = 5,   /* h2 = RMSNorm(x2) */
    DYN_OP_ROUTE = 6,   /* MoE: router logits, top-k selection, softmax weights */
    DYN_OP_GATE_UP = 7, /* [g|u] = h2 W_gate_up^T   (MoE: per selected expert) */
    DYN_OP_SILU = 8,    /* a = silu(g) * u */
    DYN_OP_DOWN = 9,    /* y = x2 + a W_down^T      (MoE: weighted sum over selected experts) */
    DYN_N_OPS = 10
};

typedef struct {
    int dtype;                 /* DYN_F32 | DYN_BF16: weights, activations and caches */
    int n_layers;              /* >= 1; layer l+1 takes layer l's output */
    int hidden, n_q_heads, n_kv_heads, head_dim, mlp_inter;
    int n_experts, top_k;      /* 0, 0 = dense MLP */
    float rms_eps, rope_base;  /* rotary: rotate-half pairing (i, i + head_dim/2) */
    int page_size;             /* positions per cache page */
    int kv_chunk_positions;    /* split-KV chunk of a single-token (decode) sequence's attention, in positions: 0 = 256,
                                  else a multiple of page_size in 64..65536.  A sequence of P pages is walked as
                                  ceil(P / chunk pages) work items of equal size whose partial results are merged in
                                  order, so the value is part of the arithmetic (a constant of the handle: every
                                  schedule of a handle gives the same bits).  Small chunks give few sequences enough
                                  work items to fill the chip; large ones write fewer partials and switch items less
                                  often (32 layers at batch 256, contexts 1024..8192: 256 -> 2048 positions takes 4.5 %
                                  off the layer; batch 128, contexts 512..4096: 1024 is 1 % faster, 2048 5 % slower) */
} dyn_layer_config;

/* One entry per layer (array of n_layers). */
typedef struct {
    const void *w_qkv, *w_o, *w_gate_up, *w_down, *g_norm1, *g_norm2;
    const float *w_router;     /* NULL for dense layers */
} dyn_layer_weights;

typedef struct {
    int n_tokens, n_seqs;
    const void *x;                 /* [n_tokens, hidden], read only */
    void *y;                       /* [n_tokens, hidden], written; must not alias x */
    const int32_t *seq_of_token;   /* [n_tokens] sequence of each token row */
    const int32_t *pos_of_token;   /* [n_tokens] position in its sequence; it attends keys 0..pos */
    const int32_t *block_table;    /* [n_seqs, max_pages_per_seq] */
    int max_pages_per_seq;
    const int32_t *q_start_host;   /* HOST [n_seqs + 1]: token rows of sequence s are
                                      q_start_host[s] .. q_start_host[s+1]-1, in position order */
    void *k_cache, *v_cache;       /* layer 0; MUTATED: this step's k', v are stored */
    size_t kv_layer_stride;        /* bytes from layer l's cache to layer l+1's (both caches) */
    void *workspace;               /* >= dyn_schedule_workspace_bytes(...) for the schedule run (dyn_layer_workspace_bytes
                                      covers every schedule), 256-byte aligned */
    size_t workspace_bytes;
    void *const *k_cache_layers;   /* HOST [n_layers] device pointers, or both NULL.  When set, layer l's caches are */
    void *const *v_cache_layers;   /* these (16-byte aligned) and k_cache, v_cache, kv_layer_stride are ignored: every
                                      layer's K and V pool can be placed on its own.  Where the two pools of a layer lie
                                      in HBM changes the rate of the attention launch that reads them together by up to
                                      14 % on MI355X (measured; see dyn_layer_forward) */
} dyn_batch;

/* One dispatch: operator `op` over micro-batches nano .. nano + n_nano - 1 (n_nano = 1 is
 * the paper's split form, n_nano > 1 its merge form) on stream `stream` of CU partition
 * `partition` (0 = whole device; p >= 1 = cu_masks row p-1).  Stream 0 of partition 0 is
 * the caller's stream. */
typedef struct {
    uint8_t op, nano, n_nano, stream, partition;
} dyn_slot;

enum { DYN_SCHED_SEQUENTIAL = 0, DYN_SCHED_EXPLICIT = 1 };
enum { DYN_MAX_NANO = 8, DYN_MAX_STREAMS = 8, DYN_MAX_PARTITIONS = 4 };

typedef struct {
    int mode;                   /* SEQUENTIAL: whole batch, chain order, caller's stream; rest ignored
                                   except use_graph */
    int k;                      /* micro-batches, 1..DYN_MAX_NANO */
    const int32_t *nano_rows;   /* HOST [k+1]: token-row cut points, 0 .. n_tokens, non-decreasing,
                                   on sequence boundaries; unequal sizes allowed */
    int n_streams;              /* stream ids 0..n_streams-1 */
    int n_partitions;           /* masked partitions 1..n_partitions */
    const uint32_t *cu_masks;   /* HOST [n_partitions, cu_mask_words] for hipExtStreamCreateWithCUMask.  On MI355X
                                   bit i of a mask (bit i % 32 of word i / 32) is compute unit i / 8 of XCD i % 8:
                                   a run of 8 n consecutive bits takes n units of every XCD, which is what a
                                   persistent launch sized for "two workgroups per unit of the partition" needs */
    int cu_mask_words;
    int n_slots;                /* issue order within one layer; the list repeats for every layer */
    const dyn_slot *slots;      /* HOST */
    int use_graph;              /* 1: capture the whole step into a HIP graph once and replay it.  Ignored
                                   (the step is issued eagerly) when a slot names a partition: a replayed graph
                                   runs on streams of its own, which carry no CU mask */
} dyn_schedule;

typedef struct dyn_layer dyn_layer;

/* Records configuration and weight pointers.  Touches no GPU state (streams, events and
 * graphs are created on first forward), so it and the validator run without a device. */
dyn_status dyn_layer_create(const dyn_layer_config *cfg, const dyn_layer_weights *weights, dyn_layer **out);

/* Releases streams, events, graphs.  Outstanding work must have been synchronised. */
void dyn_layer_destroy(dyn_layer *layer);

/* Bytes of workspace that suffice for ANY legal schedule of a forward of up to max_tokens
 * tokens when no sequence has more than max_pages_per_seq pages: every intermediate and every
 * operator's scratch for the whole batch at once, nothing shared.  A particular schedule
 * usually needs much less: see dyn_schedule_workspace_bytes. */
size_t dyn_layer_workspace_bytes(const dyn_layer *layer, int max_tokens, int max_pages_per_seq);

/* Host-only check of a schedule against a batch's shapes (no device memory is read):
 * cut points monotone, covering [0, n_tokens], on sequence boundaries; each (operator,
 * micro-batch) dispatched exactly once per layer; every dispatch issued after the
 * dispatches producing its inputs for all micro-batches it covers (ready-operator rule,
 * Section 3.2.2); stream / partition ids in range.  batch->workspace may be NULL here. */
dyn_status dyn_schedule_validate(const dyn_layer *layer, const dyn_batch *batch, const dyn_schedule *sched);

/* Creates ahead of time the GPU state a schedule's forwards need: its side streams.  A
 * CU-masked stream (partition >= 1) is a hardware queue that is only ever created while the
 * device is idle, so this call SYNCHRONISES THE DEVICE whenever it has to create one; masked
 * streams are shared by all handles of the process, keyed by (stream id, mask), and live
 * until the process ends.  Section 2.1 ("Overlapping") names partitioned contexts as the
 * second way to overlap beside plain streams; this is their set-up step.  Optional: a
 * forward creates what is missing itself (see below).  sched may be NULL or sequential
 * (no stream to create).  Also resolves the current device's copy of the static workspace
 * of dyn_layer_forward_noalloc. */
dyn_status dyn_layer_prepare(dyn_layer *layer, const dyn_schedule *sched);

/* Runs all layers.  Asynchronous: work is forked from hip_stream (a hipStream_t, not the
 * null stream when use_graph is set) and joined back to it; the host does not wait and
 * nothing is allocated on the device.  One exception to "the host does not wait": the first
 * forward that names a (stream id, CU mask) pair no earlier forward or dyn_layer_prepare
 * call of the process has used creates that masked stream, which synchronises the device
 * once (and would invalidate a stream capture the caller has open on hip_stream): call
 * dyn_layer_prepare with the schedule beforehand to keep every forward asynchronous.
 * Cross-stream dependencies are inserted by the
 * library (the backend, not the scheduler author, owns data flow; Section 3.2.2).
 * Output rows land at their global row index whatever the split (zero-copy merge,
 * Section 3.3.1).  Any legal schedule gives bit-identical y and cache contents.
 * With use_graph the captured step is cached (16 graphs, fewer when they have many parallel
 * branches; the oldest is evicted and destroyed once its last replay has finished; a burst of
 * more than 8 evictions whose replays are all still running makes the call wait for the oldest)
 * and replayed while the batch's pointers,
 * sizes, q_start_host contents, cut points and slots stay the same; the contents of device
 * arrays (positions, block table, activations, caches) may change between replays.
 * A schedule with a slot on a CU partition is never captured (see dyn_schedule.use_graph).
 * Cache placement: the attention launch of a layer streams that layer's K pool and V pool at the same
 * time, page by page, and its rate depends on which regions of HBM the two pools lie in (one
 * Llama-3-8B layer at batch 256, 2.3 GiB per pool, pools at multiples of 8 GiB inside one 224 GiB
 * allocation: 827-849, 857-885 or 940-957 us for the same launch, in blocks of 32 or 64 GiB that
 * follow the physical backing).  The library takes the pools where the caller puts them;
 * k_cache_layers / v_cache_layers let a caller place each layer after measuring. */
dyn_status dyn_layer_forward(dyn_layer *layer, const dyn_batch *batch, const dyn_schedule *sched, void *hip_stream);

/* For callers that cannot allocate device memory or create GPU objects at the point of the
 * call: code running under a HIP graph capture of their own, tight serving loops, harnesses
 * that forbid hipMalloc.  The same forward as dyn_layer_forward with the sequential schedule,
 * except that batch->workspace / workspace_bytes are ignored: the workspace is a static device
 * array inside the library (DYN_NOALLOC_MAX_WORKSPACE bytes, held by every GPU the library
 * runs on until the process ends).  All operators are issued in chain order on hip_stream;
 * no stream, event or graph is created, nothing is allocated or freed, by the library or
 * through any allocating routine.  (The array's device address is resolved once per device,
 * at the first call on it or by dyn_layer_prepare; that first resolution loads the library's
 * code object if no kernel of it has run yet.)
 *   DYN_ERR_WORKSPACE  the batch needs more than DYN_NOALLOC_MAX_WORKSPACE bytes
 *                      (dyn_layer_workspace_bytes tells): use dyn_layer_forward.
 * Every call on a GPU uses that GPU's one array, which keeps the previous call's contents
 * (nothing in it has to start at zero).  Calls that overlap in time on one GPU - from two
 * streams or two handles - race on it: keep them on one stream or order them with events. */
enum { DYN_NOALLOC_MAX_WORKSPACE = 96 << 20 };
dyn_status dyn_layer_forward_noalloc(dyn_layer *layer, const dyn_batch *batch, void *hip_stream);

/* Destroys every HIP graph the handle has captured (the cached ones and those evicted from the
 * cache whose last replay had not finished), after waiting for each one's last replay: BLOCKS
 * the host.  A schedule run with use_graph afterwards is captured again.  For callers that try
 * many schedules once each - the measured search of dyn_tune calls it after every candidate,
 * so that at most one multi-stream executable is alive while candidates are timed. */
dyn_status dyn_layer_release_graphs(dyn_layer *layer);

/* Profiling (eager schedules only): when on, every dispatch is bracketed by events on its
 * own stream.  After the caller has synchronised, dyn_layer_get_slot_times returns, for
 * the last forward, one record per dispatch in issue order (layer-major). */
typedef struct {
    int layer, op, nano, n_nano, stream, partition;
    float start_ms;            /* times relative to the fork point of that forward */
    float main_start_ms;       /* start and end of the operator's main kernel (the contraction, the attention */
    float main_stop_ms;        /* chunk kernel) where helper kernels surround it (work list, split-K reduce,
                                  split-KV combine); otherwise start_ms and stop_ms */
    float stop_ms;
} dyn_slot_time;
dyn_status dyn_layer_set_profiling(dyn_layer *layer, int on);
dyn_status dyn_layer_get_slot_times(dyn_layer *layer, dyn_slot_time *out, int capacity, int *n_out);

/* ---- Programmable scheduling (Section 3.2.2, Figure 6) -------------------------------
 *
 * The paper lets a strategy author write the schedule as a short program over three
 * calls: split the batch into micro-batches of chosen sizes, ask which operators of a
 * micro-batch are ready, and execute operators on a stream.  dyn_scheduler is that
 * interface as a recorder: the calls below check each step against the ready-operator
 * rule as it is made and append to a dyn_schedule that dyn_layer_forward then runs (and
 * replays as a HIP graph).  Host only; no GPU call, no device memory. */
typedef struct dyn_scheduler dyn_scheduler;

/* A recorder for batches of this token / sequence structure.  q_start_host as in dyn_batch
 * (copied).  The operator chain (dense or MoE) comes from cfg. */
dyn_status dyn_scheduler_create(const dyn_layer_config *cfg, int n_tokens, int n_seqs, const int32_t *q_start_host,
                                dyn_scheduler **out);
void dyn_scheduler_destroy(dyn_scheduler *s);

/* split([bs_1 .. bs_k]): micro-batch sizes in tokens, unequal sizes allowed, zero allowed;
 * they must add up to n_tokens and every cut must fall on a sequence boundary.  Discards
 * anything recorded before.  Without a split the batch is one micro-batch. */
dyn_status dyn_scheduler_split(dyn_scheduler *s, int k, const int32_t *sizes);

/* CU partitions that execute calls may name (1..n_partitions; 0 is the whole device). */
dyn_status dyn_scheduler_set_partitions(dyn_scheduler *s, int n_partitions, const uint32_t *cu_masks, int cu_mask_words);

/* get_ready_ops(i): the operators of micro-batch `nano` whose predecessors have been
 * executed and that have not been executed themselves.  Writes at most `capacity` operator
 * codes to ops and returns how many are ready (0: the micro-batch has finished the layer;
 * the layer's operators form a chain, so the answer is 0 or 1); -1 on a bad argument. */
int dyn_scheduler_get_ready_ops(const dyn_scheduler *s, int nano, uint8_t *ops, int capacity);

/* execute(ops, stream): n (operator, micro-batch) pairs.
 *   n = 1                                   split form: one micro-batch's operator.
 *   same operator, adjacent micro-batches   merge form: one dispatch over their joint rows.
 *   anything else                           no fused kernel exists for different operators:
 *                                           the sequential fallback, one dispatch per pair,
 *                                           in the order given, all on this stream.
 * Every pair must be ready (DYN_ERR_SCHEDULE otherwise, nothing recorded).  stream is
 * 0..DYN_MAX_STREAMS-1 within CU partition `partition`; stream 0 of partition 0 is the
 * stream the forward is called on. */
dyn_status dyn_scheduler_execute(dyn_scheduler *s, int n, const uint8_t *ops, const uint8_t *nanos, int stream,
                                 int partition);

/* Ends the recording: fails with DYN_ERR_SCHEDULE if some micro-batch has not finished
 * the chain.  *out borrows arrays owned by the scheduler: it stays valid until the next
 * split or destroy.  The recorded issue order is that of one layer and repeats per layer. */
dyn_status dyn_scheduler_finish(dyn_scheduler *s, int use_graph, dyn_schedule *out);

/* ---- Cost model and built-in policy (Section 2.1 "Splitting"; Section 5.3.1) ---------
 *
 * Splitting pays when a compute-bound operator of one micro-batch can run beside a
 * memory-bound operator of another, and costs a second read of the weights.  The policy
 * estimates every operator from its algorithmic bytes and FLOPs and this GPU's measured
 * rates, compares the sequential order with a two-micro-batch split at the boundary
 * between multi-token (prefill) and single-token (decode) sequences, and records the
 * winner through the scheduler calls above. */
typedef struct {
    int split;                   /* 0: sequential order chosen; 1: two micro-batches */
    int cut_row;                 /* rows [0, cut_row) | [cut_row, n_tokens) when split */
    float est_sequential_us;     /* model's estimate of one layer, sequential */
    float est_split_us;          /* model's estimate of one layer, split (0 if no legal cut) */
} dyn_policy_choice;

/* ctx_len_host[s] = keys sequence s attends including this step's tokens (HOST, n_seqs).
 * Records the chosen schedule into s (discarding earlier recordings) and fills *out;
 * choice may be NULL. */
dyn_status dyn_policy_auto(dyn_scheduler *s, const int32_t *ctx_len_host, int use_graph, dyn_schedule *out,
                           dyn_policy_choice *choice);

/* ---- Data flow and memory accounting (Section 3.3.1, Algorithm 1; Section 2.1 "Overlapping") -
 *
 * The paper's backend analyses the operator graph once: every intermediate tensor gets a
 * reference count (its out-degree) for lifetime management, and tensors that feed a merge
 * point are written straight into a preallocated buffer so that a change of the number of
 * micro-batches between producer and consumer costs no copy.  Here every intermediate lives
 * at its global row index in a batch-sized buffer of the workspace, so every split or merge
 * is in place by construction; this call is the static analysis for one schedule: it
 * derives, per (tensor, layer, micro-batch) region, the dispatches that read it (the
 * reference count) and its lifetime, and from those the peak of live intermediate bytes
 * next to what the workspace reserves.  Lifetimes follow issue order within a stream; a
 * region or a dispatch's scratch stays alive until the next dispatch on the stream of its
 * last user is issued, because dispatches issued on other streams meanwhile may run beside
 * it: overlap buffers the results of concurrently running micro-batches, which is the
 * peak-memory cost the paper names.  Host only. */
typedef struct {
    size_t workspace_bytes;             /* dyn_layer_workspace_bytes for this batch: enough for any schedule, nothing shared */
    size_t peak_live_bytes;             /* largest sum over live regions plus the running dispatch's scratch (split-K
                                           planes, split-KV partials and work lists, expert lists), this schedule */
    size_t peak_live_bytes_sequential;  /* the same for the sequential order */
    int peak_at_dispatch;               /* issue index (layer-major) at which the peak occurs */
    int n_regions;                      /* (tensor, layer, micro-batch) regions tracked */
    int max_ref_count;                  /* most dispatches reading one region */
    int n_resharded;                    /* regions written and read at different numbers of micro-batches (split form ->
                                           merge form or back): served in place, zero copies */
    size_t workspace_bytes_schedule;    /* dyn_schedule_workspace_bytes: what a forward with this schedule really needs */
} dyn_memory_report;

dyn_status dyn_schedule_memory(const dyn_layer *layer, const dyn_batch *batch, const dyn_schedule *sched,
                               dyn_memory_report *out);

/* The workspace one schedule needs for one batch shape (host only; 0 if the schedule is not
 * legal).  The backend knows every intermediate's producers and consumers (Section 3.3.1,
 * Algorithm 1), hence when its memory is free again: each intermediate tensor lives from its
 * first producer to the end of its last consumer over all micro-batches, a dispatch's scratch
 * (split-K planes, split-KV partials, expert lists) while that dispatch may run - both as the
 * streams allow: what a dispatch is the last to touch stays alive until the next dispatch on
 * its stream is issued - and regions that are never alive together share bytes (placed largest
 * first at the lowest free offset).  dyn_layer_forward lays the workspace out this way and
 * accepts any workspace of at least this size; the more micro-batches run side by side, the
 * less is shared (the peak-memory cost of overlapping, Section 2.1). */
size_t dyn_schedule_workspace_bytes(const dyn_layer *layer, const dyn_batch *batch, const dyn_schedule *sched);

/* The regions of that layout, for inspection and tests.  live_slots bit t = alive while slot t
 * of the layer's issue order (dyn_schedule.slots; the sequential order's chain) runs, in any
 * layer; stream = partition * DYN_MAX_STREAMS + stream of the dispatch a scratch region belongs
 * to, -1 for tensors.  Two regions never overlap in memory if their live_slots intersect, or if
 * they are scratch of dispatches on different streams (which may run at the same time whatever
 * the issue order).  With more than one stream every tensor is alive throughout.  Writes at most
 * capacity records, *n_out = number of regions. */
enum {
    DYN_REGION_H = 0,          /* RMSNorm outputs (both norms share it) */
    DYN_REGION_QKV = 1, DYN_REGION_ATTN = 2, DYN_REGION_X2 = 3,
    DYN_REGION_GU = 4,         /* [gate | up] when the SiLU gate is a kernel of its own */
    DYN_REGION_ACT = 5,
    DYN_REGION_ROUTING = 6,    /* MoE: selected experts and weights */
    DYN_REGION_XA = 7, DYN_REGION_XB = 8,   /* outputs of odd / even layers feeding the next layer */
    DYN_REGION_PLAN = 9,       /* attention work lists */
    DYN_REGION_PLANES = 10, DYN_REGION_PART_O = 11, DYN_REGION_PART_ML = 12, DYN_REGION_LISTS = 13,
    DYN_REGION_MOE_PLANES = 14,   /* scratch of one dispatch (slot >= 0) */
    DYN_REGION_KINDS = 15
};
typedef struct {
    int kind, slot;            /* slot = -1 for tensors */
    int stream;
    size_t offset, bytes;
    uint64_t live_slots[2];
} dyn_region;
dyn_status dyn_schedule_regions(const dyn_layer *layer, const dyn_batch *batch, const dyn_schedule *sched, dyn_region *out,
                                int capacity, int *n_out);

/* ---- Measured tuning of micro-batch sizes and CU partitions (Section 2.1; Section 5.3.4) -
 *
 * The paper names two things a strategy author has to tune by hand: the sizes of the
 * micro-batches (unequal sizes pay when operator durations differ) and the share of the
 * compute units each overlapped stream gets (hard to choose for partitioned contexts), and
 * reports a gain from choosing a kernel's share per batch size at run time.  The calls
 * below do that search by measurement: enumerate candidate schedules for a batch's
 * structure, record each through the scheduler calls above, time it on the device, and
 * keep the fastest. */
enum {
    DYN_FORM_SEQUENTIAL = 0,   /* one micro-batch, chain order, caller's stream */
    DYN_FORM_SPLIT = 1,        /* every operator per micro-batch, micro-batch b on stream b */
    DYN_FORM_MLP_MERGED = 2,   /* per micro-batch up to the second norm; router and MLP once for all (merge form) */
    DYN_FORM_ATTN_SPLIT = 3,   /* the four projections once for all; norms, rotary, attention, gate per micro-batch */
    DYN_FORM_MLP_SPLIT = 4     /* everything up to the second norm once for all, router and MLP per micro-batch:
                                  the shape of the dual-batch-overlap example (Section 3.2.2, Example 1) */
};

typedef struct {
    int k;                            /* micro-batches; 1 with DYN_FORM_SEQUENTIAL */
    int32_t rows[DYN_MAX_NANO + 1];   /* cut points rows[0] = 0 .. rows[k] = n_tokens */
    int form;                         /* DYN_FORM_* */
    int stagger;                      /* micro-batch b is issued `stagger` operators behind micro-batch b-1 */
    int cus_first;                    /* 0: plain streams.  Otherwise even micro-batches run on a partition of
                                         cus_first CUs and odd ones on the remaining CUs (the same share of
                                         every XCD); merged dispatches use the whole device */
    float us;                         /* filled by dyn_tune: time of one forward in a replay loop, microseconds;
                                         negative if the candidate could not be run */
} dyn_tune_candidate;

typedef struct {
    int max_k;          /* largest number of micro-batches enumerated, 2..4 (0 = 2) */
    int partitions;     /* CU-partition sizes tried: 0 none, 1 half | half, 2 adds 3/4 | 1/4, 3 adds 1/4 | 3/4 */
    int n_cus;          /* CUs of the device (0 = 256); dyn_tune overwrites it with the device's count */
    int warmup, iters;  /* per candidate: untimed forwards, then three timed runs of iters forwards issued
                           back to back, median of the three means (0 = 2 and 7) */
    int use_graph;      /* the use_graph field of the schedule dyn_tune records; candidates are timed with
                           eager launches either way (see dyn_tune) */
    float min_gain;     /* an overlapped candidate is chosen only if it beats the sequential order by this
                           fraction (negative = 0.02) */
} dyn_tune_options;

typedef struct {
    dyn_tune_candidate best;    /* the schedule recorded into the scheduler when dyn_tune returns */
    float us_sequential;
    int n_tried, n_skipped;     /* candidates timed / candidates the device refused (e.g. no masked stream) */
} dyn_tune_result;

/* Host only.  Writes the candidates for the scheduler's batch structure to table (at most
 * capacity) and returns how many there are (-1 on a bad argument): the sequential order;
 * for two micro-batches cuts near 1/4, 3/8, 1/2, 5/8 and 3/4 of the tokens snapped to
 * sequence boundaries, the cut that halves the summed context (ctx_len_host, HOST
 * [n_seqs], may be NULL) and the boundary between multi-token and single-token sequences
 * if there is exactly one, each in the four overlapped forms with staggers 1..2; equal
 * cuts for three and four micro-batches up to opt->max_k; CU-partitioned variants per
 * opt->partitions. */
int dyn_tune_candidates(const dyn_scheduler *s, const int32_t *ctx_len_host, const dyn_tune_options *opt,
                        dyn_tune_candidate *table, int capacity);

/* Host only.  Records candidate c into s (discarding earlier recordings, replacing its
 * partitions) and ends the recording into *out, as dyn_scheduler_finish does. */
dyn_status dyn_tune_record(dyn_scheduler *s, const dyn_tune_candidate *c, int n_cus, int use_graph, dyn_schedule *out);

/* Times every candidate on the batch (loops of eager forwards on hip_stream, each followed by
 * a wait for its end event: this call blocks, allocates no device memory, and leaves y and the
 * caches as one forward leaves them) and records the winner into s / *out with opt->use_graph.
 * s must have been created for this batch's structure.  table (may be NULL) receives the
 * candidates with their times, at most capacity of them.  The search captures no HIP graph:
 * one graph per candidate, destroyed after its replays, is a pattern under which long-lived
 * processes have died inside the HIP runtime here; eager timing includes the host's launch
 * cost, which weighs on candidates with more streams, so the search errs towards the
 * sequential order.  DYN_ERR_HIP if even the sequential order fails; DYN_ERR_INVALID_ARG for
 * opt->max_k outside 0..4. */
dyn_status dyn_tune(dyn_layer *layer, const dyn_batch *batch, const int32_t *ctx_len_host, const dyn_tune_options *opt,
                    void *hip_stream, dyn_scheduler *s, dyn_schedule *out, dyn_tune_result *result,
                    dyn_tune_candidate *table, int capacity);

/* ---- Measurement aid -----------------------------------------------------------------
 *
 * The layer's dominant operators are bound by HBM bandwidth (the memory-bound operator class
 * of Section 2), and a fraction of the datasheet peak says little without the rate the memory
 * system actually delivers.  This launches one read-only kernel that loads every 16-byte word
 * of buf[0 .. bytes) once (DEVICE pointer, 16-byte aligned, bytes a multiple of 16) and folds
 * them into sink (DEVICE, at least 32768 bytes, overwritten).  Asynchronous on hip_stream; the
 * caller times it with events.  Allocates nothing. */
dyn_status dyn_probe_hbm_read(const void *buf, size_t bytes, void *sink, void *hip_stream);

/* The same for the compute-bound operator class (Section 2): the many-row projections are priced
 * against the matrix cores' datasheet peak, and that figure assumes a clock the chip does not hold
 * under load.  This launches the main loop of the library's 256 x 256-tile projection kernel stripped
 * of its indexing - 256 workgroups of eight waves, per stage and wave 64 MFMA 16x16x32 bf16 with
 * their LDS operand reads, one barrier and the direct loads that refill the other stage buffer -
 * for n_stages stages (1 .. 2^20) on operands read from buf: DEVICE, 16-byte aligned, at least
 * 16 MiB (more is ignored), bf16 bit patterns of the caller's choosing - the rate depends on
 * them, zeros run about a third faster than random values.  sink: DEVICE, sink_bytes >= 524288,
 * overwritten.  *flops (HOST, may be NULL) receives the floating-point operations of the launch.
 * Asynchronous on hip_stream; the caller times it with events.  Allocates nothing. */
dyn_status dyn_probe_mfma_loop(const void *buf, size_t bytes, int n_stages, void *sink, size_t sink_bytes,
                               void *hip_stream, double *flops);

/* Thread-local description of the last error returned on this thread ("" if none). */
const char *dyn_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DYNLAYER_H */
