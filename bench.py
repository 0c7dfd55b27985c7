"""Benchmark of the decoder-layer forward step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5]

A step is one pass of the whole hot path (per layer: norms, projections, rotary + cache
append, paged attention, gated MLP) over one batch of seeded synthetic input that is resident
in HBM before the timed region.  The default workload is the largest configuration one GPU
holds: the 32-layer Llama-3-8B-shaped decode step at batch 256 with contexts uniform in
[1024, 8192] (c5), replayed as HIP graphs; c2, c3 and c4 are the single-layer workloads.  The
step is timed under the sequential schedule and under overlapped micro-batch schedules, every
step between two events on the stream the forward is called on; `value` is tokens / median
step time of the fastest schedule (the method falls back to the sequential order when
splitting does not pay), `config.schedule` names it, and per schedule the median, minimum,
maximum and the wall-clock mean over the K steps are reported beside it.  Prints one JSON line.
"""
import argparse
import dataclasses
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0

# HBM bytes per launch of the attention kernel, read with rocprofv3 counters (FETCH_SIZE and
# WRITE_SIZE in runs of their own, scaled by a 1 GiB copy probe).  Counters cannot be read
# from inside this process, so the figure of the committed counter summary is repeated here,
# together with the hash of the kernel's source it was measured on: if the source has changed
# since, the figure is withheld (traffic = null) instead of going stale silently.
ATTN_SOURCE = os.path.join(ROOT, "paper_2605_21603_amd", "csrc", "kernels_attn_mfma.hip")
ROCPROF_TRAFFIC = {
    "c2": {"bytes": 1272940954 + 21841510, "source_sha256_16": "1a36022dc5bf28f3", "kv_chunk_positions": 256,
           "source": "profiles/c2_sequential_attn_mfma_kernel.md (FETCH_SIZE 621,553.2 x 2.0 KiB + WRITE_SIZE 21,329.6 KiB)"},
    "c5": {"bytes": 5050486784 + 22979686, "source_sha256_16": "1a36022dc5bf28f3", "kv_chunk_positions": 1024,
           "source": "profiles/c5_sequential_32_layer_decode.md (FETCH_SIZE 2,466,058.0 x 2.0 KiB + WRITE_SIZE 22,441.1 KiB)"},
}


def source_hash(path):
    with open(path, "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()[:16]


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def candidate_schedules(B, w, use_graph):
    rows = w.nano_rows
    chain = B.MOE_CHAIN if w.shape.n_experts else B.DENSE_CHAIN
    mlp = [B.DYN_OP_GATE_UP, B.DYN_OP_SILU, B.DYN_OP_DOWN]
    gemms = [B.DYN_OP_QKV, B.DYN_OP_OPROJ, B.DYN_OP_GATE_UP, B.DYN_OP_DOWN]
    if w.shape.n_layers > 1:
        # the many-layer step: two and four micro-batches, plain and CU-partitioned streams
        lo, hi = [0x0000FFFF] * 8, [0xFFFF0000] * 8
        T = w.n_tokens
        r4 = tuple(T * i // 4 for i in range(5))
        return {
            "k2_mlp_merged_stagger2": B.nano_schedule(rows, chain, merged_ops=mlp, stagger=2, use_graph=use_graph),
            "k2_split_stagger2_cu_partitioned": B.nano_schedule(rows, chain, stagger=2, partitions=[1, 2], cu_masks=[lo, hi],
                                                                use_graph=use_graph),
            "k4_mlp_merged_stagger1_cu_partitioned": B.nano_schedule(r4, chain, merged_ops=mlp, stagger=1,
                                                                     partitions=[1, 2, 1, 2], streams=[0, 1, 2, 3],
                                                                     cu_masks=[lo, hi], use_graph=use_graph),
        }
    return {
        "k2_split_stagger0": B.nano_schedule(rows, chain, stagger=0, use_graph=use_graph),
        "k2_split_stagger2": B.nano_schedule(rows, chain, stagger=2, use_graph=use_graph),
        "k2_mlp_merged_stagger2": B.nano_schedule(rows, chain, merged_ops=mlp, stagger=2, use_graph=use_graph),
        "k2_gemms_merged_stagger1": B.nano_schedule(rows, chain, merged_ops=gemms, stagger=1, use_graph=use_graph),
    }


def time_schedule(layer, step, sched, stream, steps, warmup):
    """W untimed forwards, then K forwards issued back to back, each between two events recorded
    on the stream the forward is called on (the end event of one step is the start event of the
    next), the whole loop between two device synchronisations.  Per-step times in ms."""
    import torch
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    with torch.cuda.stream(stream):
        for _ in range(warmup):
            layer.forward(step.batch, sched, stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        evs[0].record(stream)
        for i in range(steps):
            layer.forward(step.batch, sched, stream)
            evs[i + 1].record(stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    per = [evs[i].elapsed_time(evs[i + 1]) for i in range(steps)]
    return {"median_ms": statistics.median(per), "min_ms": min(per), "max_ms": max(per), "mean_ms": sum(per) / steps,
            "wall_mean_ms": (t1 - t0) * 1e3 / steps, "slowest_step": per.index(max(per))}


def measure_stream_read(B, buf, stream, reps=7):
    """GB/s of the library's read-only streaming kernel over up to 2 GiB of a resident buffer."""
    import torch
    nbytes = min(buf.numel() * buf.element_size(), 2 << 30) & ~15
    sink = torch.empty(8192, dtype=torch.int32, device=buf.device)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    with torch.cuda.stream(stream):
        B.probe_hbm_read(buf, nbytes, sink, stream)
        evs[0].record(stream)
        for i in range(reps):
            B.probe_hbm_read(buf, nbytes, sink, stream)
            evs[i + 1].record(stream)
    torch.cuda.synchronize()
    ms = statistics.median(evs[i].elapsed_time(evs[i + 1]) for i in range(reps))
    return {"GB/s": nbytes / 1e9 / (ms * 1e-3), "bytes": nbytes, "median_ms": ms,
            "kernel": "stream_read_kernel (16-byte loads, read only, 2048 x 256 threads, grid-strided)"}


def measure_mfma_loop(B, device, stream, n_stages=4096, reps=3):
    """TFLOP/s of the library's matrix-core probe (the wide projection tile's main loop on L2-resident operands) with
    random bf16 operands N(0, 1) - what the projections work on - and with zeros."""
    import torch
    sink = torch.empty(256 * 512, dtype=torch.float32, device=device)
    gen_ = torch.Generator(device=device)
    gen_.manual_seed(1234)
    out = {}
    for name, buf in (("random_operands", torch.randn(8 << 20, dtype=torch.float32, device=device, generator=gen_).to(torch.bfloat16)),
                      ("zero_operands", torch.zeros(8 << 20, dtype=torch.bfloat16, device=device))):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        with torch.cuda.stream(stream):
            flops = B.probe_mfma_loop(buf, n_stages, sink, stream)
            evs[0].record(stream)
            for i in range(reps):
                B.probe_mfma_loop(buf, n_stages, sink, stream)
                evs[i + 1].record(stream)
        torch.cuda.synchronize()
        ms = statistics.median(evs[i].elapsed_time(evs[i + 1]) for i in range(reps))
        out[name] = {"TFLOP/s": flops / 1e12 / (ms * 1e-3), "median_ms": ms}
    out["kernel"] = ("mfma_loop_probe_kernel (256 workgroups x 8 waves, %d stages of 64 MFMA 16x16x32 bf16 per wave with LDS operand "
                     "reads, a barrier and 64 KB of direct loads per stage)" % n_stages)
    return out


def attention_bytes(w):
    """Algorithmic HBM bytes of one attention launch: every cached position of every kv head
    read once, K and V (4096 B per position for the Llama-3-8B shape), plus q in and o out."""
    sh = w.shape
    e = 2 if sh.dtype == "bf16" else 4
    kv = sum(c for _, c in w.seqs)          # a prefill chunk's keys are also read once, not once per query
    return kv * 2 * sh.n_kv * sh.head_dim * e + 2 * w.n_tokens * sh.n_q * sh.head_dim * e


def gate_up_bytes_flops(w):
    """Algorithmic bytes and flops of one gate/up projection launch (the largest projection):
    weights once (every expert's in the MoE layer), activations in, gated output out."""
    sh = w.shape
    e = 2 if sh.dtype == "bf16" else 4
    rows = w.n_tokens * (sh.top_k if sh.n_experts else 1)
    byts = 2 * sh.inter * sh.hidden * e * max(1, sh.n_experts) + w.n_tokens * sh.hidden * e + rows * sh.inter * e
    return byts, 2 * rows * sh.hidden * 2 * sh.inter


def layer_bytes_flops(w):
    sh = w.shape
    e = 2 if sh.dtype == "bf16" else 4
    attn_params = sh.qkv_rows * sh.hidden + sh.hidden * sh.n_q * sh.head_dim
    mlp_params = 3 * sh.inter * sh.hidden
    T = w.n_tokens
    pairs = sh.top_k if sh.n_experts else 1
    act = T * e * (2 * sh.hidden * 4 + 2 * sh.qkv_rows + 2 * sh.n_q * sh.head_dim + pairs * 3 * 2 * sh.inter)
    kv_pos = sum((2 * c - q + 1) * q // 2 for q, c in w.seqs)           # (query, key) pairs
    byts = (attn_params + mlp_params * max(1, sh.n_experts)) * e + attention_bytes(w) + act   # every expert is read once
    flops = 2 * (attn_params + mlp_params * pairs) * T + 4 * sh.n_q * sh.head_dim * kv_pos
    return byts * sh.n_layers, flops * sh.n_layers


def cpu_baseline(w, data, n_sample=128):
    """The oracle, as it is, on a sample of the workload's sequences (rows are independent
    per sequence), timed around the compute only."""
    import numpy as np
    from oracle import oracle as orc
    from workloads import gen
    ctx = [c for _, c in w.seqs]
    order = np.argsort(ctx)
    picks = sorted({int(order[0]), int(order[-1])} | {int(i) for i in order[:: max(1, len(order) // n_sample)][:n_sample]})
    if data["x"].device.type == "cpu":
        w2, d2 = gen.sub_batch(w, data, picks)
    else:                                   # generated in device memory: copy the sampled sequences out
        w2, d2 = gen.extract_sequences(w, data, picks)
    sh = w.shape
    dt = orc.dtype_code(sh.dtype)
    x = orc.widen(orc.to_storage(d2["x"]), dt)
    prepared = []
    for l in range(sh.n_layers):
        prepared.append(({k: orc.to_storage(v) for k, v in d2["weights"][l].items()},
                         orc.to_storage(d2["k_cache"][l]).copy(), orc.to_storage(d2["v_cache"][l]).copy()))
    t0 = time.perf_counter()
    for wts, kc, vc in prepared:
        x = orc.layer_forward(sh, wts, x, d2["seq_of_token"], d2["pos_of_token"], d2["block_table"], kc, vc)
    dt_s = time.perf_counter() - t0
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": w2.n_tokens / dt_s, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": "%d of %d sequences (incl. shortest and longest context), all layers, %.1f s wall"
                      % (len(picks), w.n_seqs, dt_s)}


def prefill_decode_mix(B, gen, stream, steps, warmup, prefill=512, decodes=64, ctx=2048):
    """Where the method's premise holds on this GPU: a chunked-prefill step - one prefill chunk of a few hundred tokens
    beside decode sequences (Section 2.1 "Splitting", Section 5.3.1) - under the sequential order and under the
    library's own policy (which records a two-micro-batch split at the prefill / decode boundary when its cost model
    predicts a gain), one Llama-3-8B-shaped layer, HIP-graph replays, medians of per-step event times."""
    import torch
    w = gen.mixed(prefill, decodes, ctx)
    data = gen.generate(w, device="cuda:0")
    layer = B.DynLayer(B.make_config(w.shape), data["weights"])
    step = B.DeviceStep(layer, data)
    md = gen.metadata(w)
    sched, choice = B.Scheduler(B.make_config(w.shape), md["q_start"]).auto(md["ctx_len"], use_graph=True)
    t_seq = time_schedule(layer, step, B.sequential(use_graph=True), stream, steps, warmup)
    out = {"workload": "%s: %d-token prefill chunk + %d decodes at context %d, 1 layer" % (w.name, prefill, decodes, ctx),
           "tokens": w.n_tokens, "sequential_ms": t_seq["median_ms"], "policy_choice": "split" if choice["split"] else "sequential",
           "policy_est_sequential_us": choice["est_sequential_us"], "policy_est_split_us": choice["est_split_us"]}
    if choice["split"]:
        t_pol = time_schedule(layer, step, sched, stream, steps, warmup)
        y_split = step.y.clone()
        layer.forward(step.batch, B.sequential(use_graph=True), stream)
        torch.cuda.synchronize()
        out.update({"policy_ms": t_pol["median_ms"], "policy_stats_ms": t_pol, "speedup_over_sequential": t_seq["median_ms"] / t_pol["median_ms"],
                    "tokens_per_s_sequential": w.n_tokens / (t_seq["median_ms"] * 1e-3), "tokens_per_s_policy": w.n_tokens / (t_pol["median_ms"] * 1e-3),
                    "bit_identical_to_sequential": bool(torch.equal(y_split.view(torch.uint8), step.y.view(torch.uint8)))})
    del step, layer, data
    torch.cuda.empty_cache()
    return out


def policy_sweep(args):
    """Where splitting starts to pay: a prefill chunk of P tokens beside D decode sequences at
    context C, Llama-3-8B layer.  For every point: measured sequential and split (two
    streams, round-robin issue; HIP-graph replays), the cost model's two estimates and the
    policy's choice.  Prints one JSON object with the table."""
    import torch
    from paper_2605_21603_amd import binding as B
    from workloads import gen
    rows, weights, layer = [], None, None
    stream = torch.cuda.Stream()
    # "fit": the grid the policy's three overlap constants were fitted on; "holdout": points between and beside them
    grid = {"fit": ((256, 512, 1024, 2048, 4096), ((64, 2048), (64, 8192), (256, 2048), (256, 8192))),
            "holdout": ((384, 768, 1536, 3072), ((32, 4096), (128, 1024), (128, 4096), (192, 8192)))}[args.sweep_grid]
    for P in grid[0]:
        for D, Cx in grid[1]:
            w = gen.mixed(P, D, Cx)
            data = gen.generate(w, device="cuda:0")
            if layer is None:                       # the same layer weights serve every point
                weights = data["weights"]
                layer = B.DynLayer(B.make_config(w.shape), weights)
            data["weights"] = weights
            step = B.DeviceStep(layer, data)
            md = gen.metadata(w)
            sch = B.Scheduler(B.make_config(w.shape), md["q_start"])
            _, choice = sch.auto(md["ctx_len"], use_graph=True)
            sch.split([P, D])
            while sch.get_ready_ops(0) or sch.get_ready_ops(1):
                for b in range(2):
                    r = sch.get_ready_ops(b)
                    if r:
                        sch.execute([(r[0], b)], stream=b)
            split = sch.finish(use_graph=True)
            t_seq = time_schedule(layer, step, B.sequential(use_graph=True), stream, args.steps, args.warmup)["median_ms"]
            t_split = time_schedule(layer, step, split, stream, args.steps, args.warmup)["median_ms"]
            rows.append({"prefill_tokens": P, "decodes": D, "decode_ctx": Cx, "sequential_us": t_seq * 1e3,
                         "split_us": t_split * 1e3, "est_sequential_us": choice["est_sequential_us"],
                         "est_split_us": choice["est_split_us"], "policy_split": choice["split"],
                         "split_is_faster": t_split < t_seq})
            log("P=%4d D=%3d ctx=%4d  sequential %7.1f us (model %7.1f)  split %7.1f us (model %7.1f)  policy: %s  measured: %s"
                % (P, D, Cx, t_seq * 1e3, choice["est_sequential_us"], t_split * 1e3, choice["est_split_us"],
                   "split" if choice["split"] else "sequential", "split" if t_split < t_seq else "sequential"))
            del step, data
            torch.cuda.empty_cache()
    agree = sum(r["policy_split"] == r["split_is_faster"] for r in rows)
    regret = [min(r["sequential_us"], r["split_us"]) / (r["split_us"] if r["policy_split"] else r["sequential_us"]) for r in rows]
    print(json.dumps({"grid": args.sweep_grid, "policy_sweep": rows, "policy_agrees_with_measurement": "%d of %d" % (agree, len(rows)),
                      "worst_policy_efficiency": min(regret)}), flush=True)


def trace_overlap(db_path):
    """Timeline overlap fraction from a rocprofv3 --kernel-trace result database: inside the
    window in which the library's kernels ran on more than one queue (the overlapped
    schedules of this run), the share of time with at least two of its kernels resident.
    Kernels of one stream never overlap, so two resident kernels belong to different
    micro-batches (or to a merged dispatch beside a split one).  Prints one JSON object."""
    import sqlite3
    cur = sqlite3.connect(db_path).cursor()
    rows = cur.execute("select start, end, queue_id, stream_id from kernels where name like '%dyn::%' order by start").fetchall()
    if not rows:
        sys.exit("bench.py: no dyn:: kernels in %s" % db_path)
    lanes = {}
    for st, en, q, sid in rows:
        lanes.setdefault((q, sid), []).append((st, en))
    main_lane = max(lanes, key=lambda k: len(lanes[k]))
    side = [iv for k, v in lanes.items() if k != main_lane for iv in v]
    out = {"kernels": len(rows), "queues": len(lanes)}
    if side:
        w0, w1 = min(a for a, _ in side), max(b for _, b in side)
        # forwards alternate main-only and forked phases: widen the window to whole forwards is not
        # needed, the fraction is taken over first side-stream start .. last side-stream end
        events = []
        for st, en, q, sid in rows:
            a, b = max(st, w0), min(en, w1)
            if b > a:
                events += [(a, 1), (b, -1)]
        events.sort()
        depth, last, busy, ovl = 0, w0, 0, 0
        for t, d in events:
            if depth >= 1:
                busy += t - last
            if depth >= 2:
                ovl += t - last
            depth += d
            last = t
        out.update({"window_ms": (w1 - w0) * 1e-6, "busy_ms": busy * 1e-6, "overlapped_ms": ovl * 1e-6,
                    "overlap_fraction_of_window": ovl / (w1 - w0), "overlap_fraction_of_busy": ovl / busy})
    else:
        out.update({"window_ms": 0.0, "overlap_fraction_of_window": 0.0})
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c5", help="c5 (default: the largest configuration), c2, c3, c4")
    ap.add_argument("--no-graph", action="store_true", help="eager launches instead of HIP-graph replay")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--schedules", default="all",
                    help="comma-separated overlapped schedules to time beside sequential ('all', or 'none')")
    ap.add_argument("--tune", action="store_true",
                    help="also run the library's measured search over micro-batch sizes, forms and CU shares and time its choice")
    ap.add_argument("--no-event-profile", action="store_true", help="skip the per-operator HIP-event pass")
    ap.add_argument("--no-mix", action="store_true", help="skip the chunked-prefill + decode step timed beside the main workload")
    ap.add_argument("--kv-placement", default="measured", choices=["measured", "stacked"],
                    help="measured: one large arena, the attention launch timed with the K and V pools at pairs of arena chunks, "
                         "every layer's pools at the fastest pair with room; stacked: one tensor per cache, layers back to back")
    ap.add_argument("--arena-gib", type=int, default=224, help="--kv-placement measured: size of the arena (chunks of 16 GiB)")
    ap.add_argument("--placement-map", action="store_true",
                    help="only print the attention launch time of the workload's first layer for every pair of arena chunks "
                         "(K pool at the row's chunk, V pool at the column's; same chunk: V right behind K)")
    ap.add_argument("--kv-chunk", default="rule",
                    help="split-KV chunk of decode attention in positions (kv_chunk_positions of the configuration): a number; "
                         "'rule' (default): 1024 when the batch has at least eight decode work items per persistent wave at 256, "
                         "else 256; 'auto': the whole attention dispatch of the first layer timed with 256, 1024 and 2048 and the fastest taken")
    ap.add_argument("--policy-sweep", action="store_true",
                    help="sequential vs split over a grid of prefill / decode mixes, beside the policy's estimates")
    ap.add_argument("--sweep-grid", default="fit", choices=["fit", "holdout"],
                    help="--policy-sweep: the grid the policy's constants were fitted on, or a held-out one")
    ap.add_argument("--copy-probe", action="store_true",
                    help="only copy 1 GiB device-to-device five times (calibrates rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--trace-overlap", metavar="DB",
                    help="only read a rocprofv3 --kernel-trace result database and print the timeline overlap fraction")
    args = ap.parse_args()
    if args.trace_overlap:
        return trace_overlap(args.trace_overlap)
    if args.policy_sweep:
        if args.gpus != 1:
            sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")
        return policy_sweep(args)
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import torch
    from paper_2605_21603_amd import binding as B
    from workloads import gen

    if args.copy_probe:
        a = torch.full((1 << 30,), 7, dtype=torch.uint8, device="cuda:0")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        for _ in range(5):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read": 1 << 30, "copy_probe_bytes_written": 1 << 30, "copies": 5}))
        return

    w = gen.config(args.workload)
    stream = torch.cuda.Stream()
    # The arena comes first, while the device memory is still in large free blocks.
    arena, placement = None, None
    if args.kv_placement == "measured" and w.shape.dtype == "bf16":
        from paper_2605_21603_amd import placement as P
        try:
            # room for the weights and everything else must remain: shrink the arena if the device has less free memory
            # than it usually has (the pools need 2 slots per layer; a 16 GiB chunk holds a whole number of them)
            sh = w.shape
            e = 2
            wbytes = sh.n_layers * e * (sh.qkv_rows * sh.hidden + sh.hidden * sh.n_q * sh.head_dim + 3 * sh.inter * sh.hidden * max(1, sh.n_experts))
            free_b, _ = torch.cuda.mem_get_info()
            n_chunks = min(args.arena_gib // 16, int((free_b - wbytes - 12 * P.GiB) // (16 * P.GiB)))
            md0 = gen.metadata(w)
            pool = md0["n_pages"] * sh.n_kv * sh.page_size * sh.head_dim * e
            slots = n_chunks * ((14 * P.GiB) // max(pool, 1)) if n_chunks > 0 else 0      # 2 GiB per chunk kept for a workspace
            if n_chunks < 2 or slots < 2 * sh.n_layers:
                raise RuntimeError("%.0f GiB free" % (free_b / P.GiB))
            if n_chunks < args.arena_gib // 16:
                log("arena reduced to %d GiB (%.0f GiB free)" % (16 * n_chunks, free_b / P.GiB))
            arena = P.Arena(n_chunks, 16 * P.GiB)
            arena.fill_random()
        except RuntimeError as e:           # not enough free memory for the arena: the plain layout
            log("no %d GiB arena (%s): stacked caches" % (args.arena_gib, str(e).splitlines()[0]))
            arena = None
            torch.cuda.empty_cache()

    if args.kv_chunk == "rule":
        from paper_2605_21603_amd import placement as P0
        kv_chunk = P0.rule_chunk([c for _, c in w.seqs], [q for q, _ in w.seqs], w.shape.n_kv) if w.shape.dtype == "bf16" else 0
    else:
        kv_chunk = 0 if args.kv_chunk == "auto" else int(args.kv_chunk)
    chunk_us = None

    ws_tensor = None

    def workspace_bytes(so_far):
        sizing = B.DynLayer(B.make_config(w.shape, 256), [{k: v.to("cuda:0") for k, v in lw.items()} for lw in so_far["weights"]])
        md_ = gen.metadata(w)
        # the smallest chunk any --kv-chunk choice uses has the most chunks and the largest partial arrays
        n = sizing.workspace_bytes(w.n_tokens, int(md_["max_pages_per_seq"])) + 512
        sizing.close()
        return n

    def the_workspace(so_far):
        """One workspace buffer for the probes and for the timed step: the attention kernel writes its split-KV partials
        there and the projections their split-K planes, and where those streams lie moves the launches like the pools'
        places do.  (Inside the arena when there is one: place() picks the chunk.)"""
        nonlocal ws_tensor
        if ws_tensor is None:
            ws_tensor = torch.empty(workspace_bytes(so_far), dtype=torch.uint8, device="cuda:0")
        return ws_tensor

    def place(so_far, k_shape, v_shape):
        """Times the first layer's attention launch on this step with the pools at pairs of arena
        chunks and hands out every layer's pools accordingly."""
        nonlocal placement
        dt = w.shape.torch_dtype
        w0 = [{k: v.to("cuda:0") for k, v in so_far["weights"][0].items()}]
        layer1 = B.DynLayer(B.make_config(dataclasses.replace(w.shape, n_layers=1), kv_chunk), w0)
        # the workspace first: the end of the chunk where everything but attention runs fastest (the weights stay where they are)
        nonlocal ws_tensor
        ws_bytes = workspace_bytes(so_far)
        arena.reserved_tail = (ws_bytes + 4095) & ~4095
        ws_us = P.measure_workspace(layer1, so_far, arena, k_shape, v_shape, dt, ws_bytes, stream)
        ws_chunk = min(ws_us, key=lambda c: ws_us[c])
        ws_tensor = P.workspace_view(arena, ws_chunk, ws_bytes)
        log("workspace: the step without attention takes %.1f .. %.1f us by the workspace's chunk -> chunk %d" % (min(ws_us.values()), max(ws_us.values()), ws_chunk))
        times = P.measure_pairs(layer1, so_far, arena, k_shape, v_shape, dt, stream, workspace=the_workspace(so_far))
        del layer1
        if args.placement_map:
            n = arena.n_chunks
            print("attention launch time in us, workload %s, split-KV chunk %d positions; arena of %d chunks of 16 GiB; rows: chunk of the K pool, "
                  "columns: chunk of the V pool" % (w.name, kv_chunk or 256, n))
            print("      " + " ".join("%5d" % j for j in range(n)))
            for i in range(n):
                print("K %3d " % i + " ".join("%5.0f" % times[(i, j)] if j >= i else "     " for j in range(n)))
            sys.stdout.flush()
            os._exit(0)
        plan = P.assign(times, w.shape.n_layers, (arena.chunk_bytes - arena.reserved_tail) // P.slot_bytes_of(k_shape, dt), arena.n_chunks)
        placement = dict(P.summary(times, plan), arena_GiB=arena.buf.numel() / P.GiB, chunk_GiB=16, workspace_chunk=ws_chunk,
                         non_attention_us_by_workspace_chunk=[ws_us[c] for c in range(arena.n_chunks)])
        log("cache placement: attention probe %.1f us fastest / %.1f median / %.1f slowest pair of chunks; chosen mean %.1f, worst %.1f"
            % (placement["probe_us_fastest"], placement["probe_us_median"], placement["probe_us_slowest"],
               placement["chosen_us_mean"], placement["chosen_us_worst"]))
        ks, vs = P.place_layers(arena, plan, k_shape, v_shape, dt)
        pick_chunk(so_far, ks[0], vs[0])
        return ks, vs


    def pick_chunk(so_far, k0, v0):
        """--kv-chunk auto: the first layer's attention dispatch on this step, pools where they will be, per candidate."""
        nonlocal kv_chunk, chunk_us
        if args.kv_chunk != "auto" or w.shape.dtype != "bf16":
            return
        from paper_2605_21603_amd import placement as P
        w0 = [{k: v.to("cuda:0") for k, v in so_far["weights"][0].items()}]
        sh1 = dataclasses.replace(w.shape, n_layers=1)
        kv_chunk, chunk_us = P.choose_chunk(lambda c: B.DynLayer(B.make_config(sh1, c), w0), so_far, k0, v0, (256, 1024, 2048), stream,
                                            workspace=the_workspace(so_far))
        log("split-KV chunk: attention dispatch %s us -> %d positions"
            % (", ".join("%d: %.1f" % (c, t) for c, t in chunk_us.items()), kv_chunk))

    log("generating %s (seed %d) ..." % (w.name, w.seed))
    host_data = None                        # the step as generated on the host, where it was
    if w.shape.n_layers > 1:                # caches beyond host memory: drawn directly in device memory
        data = gen.generate(w, device="cuda:0", stacked=True, place=place if arena is not None else None)
        torch.cuda.synchronize()
        log("generated in device memory: %.1f GB allocated" % (torch.cuda.memory_allocated() / 1e9))
    else:
        data = gen.generate(w)
        if arena is not None:               # generated on the host: copy every layer's pools to their places
            host_k, host_v = data["k_cache"], data["v_cache"]
            dev = dict(data, weights=[{k: v.to("cuda:0") for k, v in lw.items()} for lw in data["weights"]])
            ks, vs = place(dev, tuple(host_k[0].shape), tuple(host_v[0].shape))
            for l in range(w.shape.n_layers):
                ks[l].copy_(host_k[l])
                vs[l].copy_(host_v[l])
            host_data, data = data, dict(data, k_cache=ks, v_cache=vs)
    weights = [{k: v.to("cuda:0") for k, v in lw.items()} for lw in data["weights"]]
    if arena is None:                       # stacked caches: the chunk is chosen on layer 0's pools where they are
        k0 = data["k_cache"][0] if data["x"].is_cuda else data["k_cache"][0].to("cuda:0")
        v0 = data["v_cache"][0] if data["x"].is_cuda else data["v_cache"][0].to("cuda:0")
        pick_chunk(dict(data, weights=weights), k0, v0)
        del k0, v0
    layer = B.DynLayer(B.make_config(w.shape, kv_chunk), weights)
    step = B.DeviceStep(layer, data, placed=arena is not None, workspace=the_workspace(dict(data, weights=weights)))
    use_graph = not args.no_graph

    stats = {}
    seq = B.sequential(use_graph=use_graph)
    cands = candidate_schedules(B, w, use_graph)
    if args.schedules != "all":
        cands = {k: v for k, v in cands.items() if k in args.schedules.split(",")}
    for sched in cands.values():            # side streams (CU-masked ones synchronise the device) exist before anything is timed
        layer.prepare(sched)
    stats["sequential"] = time_schedule(layer, step, seq, stream, args.steps, args.warmup)
    for name, sched in cands.items():
        stats[name] = time_schedule(layer, step, sched, stream, args.steps, args.warmup)
    for name, r in stats.items():
        log("%s: median %.1f us/step (min %.1f, max %.1f at step %d, wall mean %.1f)"
            % (name, r["median_ms"] * 1e3, r["min_ms"] * 1e3, r["max_ms"] * 1e3, r["slowest_step"], r["wall_mean_ms"] * 1e3))
    results = {k: r["median_ms"] for k, r in stats.items()}
    stream_read = measure_stream_read(B, step.k_cache, stream)
    log("streaming read of resident cache: %.0f GB/s" % stream_read["GB/s"])
    mfma_loop = measure_mfma_loop(B, step.k_cache.device, stream) if w.shape.dtype == "bf16" else None
    if mfma_loop:
        log("matrix-core loop probe: %.0f TFLOP/s on random operands, %.0f on zeros"
            % (mfma_loop["random_operands"]["TFLOP/s"], mfma_loop["zero_operands"]["TFLOP/s"]))
    # the library's measured tuner: unequal micro-batch sizes, forms, staggers, CU shares
    md = gen.metadata(w)
    tuned = None
    if args.tune:
        log("tuning ...")
        many = w.shape.n_layers > 1
        sch_t = B.Scheduler(B.make_config(w.shape), md["q_start"])
        t_sched, t_res, t_table = sch_t.tune(layer, step.batch, stream, ctx_len=md["ctx_len"], max_k=2, partitions=1,
                                             warmup=1 if many else 2, iters=3 if many else 7, use_graph=use_graph)
        torch.cuda.synchronize()
        t_overlapped = [c for c in t_table if c["us"] > 0 and c["form"] != "sequential"]
        t_fastest = min(t_overlapped, key=lambda c: c["us"]) if t_overlapped else None
        tuned = {"chosen": t_res["best"], "fastest_overlapped": t_fastest, "us_sequential": t_res["us_sequential"],
                 "candidates_timed": t_res["n_tried"], "candidates_refused": t_res["n_skipped"]}
        log("tuner: chose %s; fastest overlapped candidate %s; sequential %.1f us" % (t_res["best"], t_fastest,
                                                                                      t_res["us_sequential"]))
        if t_res["best"]["form"] != "sequential":
            stats["tuned"] = time_schedule(layer, step, t_sched, stream, args.steps, args.warmup)
            results["tuned"] = stats["tuned"]["median_ms"]
            log("tuned: %.1f us/step" % (results["tuned"] * 1e3))
    # what the library's own policy would run for this batch, and its cost estimates
    _, policy = B.Scheduler(B.make_config(w.shape), md["q_start"]).auto(md["ctx_len"], use_graph=use_graph)
    best_ovl = min((k for k in results if k != "sequential" or len(results) == 1), key=lambda k: results[k])
    best = min(results, key=lambda k: results[k])

    # Dominant kernel (paged attention): average launch duration from HIP events recorded on
    # its own stream around the kernel, over `steps` eager sequential forwards.
    layer.set_profiling(True)
    eager = B.sequential(use_graph=False)
    attn_ms, gu_ms, op_ms = [], [], {}
    with torch.cuda.stream(stream):
        n_prof = min(args.steps, 20 if w.shape.n_layers > 1 else 200)
        for i in range(0 if args.no_event_profile else n_prof + 5):
            layer.forward(step.batch, eager, stream)
            torch.cuda.synchronize()
            if i < 5:
                continue
            for rec in layer.slot_times():
                op_ms.setdefault(B.OP_NAMES[rec["op"]], []).append(rec["stop_ms"] - rec["start_ms"])
                if rec["op"] == B.DYN_OP_ATTN:
                    attn_ms.append(rec["main_stop_ms"] - rec["main_start_ms"])
                if rec["op"] == B.DYN_OP_GATE_UP:
                    gu_ms.append(rec["main_stop_ms"] - rec["main_start_ms"])
    layer.set_profiling(False)
    attn_avg_ms = sum(attn_ms) / len(attn_ms) if attn_ms else float("nan")
    attn_gb = attention_bytes(w) / 1e9
    achieved = attn_gb / (attn_avg_ms * 1e-3)
    roofline = {"bound": "hbm", "kernel": "attn_mfma_kernel", "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "bytes_per_launch": attention_bytes(w),
                "avg_launch_ms": attn_avg_ms}
    # Where the gate/up projection outlasts attention (the prefill mix, the MoE layer) it is the
    # dominant kernel: priced against the matrix cores or the weight stream, whichever bounds it.
    gu_avg_ms = sum(gu_ms) / len(gu_ms) if gu_ms else float("nan")
    if gu_ms and w.shape.dtype == "bf16" and gu_avg_ms > attn_avg_ms:
        gb, gf = gate_up_bytes_flops(w)
        if gf / (MFMA_BF16_PEAK_TFLOPS * 1e12) > gb / (HBM_PEAK_GBS * 1e9):
            a = gf / 1e12 / (gu_avg_ms * 1e-3)
            roofline = {"bound": "mfma", "kernel": "gemm_bf16_kernel (gate/up, SiLU gate in the epilogue)", "achieved": a,
                        "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": a / MFMA_BF16_PEAK_TFLOPS,
                        "flops_per_launch": gf, "avg_launch_ms": gu_avg_ms}
        else:
            a = gb / 1e9 / (gu_avg_ms * 1e-3)
            roofline = {"bound": "hbm", "kernel": "gemm_bf16_kernel (gate/up, SiLU gate in the epilogue)", "achieved": a,
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": a / HBM_PEAK_GBS, "bytes_per_launch": gb,
                        "avg_launch_ms": gu_avg_ms}

    traffic = ROCPROF_TRAFFIC.get(w.name)
    if traffic and traffic["kv_chunk_positions"] != (kv_chunk or 256):
        log("the committed counters were read with another split-KV chunk size: traffic withheld")
        traffic = None
    if traffic and traffic["source_sha256_16"] != source_hash(ATTN_SOURCE):
        log("the attention kernel's source changed since its counters were read: traffic withheld")
        traffic = None
    byts, flops = layer_bytes_flops(w)
    t_roof_ms = max(byts / (HBM_PEAK_GBS * 1e9), flops / (MFMA_BF16_PEAK_TFLOPS * 1e12)) * 1e3
    T = w.n_tokens
    out = {
        "metric": "layer-forward tokens/s on 1 MI355X (overlapped vs sequential); % of roofline",
        "value": T / (results[best] * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": results[best], "timing": "median of per-step HIP-event times on the origin stream",
        "ms_per_step_min": stats[best]["min_ms"], "ms_per_step_max": stats[best]["max_ms"],
        "ms_per_step_wall_mean": stats[best]["wall_mean_ms"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.shape.dtype, "data": "synthetic",
        "config": {"workload": "%s: %d-layer decoder forward, %d tokens / %d sequences, hidden %d, heads %d/%d x %d, "
                               "mlp %d, page %d" % (w.name, w.shape.n_layers, T, w.n_seqs, w.shape.hidden, w.shape.n_q,
                                                    w.shape.n_kv, w.shape.head_dim, w.shape.inter, w.shape.page_size),
                   "schedule": best, "nano_rows": list(w.nano_rows),
                   # schedules on CU partitions are always issued eagerly: a replayed graph drops the masks
                   "hip_graph": use_graph and "cu_partitioned" not in best},
        "sequential_tokens_per_s": T / (results["sequential"] * 1e-3),
        "sequential_ms_per_step": results["sequential"],
        "best_overlapped_schedule": best_ovl,
        "best_overlapped_ms_per_step": results[best_ovl],
        "overlap_speedup": results["sequential"] / results[best_ovl],
        "schedules_ms": results,
        "schedules_stats_ms": stats,
        "hbm": {"peak_GB/s": HBM_PEAK_GBS, "measured_stream_read": stream_read},
        "kv_placement": placement if placement is not None else "stacked",
        "kv_chunk_positions": {"used": kv_chunk or 256, "attention_dispatch_us": chunk_us},
        "mfma": {"peak_TFLOP/s": MFMA_BF16_PEAK_TFLOPS, "measured_loop": mfma_loop},
        "tuned": tuned,
        "policy": {"choice": "split at row %d" % policy["cut_row"] if policy["split"] else "sequential",
                   "est_sequential_ms_per_layer": policy["est_sequential_us"] * 1e-3,
                   "est_split_ms_per_layer": policy["est_split_us"] * 1e-3 if policy["est_split_us"] else None},
        "layer_roofline": {"algorithmic_bytes": byts, "algorithmic_flops": flops, "t_roof_ms": t_roof_ms,
                           "frac_overlapped": t_roof_ms / results[best_ovl], "frac_sequential": t_roof_ms / results["sequential"]},
        "op_ms_sequential_eager": {k: sum(v) / len(v) for k, v in op_ms.items()},
        "roofline": dict(roofline, traffic=traffic["bytes"] if traffic and roofline["kernel"] == "attn_mfma_kernel" else None,
                         traffic_source=traffic["source"] if traffic and roofline["kernel"] == "attn_mfma_kernel" else None),
    }
    # the same kernel against what this machine's memory system / matrix cores gave the library's probes in this run
    if out["roofline"]["bound"] == "hbm":
        out["roofline"]["frac_of_measured_stream_read"] = out["roofline"]["achieved"] / stream_read["GB/s"]
    elif mfma_loop:
        out["roofline"]["frac_of_measured_loop_random_operands"] = out["roofline"]["achieved"] / mfma_loop["random_operands"]["TFLOP/s"]
    if not args.no_mix:
        out["prefill_decode_mix"] = prefill_decode_mix(B, gen, stream, min(args.steps, 100), args.warmup)
        log("prefill + decode mix: %s" % out["prefill_decode_mix"])
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a sample ...")
        out["cpu_baseline"] = cpu_baseline(w, host_data if host_data is not None else data, 128 if w.shape.n_layers == 1 else 16)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
