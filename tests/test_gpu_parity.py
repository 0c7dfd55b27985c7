"""GPU parity: the HIP path through the C-ABI against the CPU oracle, and every legal
schedule against the sequential one, bit for bit."""
import numpy as np
import pytest
import torch

from paper_2605_21603_amd import binding as B
from workloads import gen

from gpu_util import GpuRun, check_against_oracle, say

pytestmark = pytest.mark.gpu

SMALL = ["c1", "f32_small", "c2_small", "c3_small", "c5_small", "c4_small", "f32_moe_small", "c3_mid", "pf_long", "pf_g8",
         "pf_mha", "pf_480", "pf_640", "bf16_hd64", "bf16_ps32", "bf16_max", "stack_mixed", "pf_g16", "pf_g2", "pf_deep", "dec_deep", "moe_mid", "moe_many_a", "moe_many_b",
         "shallow_a", "shallow_b", "shallow_wide"]


def schedules_for(w):
    rows = w.nano_rows
    k = len(rows) - 1
    chain = B.MOE_CHAIN if w.shape.n_experts else B.DENSE_CHAIN
    out = {
        "split": B.nano_schedule(rows, chain),
        "split_stagger2": B.nano_schedule(rows, chain, stagger=2),
        "split_one_stream": B.nano_schedule(rows, chain, streams=[0] * k),
        "mlp_merged": B.nano_schedule(rows, chain, merged_ops=[B.DYN_OP_GATE_UP, B.DYN_OP_SILU, B.DYN_OP_DOWN], stagger=1),
        "gemms_merged": B.nano_schedule(rows, chain, stagger=1,
                                        merged_ops=[B.DYN_OP_QKV, B.DYN_OP_OPROJ, B.DYN_OP_GATE_UP, B.DYN_OP_DOWN]),
        "route_merged_experts_split": B.nano_schedule(rows, chain, merged_ops=[B.DYN_OP_ROUTE, B.DYN_OP_NORM2], stagger=1),
        "with_empty_nano": B.nano_schedule((0,) + tuple(rows) if rows[1] != 0 else rows, chain),
    }
    if not w.shape.n_experts:
        del out["route_merged_experts_split"]
    return out


@pytest.mark.parametrize("name", SMALL)
def test_sequential_matches_oracle(name):
    say("case %s sequential" % name)
    w = gen.config(name)
    data = gen.generate(w)
    run = GpuRun(w, data)
    y, kc, vc = run.run(B.sequential())
    err = check_against_oracle(w, data, y, kc, vc)
    say("case %s max rel err %.3e" % (name, err))


@pytest.mark.parametrize("name", SMALL)
def test_every_schedule_is_bit_exact_against_sequential(name):
    w = gen.config(name)
    data = gen.generate(w)
    run = GpuRun(w, data)
    y0, k0, v0 = run.run(B.sequential())
    for label, sched in schedules_for(w).items():
        say("case %s schedule %s" % (name, label))
        y, kc, vc = run.run(sched)
        assert torch.equal(y.view(torch.uint8), y0.view(torch.uint8)), label
        assert torch.equal(kc.view(torch.uint8), k0.view(torch.uint8)), label
        assert torch.equal(vc.view(torch.uint8), v0.view(torch.uint8)), label


def test_empty_batch_is_a_no_op():
    w = gen.config("c2_small")
    data = gen.generate(w)
    run = GpuRun(w, data)
    step = B.DeviceStep(run.layer, data)
    step.batch.n_tokens = 0
    step.batch.n_seqs = 0
    run.layer.forward(step.batch, B.sequential(), torch.cuda.Stream())
    torch.cuda.synchronize()


def test_forward_rejects_small_workspace_and_aliasing():
    w = gen.config("c2_small")
    data = gen.generate(w)
    run = GpuRun(w, data)
    step = B.DeviceStep(run.layer, data)
    step.batch.workspace_bytes = 1024
    with pytest.raises(B.DynError) as e:
        run.layer.forward(step.batch, B.sequential(), torch.cuda.Stream())
    assert e.value.status == B.DYN_ERR_WORKSPACE
    step = B.DeviceStep(run.layer, data)
    step.batch.y = step.batch.x
    with pytest.raises(B.DynError) as e:
        run.layer.forward(step.batch, B.sequential(), torch.cuda.Stream())
    assert e.value.status == B.DYN_ERR_INVALID_ARG


def cu_masks_halves():
    """Two CU masks that split every XCD's CUs in half (bit i of the mask is CU i / 8 of XCD
    i % 8; 256 CUs -> 8 words)."""
    lo = [0x0000FFFF] * 8
    hi = [0xFFFF0000] * 8
    return [lo, hi]


@pytest.mark.parametrize("name", ["c2_small", "c5_small", "stack_mixed"])
def test_cu_partitioned_streams_and_graph_replay(name):
    """Micro-batches on CU-masked streams, with and without use_graph (the library issues a
    schedule on CU partitions eagerly either way: a replayed graph would drop the masks),
    several forwards with eager forwards and synchronisations in between; each must reproduce
    the sequential bits."""
    w = gen.config(name)
    data = gen.generate(w)
    run = GpuRun(w, data)
    y0, k0, v0 = run.run(B.sequential())
    k = len(w.nano_rows) - 1
    parts = [1 + (b % 2) for b in range(k)]
    for use_graph in (False, True):
        sched = B.nano_schedule(w.nano_rows, stagger=1, partitions=parts, cu_masks=cu_masks_halves(), use_graph=use_graph)
        say("case %s masked partitions graph=%s" % (name, use_graph))
        step = B.DeviceStep(run.layer, data)
        st = torch.cuda.Stream()
        for rep in range(4):
            say("case %s masked partitions graph=%s replay %d" % (name, use_graph, rep))
            step.y.zero_()
            torch.cuda.synchronize()
            with torch.cuda.stream(st):
                run.layer.forward(step.batch, sched, st)
            say("  issued")
            st.synchronize()
            say("  done")
            assert torch.equal(step.y.cpu().view(torch.uint8), y0.view(torch.uint8)), (use_graph, rep)
            # eager work of the program itself between replays
            y1, _, _ = run.run(B.sequential())
            assert torch.equal(y1.view(torch.uint8), y0.view(torch.uint8))
        assert torch.equal(step.k_cache.cpu().view(torch.uint8), k0.view(torch.uint8))
    seq_graph = B.sequential(use_graph=True)
    y2, k2, _ = run.run(seq_graph, repeat=3)
    assert torch.equal(y2.view(torch.uint8), y0.view(torch.uint8))


@pytest.mark.parametrize("name", ["c5_small", "c3_small", "c4_small"])
def test_partitions_by_operator_class_match_sequential(name):
    """Every micro-batch's attention on one CU partition (the low 128 bits of the mask: 16 CUs of
    every XCD) and all its other operators on the other half, so consecutive operators of a
    micro-batch change hardware queues and every dependency is an event between two masked
    streams.  Same bits as the sequential order; use_graph is set and ignored."""
    w = gen.config(name)
    data = gen.generate(w)
    run = GpuRun(w, data)
    y0, k0, v0 = run.run(B.sequential())
    chain = B.MOE_CHAIN if w.shape.n_experts else B.DENSE_CHAIN
    masks = [[0xFFFFFFFF] * 4 + [0] * 4, [0] * 4 + [0xFFFFFFFF] * 4]
    k = len(w.nano_rows) - 1
    for use_graph in (False, True):
        sched = B.nano_schedule(w.nano_rows, chain, stagger=2, partitions=[2] * k, op_partitions={B.DYN_OP_ATTN: 1},
                                cu_masks=masks, use_graph=use_graph)
        say("case %s attention on its own partition graph=%s" % (name, use_graph))
        y1, k1, v1 = run.run(sched, repeat=2)
        assert torch.equal(y1.view(torch.uint8), y0.view(torch.uint8))
        assert torch.equal(k1.view(torch.uint8), k0.view(torch.uint8)) and torch.equal(v1.view(torch.uint8), v0.view(torch.uint8))


@pytest.mark.parametrize("name", ["c5_small", "stack_mixed"])
def test_caches_placed_layer_by_layer_match_the_stacked_ones(name):
    """k_cache_layers / v_cache_layers: every layer's K and V pool in a buffer of its own, in
    shuffled order inside one arena with gaps, instead of one stacked tensor with a uniform
    stride.  Same output bits and same cache contents, eagerly and as a replayed graph."""
    w = gen.config(name)
    data = gen.generate(w)
    run = GpuRun(w, data)
    y0, k0, v0 = run.run(B.sequential())
    L = w.shape.n_layers
    n = data["k_cache"][0].numel()
    slot = n + 1024                                   # elements; keeps every pool 16-byte aligned and apart
    arena = torch.zeros(2 * L * slot, dtype=data["k_cache"][0].dtype, device="cuda:0")
    order = torch.randperm(2 * L, generator=torch.Generator().manual_seed(3)).tolist()
    for use_graph in (False, True):
        ks = [arena[order[l] * slot: order[l] * slot + n].view(data["k_cache"][l].shape) for l in range(L)]
        vs = [arena[order[L + l] * slot: order[L + l] * slot + n].view(data["v_cache"][l].shape) for l in range(L)]
        for l in range(L):
            ks[l].copy_(data["k_cache"][l])
            vs[l].copy_(data["v_cache"][l])
        step = B.DeviceStep(run.layer, dict(data, k_cache=ks, v_cache=vs), placed=True)
        st = torch.cuda.Stream()
        say("case %s placed layers graph=%s" % (name, use_graph))
        with torch.cuda.stream(st):
            for _ in range(3 if use_graph else 1):
                run.layer.forward(step.batch, B.sequential(use_graph=use_graph), st)
        st.synchronize()
        torch.cuda.synchronize()
        assert torch.equal(step.y.cpu().view(torch.uint8), y0.view(torch.uint8))
        for l in range(L):
            assert torch.equal(ks[l].cpu().view(torch.uint8), k0[l].view(torch.uint8)), l
            assert torch.equal(vs[l].cpu().view(torch.uint8), v0[l].view(torch.uint8)), l
    sched = B.nano_schedule(w.nano_rows, stagger=2, use_graph=True)
    with torch.cuda.stream(st):
        run.layer.forward(step.batch, sched, st)
    st.synchronize()
    assert torch.equal(step.y.cpu().view(torch.uint8), y0.view(torch.uint8))


@pytest.mark.parametrize("name,chunk", [("c2_small", 64), ("c2_small", 1024), ("c5_small", 128), ("c5_small", 2048), ("dec_deep", 1024),
                                        ("dec_deep", 8192), ("c3_small", 512), ("stack_mixed", 64), ("bf16_ps32", 1024), ("f32_small", 64)])
def test_other_split_kv_chunk_sizes_match_the_oracle_and_every_schedule(name, chunk):
    """kv_chunk_positions of the configuration: the chunking of decode attention is part of the
    arithmetic of a handle, not of a schedule.  Against the oracle, and bit for bit between the
    sequential order, a split and a merged-MLP form (eager and as a graph), for chunks from four
    pages to far more than any sequence has (no split at all) and a context of 70 thousand
    positions in 9 and 69 chunks (one- and two-level merges)."""
    w = gen.config(name)
    data = gen.generate(w)
    run = GpuRun(w, data, kv_chunk_positions=chunk)
    say("case %s chunk %d sequential" % (name, chunk))
    y0, k0, v0 = run.run(B.sequential())
    err = check_against_oracle(w, data, y0, k0, v0)
    say("case %s chunk %d: max rel err vs oracle %.3e" % (name, chunk, err))
    chain = B.MOE_CHAIN if w.shape.n_experts else B.DENSE_CHAIN
    mlp = [B.DYN_OP_GATE_UP, B.DYN_OP_SILU, B.DYN_OP_DOWN]
    for label, sched in [("split", B.nano_schedule(w.nano_rows, chain, stagger=2)),
                         ("mlp merged, graph", B.nano_schedule(w.nano_rows, chain, merged_ops=mlp, stagger=1, use_graph=True))]:
        say("case %s chunk %d %s" % (name, chunk, label))
        y1, k1, v1 = run.run(sched, repeat=2 if sched.use_graph else 1)
        assert torch.equal(y1.view(torch.uint8), y0.view(torch.uint8)), label
        assert torch.equal(k1.view(torch.uint8), k0.view(torch.uint8)) and torch.equal(v1.view(torch.uint8), v0.view(torch.uint8)), label


def test_profiling_reports_every_dispatch():
    w = gen.config("c2_small")
    data = gen.generate(w)
    run = GpuRun(w, data)
    run.layer.set_profiling(True)
    sched = B.nano_schedule(w.nano_rows, stagger=1)
    run.run(sched)
    recs = run.layer.slot_times()
    run.layer.set_profiling(False)
    assert len(recs) == len(sched.slots)
    for r, s in zip(recs, sched.slots):
        assert (r["op"], r["nano"], r["n_nano"], r["stream"]) == tuple(s[:4])
        assert r["start_ms"] <= r["main_start_ms"] <= r["main_stop_ms"] <= r["stop_ms"]
    with pytest.raises(B.DynError):          # profiling is for eager schedules
        run.layer.set_profiling(True)
        try:
            run.run(B.sequential(use_graph=True))
        finally:
            run.layer.set_profiling(False)


def test_graph_cache_eviction_keeps_replays_correct():
    """More distinct schedules than the graph cache holds, replayed back to back without a host
    wait in between: an evicted graph may still be running when it leaves the cache and is
    destroyed only after its last replay has finished.  Every replay reproduces the sequential
    result, and a schedule evicted earlier is captured again when it comes back."""
    w = gen.config("c2_small")
    data = gen.generate(w)
    run = GpuRun(w, data)
    y0, k0, v0 = run.run(B.sequential())
    md = gen.metadata(w)
    sch = B.Scheduler(B.make_config(w.shape), md["q_start"])
    cands = [c for c in sch.tune_candidates(md["ctx_len"], max_k=2) if c.cus_first == 0][:20]
    assert len(cands) == 20
    step = B.DeviceStep(run.layer, data, run.device)
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        for _ in range(2):                        # second pass: the first entries were evicted by then
            for c in cands:
                run.layer.forward(step.batch, sch.tune_record(c, use_graph=True), st)
                run.layer.forward(step.batch, sch.tune_record(c, use_graph=True), st)
    st.synchronize()
    torch.cuda.synchronize()
    assert torch.equal(step.y.cpu().view(torch.uint8), y0.view(torch.uint8))
    assert torch.equal(step.k_cache.cpu().view(torch.uint8), k0.view(torch.uint8))


def test_cached_graph_is_not_replayed_for_another_sequence_structure():
    """Two batches that agree in every pointer, in n_tokens, n_seqs and the cut row, and differ
    only in where the two-token sequence sits: (2,1,1) against (1,1,2), cut at row 2.  Which
    attention kernels a micro-batch launches follows from that structure, so a graph captured for
    one must not be replayed for the other.  Same buffers throughout, contents swapped in place."""
    import dataclasses
    sh = gen.LayerShape("bf16", 512, 8, 2, 128, 1024)
    wa = gen.Workload("swap_a", sh, ((2, 40), (1, 70), (1, 100)), 31, (0, 2, 4))
    wb = gen.Workload("swap_b", sh, ((1, 100), (1, 70), (2, 40)), 32, (0, 2, 4))
    da, db = gen.generate(wa), gen.generate(wb)
    db["weights"] = da["weights"]            # one layer handle serves both batches
    assert da["block_table"].shape == db["block_table"].shape and da["n_pages"] == db["n_pages"]
    run = GpuRun(wa, da)
    step = B.DeviceStep(run.layer, da)
    step.q_start_host = step.q_start_host.copy()          # a host array of the step's own, rewritten in place below
    step.batch.q_start_host = step.q_start_host.ctypes.data
    sched = B.nano_schedule((0, 2, 4), stagger=1, use_graph=True)
    st = torch.cuda.Stream()

    def load(data):
        step.x.copy_(data["x"])
        step.k_cache.copy_(torch.stack(data["k_cache"]))
        step.v_cache.copy_(torch.stack(data["v_cache"]))
        step.seq_of_token.copy_(torch.from_numpy(data["seq_of_token"]))
        step.pos_of_token.copy_(torch.from_numpy(data["pos_of_token"]))
        step.block_table.copy_(torch.from_numpy(np.ascontiguousarray(data["block_table"])))
        step.q_start_host[:] = data["q_start"]
        step.y.zero_()
        torch.cuda.synchronize()

    for label, (w, data) in (("a", (wa, da)), ("b", (wb, db)), ("a again", (wa, da)), ("b again", (wb, db))):
        say("case swap: structure %s under the same buffers" % label)
        load(data)
        with torch.cuda.stream(st):
            run.layer.forward(step.batch, sched, st)
        st.synchronize()
        err = check_against_oracle(w, data, step.y.cpu(), step.k_cache.cpu(), step.v_cache.cpu())
        say("case swap %s: max rel err %.3e" % (label, err))


def test_released_graphs_are_captured_again():
    """dyn_layer_release_graphs waits for and destroys every captured graph; the same schedules
    then capture afresh and reproduce the same bits."""
    w = gen.config("c3_small")
    data = gen.generate(w)
    run = GpuRun(w, data)
    y0, k0, v0 = run.run(B.sequential())
    scheds = [B.sequential(use_graph=True), B.nano_schedule(w.nano_rows, stagger=1, use_graph=True),
              B.nano_schedule(w.nano_rows, stagger=2, merged_ops=[B.DYN_OP_GATE_UP, B.DYN_OP_SILU, B.DYN_OP_DOWN], use_graph=True)]
    step = B.DeviceStep(run.layer, data)
    st = torch.cuda.Stream()
    for rnd in range(3):
        for sched in scheds:
            step.y.zero_()
            torch.cuda.synchronize()
            with torch.cuda.stream(st):
                run.layer.forward(step.batch, sched, st)
                run.layer.forward(step.batch, sched, st)
            if rnd == 1:
                run.layer.release_graphs()          # replays still in flight: the call waits for them
            st.synchronize()
            assert torch.equal(step.y.cpu().view(torch.uint8), y0.view(torch.uint8)), rnd
        run.layer.release_graphs()
    assert torch.equal(step.k_cache.cpu().view(torch.uint8), k0.view(torch.uint8))


@pytest.mark.parametrize("name", ["c2_small", "c3_small", "c4_small", "c5_small", "f32_moe_small", "moe_many_b", "stack_mixed", "pf_640"])
def test_schedule_sized_workspace_with_shared_regions_is_bit_exact(name):
    """The workspace sized for one schedule (regions that are never alive together share bytes),
    filled with 0xFF, with a guard behind it: same bits as with the any-schedule workspace, the
    guard untouched, a second forward on the used workspace the same again."""
    w = gen.config(name)
    data = gen.generate(w)
    run = GpuRun(w, data)
    y0, k0, v0 = run.run(B.sequential())
    scheds = dict(schedules_for(w), sequential=B.sequential(), sequential_graph=B.sequential(use_graph=True))
    st = torch.cuda.Stream()
    for label, sched in scheds.items():
        step = B.DeviceStep(run.layer, data, sched=sched, guard=4096)
        bound = run.layer.workspace_bytes(w.n_tokens, step.batch.max_pages_per_seq)
        say("case %s schedule %s: workspace %d bytes (any schedule: %d)" % (name, label, step.batch.workspace_bytes, bound))
        assert step.batch.workspace_bytes <= bound
        step.workspace.fill_(0xFF)
        torch.cuda.synchronize()
        for rep in range(2):
            step.y.zero_()
            torch.cuda.synchronize()
            with torch.cuda.stream(st):
                run.layer.forward(step.batch, sched, st)
            st.synchronize()
            assert torch.equal(step.y.cpu().view(torch.uint8), y0.view(torch.uint8)), (label, rep)
        assert torch.equal(step.k_cache.cpu().view(torch.uint8), k0.view(torch.uint8)), label
        assert torch.equal(step.v_cache.cpu().view(torch.uint8), v0.view(torch.uint8)), label
        guard = step.workspace[step.workspace_offset + step.batch.workspace_bytes:]
        assert bool((guard == 0xFF).all()), label
        # one byte less is refused
        step.batch.workspace_bytes -= 1
        with pytest.raises(B.DynError) as e:
            run.layer.forward(step.batch, sched, st)
        assert e.value.status == B.DYN_ERR_WORKSPACE


def test_matrix_core_probe_multiplies_what_it_says():
    """The measurement aid behind bench.py's `mfma.measured_loop`: with every operand 1.0 each of a lane's 128
    accumulator elements gains 32 per MFMA and sees two MFMAs per stage, so its sum is 8192 x stages exactly - the
    probe issues the 64 MFMAs per wave and stage its FLOP count claims - and with zeros it is zero."""
    dev = torch.device("cuda:0")
    stream = torch.cuda.Stream()
    sink = torch.full((256 * 512,), -1.0, dtype=torch.float32, device=dev)
    ones = torch.ones(8 << 20, dtype=torch.bfloat16, device=dev)
    zeros = torch.zeros(8 << 20, dtype=torch.bfloat16, device=dev)
    torch.cuda.synchronize()
    for stages in (1, 8, 13):
        say("matrix-core probe, ones, %d stages" % stages)
        flops = B.probe_mfma_loop(ones, stages, sink, stream)
        torch.cuda.synchronize()
        assert flops == 256 * 8 * stages * 64 * 16 * 16 * 32 * 2
        assert torch.equal(sink, torch.full_like(sink, 8192.0 * stages))
    say("matrix-core probe, zeros")
    B.probe_mfma_loop(zeros, 5, sink, stream)
    torch.cuda.synchronize()
    assert torch.count_nonzero(sink).item() == 0
    with pytest.raises(B.DynError):
        B.probe_mfma_loop(ones[: (8 << 20) - 8], 4, sink, stream)
