"""Host-side tests (no GPU) of the programmable scheduling calls: split, get_ready_ops,
execute in its split, merge and sequential-fallback forms, finish, and the built-in policy.
Strategies below are written the way the paper's are (Section 3.2.2, Figure 6): a short
program over those calls; the library checks every step against the ready-operator rule."""
import numpy as np
import pytest

from paper_2605_21603_amd import binding as B
from workloads import gen

from test_abi_host import fake_layer, host_batch


def scheduler_for(name):
    w = gen.config(name)
    md = gen.metadata(w)
    return w, md, B.Scheduler(B.make_config(w.shape), md["q_start"])


def round_robin(sch, k, streams=None):
    """Each micro-batch on its own stream, one ready operator at a time."""
    while True:
        issued = False
        for b in range(k):
            ready = sch.get_ready_ops(b)
            if ready:
                sch.execute([(ready[0], b)], stream=streams[b] if streams else b)
                issued = True
        if not issued:
            return


def sizes_of(w):
    r = list(w.nano_rows)
    return [r[i + 1] - r[i] for i in range(len(r) - 1)]


def test_ready_ops_walk_the_chain_in_order():
    w, md, sch = scheduler_for("c2_small")
    sch.split(sizes_of(w))
    seen = []
    while True:
        ready = sch.get_ready_ops(0)
        if not ready:
            break
        assert len(ready) == 1
        seen.append(ready[0])
        # the other micro-batch is unaffected by this one's progress
        assert sch.get_ready_ops(1) == [B.DYN_OP_NORM1]
        sch.execute([(ready[0], 0)])
    assert seen == B.DENSE_CHAIN


def test_moe_chain_has_the_router():
    w, md, sch = scheduler_for("c4_small")
    seen = []
    while sch.get_ready_ops(0):
        op = sch.get_ready_ops(0)[0]
        seen.append(op)
        sch.execute([(op, 0)])
    assert seen == B.MOE_CHAIN


def test_round_robin_strategy_reproduces_the_descriptor_builder_and_validates():
    for name in ("c2_small", "c3_small", "c4_small"):
        w, md, sch = scheduler_for(name)
        k = len(w.nano_rows) - 1
        sch.split(sizes_of(w))
        round_robin(sch, k)
        rec = sch.finish(use_graph=True)
        chain = B.MOE_CHAIN if w.shape.n_experts else B.DENSE_CHAIN
        ref = B.nano_schedule(w.nano_rows, chain, stagger=0)
        assert rec.slots == [tuple(s) for s in ref.slots]
        assert rec.nano_rows == list(w.nano_rows)
        assert rec.to_c().n_streams == k and rec.to_c().use_graph == 1
        _, layer = fake_layer(name)
        layer.validate(host_batch(w), rec)


def test_execute_refuses_an_operator_that_is_not_ready_and_records_nothing():
    w, md, sch = scheduler_for("c2_small")
    sch.split(sizes_of(w))
    with pytest.raises(B.DynError) as e:
        sch.execute([(B.DYN_OP_QKV, 0)])
    assert e.value.status == B.DYN_ERR_SCHEDULE and "not ready" in str(e.value)
    assert sch.get_ready_ops(0) == [B.DYN_OP_NORM1]
    sch.execute([(B.DYN_OP_NORM1, 0)])
    with pytest.raises(B.DynError):                      # the same operator twice
        sch.execute([(B.DYN_OP_NORM1, 0)])
    with pytest.raises(B.DynError):                      # a second pair that is not ready undoes the first
        sch.execute([(B.DYN_OP_QKV, 0), (B.DYN_OP_QKV, 1)])
    assert sch.get_ready_ops(0) == [B.DYN_OP_QKV]
    with pytest.raises(B.DynError):                      # dense layer: no router
        sch.execute([(B.DYN_OP_ROUTE, 0)])
    with pytest.raises(B.DynError):                      # micro-batch out of range
        sch.execute([(B.DYN_OP_NORM1, 5)])
    with pytest.raises(B.DynError):                      # partition never declared
        sch.execute([(B.DYN_OP_NORM1, 1)], partition=1)


def test_merge_form_and_sequential_fallback():
    w, md, sch = scheduler_for("c5_small")             # four micro-batches
    k = len(w.nano_rows) - 1
    assert k == 4
    sch.split(sizes_of(w))
    # same operator, adjacent micro-batches: one merged dispatch
    sch.execute([(B.DYN_OP_NORM1, b) for b in range(k)])
    # different operators in one call: dispatched one after another on that stream
    sch.execute([(B.DYN_OP_QKV, 0), (B.DYN_OP_QKV, 1), (B.DYN_OP_ROPE_KV, 0)], stream=2)
    # same operator but not adjacent: also the fallback
    sch.execute([(B.DYN_OP_QKV, 3), (B.DYN_OP_QKV, 2)], stream=1)
    round_robin(sch, k)
    rec = sch.finish()
    assert rec.slots[0] == (B.DYN_OP_NORM1, 0, 4, 0, 0)
    assert rec.slots[1:4] == [(B.DYN_OP_QKV, 0, 1, 2, 0), (B.DYN_OP_QKV, 1, 1, 2, 0), (B.DYN_OP_ROPE_KV, 0, 1, 2, 0)]
    assert rec.slots[4:6] == [(B.DYN_OP_QKV, 3, 1, 1, 0), (B.DYN_OP_QKV, 2, 1, 1, 0)]
    _, layer = fake_layer("c5_small")
    layer.validate(host_batch(w), rec)


def test_merged_operator_waits_for_every_micro_batch():
    """A merge needs all of its micro-batches at that operator: the strategy has to bring
    them there first (the paper's merged MLP after split attention)."""
    w, md, sch = scheduler_for("c2_small")
    sch.split(sizes_of(w))
    for op in B.DENSE_CHAIN[:6]:
        sch.execute([(op, 0)])
    with pytest.raises(B.DynError):
        sch.execute([(B.DYN_OP_GATE_UP, 0), (B.DYN_OP_GATE_UP, 1)])
    for op in B.DENSE_CHAIN[:6]:
        sch.execute([(op, 1)], stream=1)
    for op in B.DENSE_CHAIN[6:]:
        sch.execute([(op, 0), (op, 1)])
    rec = sch.finish()
    assert [s[2] for s in rec.slots[-3:]] == [2, 2, 2]
    _, layer = fake_layer("c2_small")
    layer.validate(host_batch(w), rec)


def test_split_checks_sizes_and_sequence_boundaries():
    w, md, sch = scheduler_for("c3_small")
    T = w.n_tokens
    with pytest.raises(B.DynError):
        sch.split([T - 1])                               # does not cover the batch
    with pytest.raises(B.DynError):
        sch.split([1] * 9 + [T - 9])                     # more than DYN_MAX_NANO
    q = md["q_start"]
    inside = next(r for r in range(1, T) if r not in set(int(v) for v in q))
    with pytest.raises(B.DynError) as e:
        sch.split([inside, T - inside])
    assert "inside a sequence" in str(e.value)
    sch.split([0, T])                                    # an empty micro-batch is legal
    round_robin(sch, 2)
    sch.finish()
    sch.split([T])                                       # a new split discards the recording
    assert sch.get_ready_ops(0) == [B.DYN_OP_NORM1]


def test_finish_refuses_an_incomplete_layer():
    w, md, sch = scheduler_for("c2_small")
    sch.split(sizes_of(w))
    for op in B.DENSE_CHAIN:
        sch.execute([(op, 0)])
    with pytest.raises(B.DynError) as e:
        sch.finish()
    assert e.value.status == B.DYN_ERR_SCHEDULE and "micro-batch 1" in str(e.value)


def test_partitions_are_declared_before_use():
    w, md, sch = scheduler_for("c2_small")
    sch.split(sizes_of(w))
    with pytest.raises(B.DynError):
        sch.set_partitions([[0] * 8])                    # empty mask
    sch.set_partitions([[0x0000FFFF] * 8, [0xFFFF0000] * 8])
    k = 2
    while sch.get_ready_ops(0) or sch.get_ready_ops(1):
        for b in range(k):
            r = sch.get_ready_ops(b)
            if r:
                sch.execute([(r[0], b)], stream=0, partition=b + 1)
    rec = sch.finish()
    c = rec.to_c()
    assert c.n_partitions == 2 and c.cu_mask_words == 8
    assert {s[4] for s in rec.slots} == {1, 2}
    _, layer = fake_layer("c2_small")
    layer.validate(host_batch(w), rec)


def test_policy_never_splits_pure_decode_and_its_schedule_validates():
    for name in ("c2", "c4", "c2_small"):
        w, md, sch = scheduler_for(name)
        rec, choice = sch.auto(md["ctx_len"])
        assert not choice["split"] and choice["est_split_us"] == 0.0
        assert choice["est_sequential_us"] > 0
        chain = B.MOE_CHAIN if w.shape.n_experts else B.DENSE_CHAIN
        assert rec.slots == [(op, 0, 1, 0, 0) for op in chain]
        _, layer = fake_layer(name)
        layer.validate(host_batch(w), rec)


def test_policy_estimates_follow_the_roofline():
    """Closed-form checks of the cost model on the Llama-3-8B decode shape: the estimate is
    bounded below by bytes at the datasheet bandwidth, grows with context by the K/V bytes
    at the modelled stream rate, and does not grow with a few more decode rows (weights
    dominate below the ridge)."""
    w = gen.config("c2")
    cfg = B.make_config(w.shape)

    def est(n, ctx):
        sch = B.Scheduler(cfg, list(range(n + 1)))
        return sch.auto([ctx] * n)[1]["est_sequential_us"]
    weights_mb, kv_per_pos = 436.2, 4096
    base = est(128, 1024)
    assert base > (weights_mb * 1e6 + 128 * 1024 * kv_per_pos) / 8e12 * 1e6          # slower than the 8 TB/s bound
    assert base < 3 * (weights_mb * 1e6 + 128 * 1024 * kv_per_pos) / 8e12 * 1e6      # and within 3x of it
    more_ctx = est(128, 2048)
    assert more_ctx - base == pytest.approx(128 * 1024 * kv_per_pos / 5.0e12 * 1e6, rel=0.02)
    # 16 more decode rows inside the same 128-row tile add their K/V and a little activation
    # traffic, no weight time
    extra = base - est(112, 1024)
    kv16 = 16 * 1024 * kv_per_pos / 5.0e12 * 1e6
    assert kv16 <= extra < kv16 + 5.0


def test_policy_considers_only_a_clean_prefill_decode_boundary():
    w = gen.config("c3")
    cfg = B.make_config(w.shape)
    # prefill chunk, decodes, another prefill chunk: two boundaries -> no split considered
    q = [0, 512] + [512 + i for i in range(1, 33)] + [512 + 32 + 512]
    ctx = [512] + [2048] * 32 + [512]
    sch = B.Scheduler(cfg, q)
    rec, choice = sch.auto(ctx)
    assert not choice["split"] and choice["est_split_us"] == 0.0
    # ctx shorter than the tokens of the step is an error
    with pytest.raises(B.DynError):
        sch.auto([100] + [2048] * 32 + [512])
    # one clean boundary: the split is priced, and whichever wins is a valid schedule
    md = gen.metadata(w)
    sch = B.Scheduler(cfg, md["q_start"])
    rec, choice = sch.auto(md["ctx_len"])
    assert choice["est_split_us"] > 0
    if choice["split"]:
        assert choice["cut_row"] == 2048 and rec.nano_rows == [0, 2048, 2112]
    _, layer = fake_layer("c3")
    layer.validate(host_batch(w), rec)
