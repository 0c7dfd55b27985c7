"""Host-side tests (no GPU) of the measured tuner's candidate set and recording (the knobs of
Section 2.1: unequal micro-batch sizes and the share of compute units per overlapped stream):
every candidate is a legal schedule, cuts are sequence boundaries, the set holds unequal
sizes, the context-balanced cut and the prefill / decode boundary, masks take the same share
of every XCD, and bad arguments are refused before any device call."""
import ctypes as C

import numpy as np
import pytest

from paper_2605_21603_amd import binding as B
from workloads import gen

from test_abi_host import fake_layer, host_batch


def scheduler_for(name):
    w = gen.config(name)
    md = gen.metadata(w)
    return w, md, B.Scheduler(B.make_config(w.shape), md["q_start"])


@pytest.mark.parametrize("name", ["c1", "c2_small", "c3_small", "c4_small", "c5_small", "pf_long"])
def test_every_candidate_records_into_a_legal_schedule(name):
    w, md, sch = scheduler_for(name)
    _, layer = fake_layer(name)
    cands = sch.tune_candidates(md["ctx_len"], max_k=4, partitions=3)
    assert cands[0].form == B.DYN_FORM_SEQUENTIAL and cands[0].k == 1
    assert [cands[0].rows[0], cands[0].rows[1]] == [0, w.n_tokens]
    bounds = set(int(q) for q in md["q_start"])
    keys = set()
    chain = B.MOE_CHAIN if w.shape.n_experts else B.DENSE_CHAIN
    for c in cands:
        d = c.as_dict()
        key = (d["k"], tuple(d["rows"]), d["form"], d["stagger"], d["cus_first"])
        assert key not in keys, "duplicate candidate %s" % (key,)
        keys.add(key)
        assert d["rows"][0] == 0 and d["rows"][-1] == w.n_tokens
        assert all(r in bounds for r in d["rows"])
        assert all(b > a for a, b in zip(d["rows"], d["rows"][1:])), "empty micro-batch in %s" % (d,)
        rec = sch.tune_record(c, n_cus=256, use_graph=True)
        layer.validate(host_batch(w), rec)
        # every (operator, micro-batch) exactly once
        seen = []
        for op, nano, n_nano, stream, part in rec.slots:
            seen += [(op, nano + j) for j in range(n_nano)]
            assert part == 0 or d["cus_first"] > 0
            if n_nano > 1:
                assert (stream, part) == (0, 0)          # merged dispatches use the whole device
        assert sorted(seen) == sorted((op, b) for op in chain for b in range(d["k"]))


def test_sequential_is_the_only_candidate_for_a_single_sequence():
    w, md, sch = scheduler_for("pf_long")
    if w.n_seqs == 1:
        assert len(sch.tune_candidates(md["ctx_len"])) == 1
    sch1 = B.Scheduler(B.make_config(w.shape), [0, 7])
    assert [c.as_dict()["form"] for c in sch1.tune_candidates([7], max_k=4, partitions=3)] == ["sequential"]


def test_cut_points_cover_unequal_sizes_the_context_balance_and_the_prefill_boundary():
    # 32 decodes whose contexts grow with the index: the cut that halves the keys is far from the middle
    q = list(range(33))
    ctx = [16 * (i + 1) for i in range(32)]
    cfg = B.make_config(gen.config("c2_small").shape)
    sch = B.Scheduler(cfg, q)
    cuts = sorted({c.rows[1] for c in sch.tune_candidates(ctx) if c.k == 2})
    assert {8, 12, 16, 20, 24} <= set(cuts)                     # 1/4 .. 3/4 of the tokens
    half = next(i + 1 for i in range(32) if sum(ctx[:i + 1]) >= sum(ctx) / 2)
    assert half in cuts and half not in (8, 12, 16, 20, 24)
    without_ctx = sorted({c.rows[1] for c in sch.tune_candidates(None) if c.k == 2})
    assert half not in without_ctx
    # a 40-token prefill chunk followed by 6 decodes: the boundary is a cut although no fraction lands on it
    q2 = [0, 40] + [41 + i for i in range(6)]
    sch2 = B.Scheduler(cfg, q2)
    cuts2 = {c.rows[1] for c in sch2.tune_candidates([40] + [100] * 6) if c.k == 2}
    assert 40 in cuts2


def test_forms_and_staggers_offered_per_cut():
    w, md, sch = scheduler_for("c2_small")
    cands = [c.as_dict() for c in sch.tune_candidates(md["ctx_len"], max_k=2, partitions=1)]
    cut = cands[1]["rows"][1]
    here = [(c["form"], c["stagger"], c["cus_first"]) for c in cands if c["k"] == 2 and c["rows"][1] == cut]
    assert here == [("split", 2, 0), ("mlp_merged", 1, 0), ("mlp_merged", 2, 0), ("attn_split", 1, 0), ("mlp_split", 1, 0),
                    ("split", 2, 128), ("mlp_merged", 2, 128)]
    assert all(c["k"] <= 2 for c in cands)
    assert any(c["k"] == 4 for c in (x.as_dict() for x in sch.tune_candidates(md["ctx_len"], max_k=4)))


def test_recorded_forms_merge_what_they_say():
    w, md, sch = scheduler_for("c4_small")
    by_form = {}
    for c in sch.tune_candidates(md["ctx_len"]):
        by_form.setdefault(c.form, c)
    merged = lambda rec: sorted({op for op, nano, n_nano, s, p in rec.slots if n_nano > 1})
    assert merged(sch.tune_record(by_form[B.DYN_FORM_SPLIT])) == []
    assert merged(sch.tune_record(by_form[B.DYN_FORM_MLP_MERGED])) == [B.DYN_OP_ROUTE, B.DYN_OP_GATE_UP, B.DYN_OP_SILU,
                                                                        B.DYN_OP_DOWN]
    assert merged(sch.tune_record(by_form[B.DYN_FORM_ATTN_SPLIT])) == [B.DYN_OP_QKV, B.DYN_OP_OPROJ, B.DYN_OP_GATE_UP,
                                                                        B.DYN_OP_DOWN]
    assert merged(sch.tune_record(by_form[B.DYN_FORM_MLP_SPLIT])) == [B.DYN_OP_NORM1, B.DYN_OP_QKV, B.DYN_OP_ROPE_KV,
                                                                       B.DYN_OP_ATTN, B.DYN_OP_OPROJ, B.DYN_OP_NORM2]
    seq = sch.tune_record(by_form[B.DYN_FORM_SEQUENTIAL])
    assert [s[0] for s in seq.slots] == B.MOE_CHAIN and all(s[3] == 0 and s[4] == 0 for s in seq.slots)


def test_stagger_delays_the_second_micro_batch():
    w, md, sch = scheduler_for("c2_small")
    c = next(c for c in sch.tune_candidates(md["ctx_len"]) if c.form == B.DYN_FORM_SPLIT and c.stagger == 2)
    order = [(op, nano) for op, nano, n, s, p in sch.tune_record(c).slots]
    assert order[:3] == [(B.DYN_OP_NORM1, 0), (B.DYN_OP_QKV, 0), (B.DYN_OP_ROPE_KV, 0)]
    assert order[3] == (B.DYN_OP_NORM1, 1)


def test_partition_masks_take_the_same_share_of_every_xcd():
    w, md, sch = scheduler_for("c2_small")
    for cus, lo in ((128, 0x0000FFFF), (64, 0x000000FF), (192, 0x00FFFFFF)):
        c = next(c for c in sch.tune_candidates(md["ctx_len"], partitions=3) if c.cus_first == cus)
        sc = sch.tune_record(c, n_cus=256).to_c()
        assert sc.n_partitions == 2 and sc.cu_mask_words == 8
        masks = C.cast(sc.cu_masks, C.POINTER(C.c_uint32))
        assert [masks[i] for i in range(8)] == [lo] * 8
        assert [masks[8 + i] for i in range(8)] == [0xFFFFFFFF & ~lo] * 8
    # recording an unpartitioned candidate afterwards drops the masks again
    c0 = next(c for c in sch.tune_candidates(md["ctx_len"]) if c.k == 2)
    assert sch.tune_record(c0).to_c().n_partitions == 0
    # a device with 64 CUs: two mask words of 32
    c64 = next(c for c in sch.tune_candidates(md["ctx_len"], partitions=1, n_cus=64) if c.cus_first)
    assert c64.cus_first == 32
    sc = sch.tune_record(c64, n_cus=64).to_c()
    masks = C.cast(sc.cu_masks, C.POINTER(C.c_uint32))
    assert sc.cu_mask_words == 2 and [masks[i] for i in range(4)] == [0xFFFF, 0xFFFF, 0xFFFF0000, 0xFFFF0000]


def test_bad_arguments_are_refused_on_the_host():
    w, md, sch = scheduler_for("c2_small")
    with pytest.raises(B.DynError):
        sch.tune_candidates(md["ctx_len"], max_k=5)
    with pytest.raises(B.DynError):
        sch.tune_candidates(md["ctx_len"], partitions=4)
    with pytest.raises(B.DynError):
        sch.tune_candidates(md["ctx_len"], n_cus=100)
    good = next(c for c in sch.tune_candidates(md["ctx_len"]) if c.k == 2)

    def variant(**kw):
        c = B.dyn_tune_candidate()
        C.memmove(C.byref(c), C.byref(good), C.sizeof(c))
        for k, v in kw.items():
            setattr(c, k, v)
        return c

    for bad in (variant(k=0), variant(form=9), variant(stagger=-1), variant(form=B.DYN_FORM_SEQUENTIAL),
                variant(cus_first=100), variant(cus_first=256)):
        with pytest.raises(B.DynError):
            sch.tune_record(bad, n_cus=256)
    inside = variant()
    inside.rows[1] = good.rows[1]
    inside.rows[2] = w.n_tokens - 1                       # does not cover the batch
    with pytest.raises(B.DynError):
        sch.tune_record(inside)
    # the device call checks its pointers before touching the GPU
    opt = B.dyn_tune_options()
    res = B.dyn_tune_result()
    sc = B.dyn_schedule()
    rc = B.lib().dyn_tune(None, None, None, C.byref(opt), None, None, C.byref(sc), C.byref(res), None, 0)
    assert rc == B.DYN_ERR_INVALID_ARG and "NULL" in B.dyn_last_error()
    # more than four micro-batches are refused before any device call
    _, layer = fake_layer("c2_small")
    batch = host_batch(w)
    fake_stream = C.c_void_p(1)
    opt_k = B.dyn_tune_options(max_k=5)
    rc = B.lib().dyn_tune(layer.handle, C.byref(batch), None, C.byref(opt_k), fake_stream, sch._h, C.byref(sc), C.byref(res), None, 0)
    assert rc == B.DYN_ERR_INVALID_ARG and "four micro-batches" in B.dyn_last_error()
