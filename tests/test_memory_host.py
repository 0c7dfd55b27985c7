"""Host-side tests (no GPU) of the static data-flow analysis (Section 3.3.1, Algorithm 1:
reference counts, merge points served in place; Section 2.1: overlap raises peak memory)."""
import numpy as np
import pytest

from paper_2605_21603_amd import binding as B
from workloads import gen

from test_abi_host import fake_layer, host_batch


def setup(name):
    w = gen.config(name)
    md = gen.metadata(w)
    _, layer = fake_layer(name)
    return w, md, layer, host_batch(w), B.Scheduler(B.make_config(w.shape), md["q_start"])


def test_sequential_peak_of_the_fp32_layer_by_hand():
    """c1: 4 tokens, hidden 256, 4 heads of 64, MLP 1024, fp32, 8 pages of 16 per sequence.
    Row bytes (GEMM inputs carry 256 bytes of padding): h 1280, qkv 3072, attention out 1280,
    x2 1024, gate|up 8192, act 4352.  Attention scratch: 4 tokens x 4 heads x 1 chunk x
    (64 + 2) floats + (4 + 8) x 4 ints = 4416.  Alive while each operator runs:
      norm1 h | qkv (+ rotary, cache append) h+qkv | attn qkv+out+scratch | oproj (+ second norm) out+x2+h |
      gate_up x2+h+gu | silu x2+gu+act | down x2+act
    The gate (fp32: not fused into the projection) is the peak: 4 x (1024 + 8192 + 4352)."""
    w, md, layer, hb, sch = setup("c1")
    r = layer.memory(hb, B.sequential())
    assert r["peak_live_bytes"] == 4 * (1024 + 8192 + 4352) == 54272
    assert r["peak_at_dispatch"] == 7
    assert r["peak_live_bytes_sequential"] == r["peak_live_bytes"]
    assert r["n_regions"] == 7 and r["max_ref_count"] == 1 and r["n_resharded"] == 0
    assert r["workspace_bytes"] == layer.workspace_bytes(w.n_tokens, md["max_pages_per_seq"])
    assert r["peak_live_bytes"] < r["workspace_bytes"]


@pytest.mark.parametrize("name", ["c2_small", "c3_small", "c4_small", "c5_small"])
def test_every_candidate_schedule_accounts_consistently(name):
    w, md, layer, hb, sch = setup(name)
    seq = layer.memory(hb, B.sequential())
    L = w.shape.n_layers
    per_layer = seq["n_regions"] + 1            # layer 0 has no inter-layer input region
    assert per_layer % L == 0
    tensors = per_layer // L
    for c in sch.tune_candidates(md["ctx_len"], max_k=4):
        r = layer.memory(hb, sch.tune_record(c))
        assert r["workspace_bytes"] == seq["workspace_bytes"]
        assert 0 < r["peak_live_bytes"] <= r["workspace_bytes"]
        assert r["peak_live_bytes_sequential"] == seq["peak_live_bytes"]
        assert r["n_regions"] == c.k * (tensors * L - 1)
        assert r["max_ref_count"] == (2 if w.shape.n_experts else 1)     # only the routing result has two readers (gate/up, down)
        if c.form in (B.DYN_FORM_SEQUENTIAL, B.DYN_FORM_SPLIT):
            assert r["n_resharded"] == 0          # producer and consumers always at the same number of micro-batches
        else:
            assert r["n_resharded"] > 0           # split <-> merge transitions, all in place
        if c.form == B.DYN_FORM_SEQUENTIAL:
            assert r["peak_live_bytes"] == seq["peak_live_bytes"]


def test_reshard_points_of_the_mlp_merged_form():
    """Two micro-batches up to the second norm, MLP once: x2 (read by the merged down projection)
    and the normed input of the MLP change from two producers to one consumer, per micro-batch."""
    w, md, layer, hb, sch = setup("c2_small")
    c = next(c for c in sch.tune_candidates(md["ctx_len"]) if c.form == B.DYN_FORM_MLP_MERGED)
    assert layer.memory(hb, sch.tune_record(c))["n_resharded"] == 2 * 2
    # router and MLP split after a merged attention: x2 and the normed input again, the other way round
    c = next(c for c in sch.tune_candidates(md["ctx_len"]) if c.form == B.DYN_FORM_MLP_SPLIT)
    assert layer.memory(hb, sch.tune_record(c))["n_resharded"] == 2 * 2


def test_concurrency_keeps_more_alive_than_one_stream():
    """The same split issued on one stream and on two: on one stream a micro-batch's buffers die
    as the next dispatch is issued; on two, what the other stream issued meanwhile may still run."""
    w, md, layer, hb, sch = setup("c2_small")
    chain = B.DENSE_CHAIN
    one = layer.memory(hb, B.nano_schedule(w.nano_rows, chain, streams=[0, 0]))
    two = layer.memory(hb, B.nano_schedule(w.nano_rows, chain))
    seq = layer.memory(hb, B.sequential())
    assert one["peak_live_bytes"] < two["peak_live_bytes"]
    assert one["peak_live_bytes"] <= seq["peak_live_bytes"]


def test_empty_micro_batch_has_no_regions():
    w, md, layer, hb, sch = setup("c2_small")
    rows = tuple(w.nano_rows)
    full = layer.memory(hb, B.nano_schedule(rows, B.DENSE_CHAIN))
    padded = layer.memory(hb, B.nano_schedule((0,) + rows, B.DENSE_CHAIN))
    assert padded["n_regions"] == full["n_regions"]


def test_bad_arguments():
    w, md, layer, hb, sch = setup("c2_small")
    rc = B.lib().dyn_schedule_memory(layer.handle, None, None, None)
    assert rc == B.DYN_ERR_INVALID_ARG
    bad = B.nano_schedule((0, 1, w.n_tokens), B.DENSE_CHAIN[:-1])     # incomplete chain
    with pytest.raises(B.DynError):
        layer.memory(hb, bad)


def _conflict(a, b):
    """Must never share bytes: alive at the same time, or scratch of dispatches on different streams."""
    return bool(a["live"] & b["live"]) or (a["slot"] >= 0 and b["slot"] >= 0 and a["stream"] != b["stream"])


def _check_layout(layer, hb, sched):
    regions = layer.schedule_regions(hb, sched)
    total = layer.schedule_workspace_bytes(hb, sched)
    assert regions and total > 0
    for r in regions:
        assert r["offset"] % 256 == 0 and r["bytes"] > 0 and r["offset"] + r["bytes"] <= total and r["live"]
    for i, a in enumerate(regions):
        for b in regions[i + 1:]:
            if _conflict(a, b):
                assert a["offset"] + a["bytes"] <= b["offset"] or b["offset"] + b["bytes"] <= a["offset"], (a, b)
    assert max(r["offset"] + r["bytes"] for r in regions) > total - 256          # nothing is reserved beyond the last region
    return regions, total


@pytest.mark.parametrize("name", ["c1", "c2_small", "c3_small", "c4_small", "c5_small", "f32_moe_small", "moe_many_b", "stack_mixed"])
def test_layout_never_overlaps_regions_that_can_be_alive_together(name):
    """The workspace layout of every candidate schedule, checked region pair by region pair with
    the rule restated here: the placement may share bytes only between regions that are never
    alive together.  The schedule's need never exceeds the bound that holds for every schedule;
    one stream shares more than several."""
    w, md, layer, hb, sch = setup(name)
    bound = layer.workspace_bytes(w.n_tokens, md["max_pages_per_seq"])
    _, seq_total = _check_layout(layer, hb, B.sequential())
    assert seq_total < bound
    assert layer.memory(hb, B.sequential())["workspace_bytes_schedule"] == seq_total
    for c in sch.tune_candidates(md["ctx_len"], max_k=4, partitions=1):
        sched = sch.tune_record(c, n_cus=256)
        regions, total = _check_layout(layer, hb, sched)
        assert seq_total <= total <= bound
        if c.form != B.DYN_FORM_SEQUENTIAL and c.k > 1:
            tensors = [r for r in regions if r["slot"] < 0]
            assert all(r["live"] == tensors[0]["live"] for r in tensors)           # several streams: every tensor alive throughout
    # micro-batches on one stream are as good as the sequential order for sharing tensors
    one = B.nano_schedule(w.nano_rows, B.MOE_CHAIN if w.shape.n_experts else B.DENSE_CHAIN, streams=[0] * (len(w.nano_rows) - 1))
    regions, total = _check_layout(layer, hb, one)
    assert total < bound and any(r["slot"] < 0 and r["live"] != regions[0]["live"] for r in regions)


def test_sequential_layout_of_the_prefill_decode_mix_shares_most_of_the_workspace():
    """c3 at full size (2048-token chunk + 64 decodes): the any-schedule bound reserves split-K
    planes for every projection and every tensor side by side, about 1.2 GB; the sequential order
    needs the split-KV partials plus what is alive beside them."""
    w, md, layer, hb, sch = setup("c3")
    bound = layer.workspace_bytes(w.n_tokens, md["max_pages_per_seq"])
    regions, total = _check_layout(layer, hb, B.sequential())
    assert bound > 1.1e9 and total < 0.35e9
    by_kind = {r["kind"]: r for r in regions}
    assert "planes" not in by_kind                      # 2112-row launches fold their planes in registers
    # the gated activation reuses bytes of the attention's partials, which are dead by then
    act, part = by_kind["act"], by_kind["part_o"]
    assert not (act["live"] & part["live"])
    assert act["offset"] < part["offset"] + part["bytes"] and part["offset"] < act["offset"] + act["bytes"]
    split = B.nano_schedule(w.nano_rows, stagger=1)
    _, total_split = _check_layout(layer, hb, split)
    assert total < total_split < bound
