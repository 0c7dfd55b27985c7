"""Host-side checks that need no GPU: the library loads, exports every symbol the header
declares, and the schedule validator enforces the ready-operator rule."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2605_21603_amd import binding as B
from workloads import gen

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "dynlayer.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dyn_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    names = header_functions()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert hasattr(B.lib(), n), n


def fake_layer(name="c2_small"):
    w = gen.config(name)
    cfg = B.make_config(w.shape)
    fake = {n: 0x1000 for n in ("w_qkv", "w_o", "w_gate_up", "w_down", "g_norm1", "g_norm2")}
    if w.shape.n_experts:
        fake["w_router"] = 0x1000
    return w, B.DynLayer(cfg, [fake] * w.shape.n_layers)


def host_batch(w):
    md = gen.metadata(w)
    q = np.ascontiguousarray(md["q_start"])
    b = B.dyn_batch(w.n_tokens, w.n_seqs, None, None, None, None, None, md["max_pages_per_seq"], q.ctypes.data,
                    None, None, 0, None, 0)
    b._keep = q
    return b


def test_struct_sizes_match_header_layout():
    assert C.sizeof(B.dyn_slot) == 5
    assert C.sizeof(B.dyn_layer_config) == 13 * 4
    assert C.sizeof(B.dyn_slot_time) == 10 * 4


def test_forward_rejects_inconsistent_per_layer_cache_pointers():
    """k_cache_layers / v_cache_layers: both or neither, one non-NULL 16-byte-aligned pointer per
    layer.  The check comes before anything touches a GPU."""
    w, layer = fake_layer("c5_small")
    b = host_batch(w)
    for name in ("x", "seq_of_token", "pos_of_token", "block_table"):
        setattr(b, name, 0x10000)
    b.y = 0x20000
    L = w.shape.n_layers
    good = (C.c_void_p * L)(*[0x100000 * (i + 1) for i in range(L)])
    hole = (C.c_void_p * L)(*([0x100000] * (L - 1) + [None]))
    odd = (C.c_void_p * L)(*([0x100000] * (L - 1) + [0x100008]))
    for k, v, needle in [(good, None, "go together"), (None, good, "go together"), (good, hole, "NULL cache pointer"),
                         (odd, good, "not 16-byte aligned")]:
        b.k_cache_layers = C.cast(k, C.c_void_p) if k is not None else None
        b.v_cache_layers = C.cast(v, C.c_void_p) if v is not None else None
        sc = B.sequential().to_c()
        rc = B.lib().dyn_layer_forward(layer.handle, C.addressof(b), C.addressof(sc), None)
        msg = B.lib().dyn_last_error().decode()
        assert rc == B.DYN_ERR_INVALID_ARG and needle in msg, (rc, msg)


def test_create_rejects_bad_configs():
    w = gen.config("c2_small")
    good = {n: 0x1000 for n in ("w_qkv", "w_o", "w_gate_up", "w_down", "g_norm1", "g_norm2")}
    for field, value, status in [("n_kv_heads", 3, B.DYN_ERR_INVALID_ARG), ("head_dim", 96, B.DYN_ERR_UNSUPPORTED),
                                 ("dtype", 7, B.DYN_ERR_INVALID_ARG), ("hidden", 0, B.DYN_ERR_INVALID_ARG),
                                 ("top_k", 2, B.DYN_ERR_INVALID_ARG), ("mlp_inter", 100, B.DYN_ERR_UNSUPPORTED),
                                 ("kv_chunk_positions", 32, B.DYN_ERR_INVALID_ARG), ("kv_chunk_positions", 1000, B.DYN_ERR_INVALID_ARG),
                                 ("kv_chunk_positions", 131072, B.DYN_ERR_INVALID_ARG)]:
        cfg = B.make_config(w.shape)
        setattr(cfg, field, value)
        with pytest.raises(B.DynError) as e:
            B.DynLayer(cfg, [good])
        assert e.value.status == status, field
    with pytest.raises(B.DynError) as e:
        B.DynLayer(B.make_config(w.shape), [dict(good, w_o=None)])
    assert e.value.status == B.DYN_ERR_INVALID_ARG and "NULL weight" in str(e.value)


def test_sequential_and_generated_schedules_validate():
    for name in ("c2_small", "c3_small", "c5_small", "f32_small"):
        w, layer = fake_layer(name)
        b = host_batch(w)
        layer.validate(b, B.sequential())
        layer.validate(b, B.nano_schedule(w.nano_rows))
        layer.validate(b, B.nano_schedule(w.nano_rows, stagger=2))
        layer.validate(b, B.nano_schedule(w.nano_rows, merged_ops=[B.DYN_OP_GATE_UP, B.DYN_OP_SILU, B.DYN_OP_DOWN], stagger=1))
        layer.validate(b, B.nano_schedule(w.nano_rows, merged_ops=[B.DYN_OP_QKV, B.DYN_OP_DOWN], stagger=3))


def expect_schedule_error(layer, b, sched, needle):
    with pytest.raises(B.DynError) as e:
        layer.validate(b, sched)
    assert e.value.status == B.DYN_ERR_SCHEDULE
    assert needle in str(e.value), str(e.value)


@pytest.mark.parametrize("name", ["c5_small", "c3_small", "c4_small"])
def test_validator_accepts_partitions_by_operator_class(name):
    """A slot's partition need not follow its micro-batch: attention of every micro-batch on
    partition 1, its other operators on partition 2."""
    w, layer = fake_layer(name)
    chain = B.MOE_CHAIN if w.shape.n_experts else B.DENSE_CHAIN
    k = len(w.nano_rows) - 1
    masks = [[0xFFFFFFFF] * 4 + [0] * 4, [0] * 4 + [0xFFFFFFFF] * 4]
    sched = B.nano_schedule(w.nano_rows, chain, stagger=2, partitions=[2] * k, op_partitions={B.DYN_OP_ATTN: 1}, cu_masks=masks)
    assert {s[4] for s in sched.slots if s[0] == B.DYN_OP_ATTN} == {1}
    assert {s[4] for s in sched.slots if s[0] != B.DYN_OP_ATTN} == {2}
    layer.validate(host_batch(w), sched)


def test_validator_rejects_illegal_schedules():
    w, layer = fake_layer("c2_small")        # 13 decode sequences, cut (0, 6, 13)
    b = host_batch(w)
    base = B.nano_schedule(w.nano_rows)
    slots = list(base.slots)
    # out of order: attention of micro-batch 1 before its rope
    i_attn = slots.index((B.DYN_OP_ATTN, 1, 1, 1, 0))
    i_rope = slots.index((B.DYN_OP_ROPE_KV, 1, 1, 1, 0))
    bad = list(slots)
    bad[i_attn], bad[i_rope] = bad[i_rope], bad[i_attn]
    expect_schedule_error(layer, b, B.Schedule(1, w.nano_rows, bad, 2), "before its producer")
    # a merged dispatch needs every covered micro-batch ready
    bad = [s for s in slots if s[0] != B.DYN_OP_QKV]
    k = bad.index((B.DYN_OP_NORM1, 1, 1, 1, 0))
    bad.insert(k, (B.DYN_OP_QKV, 0, 2, 0, 0))       # before norm1 of micro-batch 1
    expect_schedule_error(layer, b, B.Schedule(1, w.nano_rows, bad, 2), "before its producer")
    # missing and duplicated dispatches
    expect_schedule_error(layer, b, B.Schedule(1, w.nano_rows, slots[:-1], 2), "never dispatched")
    expect_schedule_error(layer, b, B.Schedule(1, w.nano_rows, slots + [slots[-1]], 2), "dispatched twice")
    # ids out of range
    expect_schedule_error(layer, b, B.Schedule(1, w.nano_rows, slots, 1), "stream 1 out of range")
    bad = list(slots)
    bad[0] = (B.DYN_OP_NORM1, 0, 1, 0, 2)
    expect_schedule_error(layer, b, B.Schedule(1, w.nano_rows, bad, 2), "partition 2 out of range")
    bad[0] = (B.DYN_OP_NORM1, 1, 2, 0, 0)
    expect_schedule_error(layer, b, B.Schedule(1, w.nano_rows, bad, 2), "outside 0..1")
    bad[0] = (B.DYN_OP_ROUTE, 0, 1, 0, 0)
    expect_schedule_error(layer, b, B.Schedule(1, w.nano_rows, bad, 2), "not part of this layer")
    # cut points
    expect_schedule_error(layer, b, B.Schedule(1, (0, 6, 12), slots, 2), "0 to n_tokens")
    expect_schedule_error(layer, b, B.Schedule(1, (0, 8, 6, 13), B.nano_schedule((0, 8, 6, 13)).slots, 3), "decreases")
    expect_schedule_error(layer, b, B.Schedule(1, tuple(range(0, 10)) + (13,), slots, 2), "k = 10")
    expect_schedule_error(layer, b, B.Schedule(1, w.nano_rows, slots, 2, cu_masks=[[0, 0]]), "empty")
    expect_schedule_error(layer, b, B.Schedule(5), "unknown schedule mode")


def test_cut_inside_a_sequence_is_rejected():
    w, layer = fake_layer("c3_small")        # first sequence has 150 tokens
    b = host_batch(w)
    expect_schedule_error(layer, b, B.nano_schedule((0, 100, w.n_tokens)), "inside a sequence")
    layer.validate(b, B.nano_schedule((0, 150, w.n_tokens)))
    layer.validate(b, B.nano_schedule((0, 0, 150, 150, w.n_tokens)))      # empty micro-batches are legal


def test_batch_shape_errors():
    w, layer = fake_layer("c2_small")
    b = host_batch(w)
    b.n_tokens = 12
    with pytest.raises(B.DynError) as e:
        layer.validate(b, B.sequential())
    assert e.value.status == B.DYN_ERR_INVALID_ARG
    b = host_batch(w)
    b.q_start_host = None
    with pytest.raises(B.DynError) as e:
        layer.validate(b, B.sequential())
    assert e.value.status == B.DYN_ERR_INVALID_ARG


def test_workspace_grows_with_tokens_and_context_not_with_k():
    w, layer = fake_layer("c2_small")
    a = layer.workspace_bytes(16, 8)
    assert a > 0 and a % 256 == 0
    assert layer.workspace_bytes(32, 8) > a
    assert layer.workspace_bytes(16, 64) > a
    assert layer.workspace_bytes(0, 0) >= 0


def test_measurement_probes_reject_bad_arguments_before_touching_the_gpu():
    l = B.lib()
    assert l.dyn_probe_hbm_read(None, 1 << 20, None, None) == B.DYN_ERR_INVALID_ARG
    flops = C.c_double(-1.0)
    buf = C.create_string_buffer(64)                    # a host address: never dereferenced, the sizes are refused first
    p = C.c_void_p((C.addressof(buf) + 15) & ~15)
    assert l.dyn_probe_mfma_loop(None, 16 << 20, 8, p, 1 << 20, None, C.byref(flops)) == B.DYN_ERR_INVALID_ARG
    assert l.dyn_probe_mfma_loop(p, (16 << 20) - 16, 8, p, 1 << 20, None, C.byref(flops)) == B.DYN_ERR_INVALID_ARG     # operands short of 16 MiB
    assert l.dyn_probe_mfma_loop(p, 16 << 20, 8, p, 524288 - 4, None, C.byref(flops)) == B.DYN_ERR_INVALID_ARG         # sink too small
    assert l.dyn_probe_mfma_loop(p, 16 << 20, 0, p, 1 << 20, None, C.byref(flops)) == B.DYN_ERR_INVALID_ARG            # no stages
    assert flops.value == -1.0
    assert b"16777216" in l.dyn_last_error() or b"stages" in l.dyn_last_error()
