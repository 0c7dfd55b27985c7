"""Full-size parity: the benchmark configurations in the launch configuration bench.py times
(HIP-graph replay, sequential and overlapped schedules), checked on sampled sequences the
oracle can compute one by one (rows are independent per sequence), and bit for bit between
schedules over the whole batch."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2605_21603_amd import binding as B
from workloads import gen

from gpu_util import TOL, GpuRun, as_f64, row_rel_err, say, stack_tol

pytestmark = pytest.mark.gpu


def bench_schedules(w):
    chain = B.MOE_CHAIN if w.shape.n_experts else B.DENSE_CHAIN
    mlp = [B.DYN_OP_GATE_UP, B.DYN_OP_SILU, B.DYN_OP_DOWN]
    return {"sequential": B.sequential(use_graph=True),
            "k2_split_stagger2": B.nano_schedule(w.nano_rows, chain, stagger=2, use_graph=True),
            "k2_mlp_merged_stagger2": B.nano_schedule(w.nano_rows, chain, merged_ops=mlp, stagger=2, use_graph=True)}


def sample_ids(w, n):
    ctx = np.array([c for _, c in w.seqs])
    order = np.argsort(ctx, kind="stable")
    ids = {int(order[0]), int(order[-1])}
    rng = np.random.default_rng(11)
    while len(ids) < n:
        ids.add(int(rng.integers(0, w.n_seqs)))
    return sorted(ids)


@pytest.mark.parametrize("name,n_sample", [("c2", 6), ("c4", 6), ("d300", 6), ("d600", 6), ("d1100", 6)])
def test_decode_configs_full_size(name, n_sample):
    say("case %s: generating" % name)
    w = gen.config(name)
    data = gen.generate(w)
    run = GpuRun(w, data)
    outs = {}
    for label, sched in bench_schedules(w).items():
        say("case %s: schedule %s (graph, replayed 3 times)" % (name, label))
        outs[label] = run.run(sched, repeat=3)
    y0, k0, v0 = outs["sequential"]
    for label, (y, kc, vc) in outs.items():
        assert torch.equal(y.view(torch.uint8), y0.view(torch.uint8)), label
        assert torch.equal(kc.view(torch.uint8), k0.view(torch.uint8)), label
        assert torch.equal(vc.view(torch.uint8), v0.view(torch.uint8)), label
    ids = sample_ids(w, n_sample)
    say("case %s: oracle on sequences %s" % (name, ids))
    w2, d2 = gen.sub_batch(w, data, ids)
    routing = [] if w.shape.n_experts else None
    y_ref, kcs, _ = orc.forward(w2, d2, routing_out=routing)
    y_got = as_f64(y0)[d2["rows"]]
    if routing:
        logits = routing[0]["logits"]
        srt = np.sort(logits, axis=1)[:, ::-1]
        assert (srt[:, w.shape.top_k - 1] - srt[:, w.shape.top_k]).min() > 1e-3, "pick other samples: router near tie"
    err = row_rel_err(y_got, y_ref)
    say("case %s: max rel err %.3e on %d sampled rows" % (name, err, len(ids)))
    assert err <= TOL[w.shape.dtype]
    # appended cache entries of the sampled sequences
    ps = w.shape.page_size
    k_ref = orc.widen(kcs[0], orc.dtype_code(w.shape.dtype))
    k_got = as_f64(k0[0])
    for s in ids:
        p = w.seqs[s][1] - 1
        page, slot = data["block_table"][s, p // ps], p % ps
        scale = np.abs(k_ref[page, :, slot, :]).max()
        assert np.abs(k_got[page, :, slot, :] - k_ref[page, :, slot, :]).max() <= TOL[w.shape.dtype] * scale


def test_prefill_decode_mix_full_size():
    """c3: one 2048-token prefill chunk plus 64 decodes.  The oracle's operators are applied
    in layer order, with keys and values computed for every token of the chunk but the rest
    of the layer only for sampled token rows (a token's output needs the other tokens only
    through the cache)."""
    say("case c3: generating")
    w = gen.config("c3")
    data = gen.generate(w)
    run = GpuRun(w, data)
    outs = {}
    for label, sched in bench_schedules(w).items():
        say("case c3: schedule %s" % label)
        outs[label] = run.run(sched, repeat=2)
    y0, k0, v0 = outs["sequential"]
    for label, (y, kc, vc) in outs.items():
        assert torch.equal(y.view(torch.uint8), y0.view(torch.uint8)), label
        assert torch.equal(kc.view(torch.uint8), k0.view(torch.uint8)), label
    sh = w.shape
    dt = orc.dtype_code(sh.dtype)
    cfg = orc.make_config(sh)
    wt = {k: orc.to_storage(v) for k, v in data["weights"][0].items()}
    d, nq, nkv, H = sh.head_dim, sh.n_q, sh.n_kv, sh.hidden
    x = orc.widen(orc.to_storage(data["x"]), dt)
    say("case c3: oracle keys/values for all %d tokens" % w.n_tokens)
    h1 = orc.rmsnorm(x, wt["g_norm1"], dt, sh.eps)
    kv = orc.linear(h1, wt["w_qkv"][nq * d:], dt)
    k = orc.rope(kv[:, :nkv * d].reshape(-1, nkv, d), data["pos_of_token"], sh.rope_base)
    v = kv[:, nkv * d:].reshape(-1, nkv, d)
    kc, vc = orc.to_storage(data["k_cache"][0]).copy(), orc.to_storage(data["v_cache"][0]).copy()
    orc.cache_append(cfg, k, v, data["seq_of_token"], data["pos_of_token"], data["block_table"], kc, vc)
    rows = np.array(sorted({0, 1, 15, 16, 255, 256, 1000, 2046, 2047, 2048, 2049, 2111} |
                           {int(r) for r in np.random.default_rng(5).integers(0, w.n_tokens, 12)}))
    say("case c3: oracle layer for %d sampled rows" % len(rows))
    q = orc.rope(orc.linear(h1[rows], wt["w_qkv"][:nq * d], dt).reshape(-1, nq, d), data["pos_of_token"][rows], sh.rope_base)
    o = orc.attention(cfg, q, np.ascontiguousarray(data["seq_of_token"][rows]),
                      np.ascontiguousarray(data["pos_of_token"][rows]), data["block_table"], kc, vc)
    x2 = x[rows] + orc.linear(o, wt["w_o"], dt)
    h2 = orc.rmsnorm(x2, wt["g_norm2"], dt, sh.eps)
    y_ref = x2 + orc.linear(orc.silu_mul(orc.linear(h2, wt["w_gate_up"], dt)), wt["w_down"], dt)
    err = row_rel_err(as_f64(y0)[rows], y_ref)
    say("case c3: max rel err %.3e on %d sampled rows" % (err, len(rows)))
    assert err <= TOL[sh.dtype]
    # every key the chunk appended
    k_ref, k_got = orc.widen(kc, dt), as_f64(k0[0])
    pages = data["block_table"][0, :128]
    scale = np.abs(k_ref[pages]).max()
    assert np.abs(k_got[pages] - k_ref[pages]).max() <= TOL[sh.dtype] * scale


def test_32_layer_decode_step_full_size():
    """c5: 32 layers, batch 256, contexts up to 8192 (about 155 GB of cache, generated in
    device memory).  Sequential, 2 and 4 micro-batches on CU-partitioned streams, all as HIP
    graphs; outputs and appended cache entries bit for bit; the oracle runs 4 sampled
    sequences through all 32 layers."""
    free, total = torch.cuda.mem_get_info()
    if total < 200 * 2 ** 30:
        pytest.skip("needs a 288 GB device")
    say("case c5: generating on the device")
    w = gen.config("c5")
    data = gen.generate(w, device="cuda:0", stacked=True)
    layer = B.DynLayer(B.make_config(w.shape), data["weights"])
    step = B.DeviceStep(layer, data)
    st = torch.cuda.Stream()
    ps = w.shape.page_size
    tok_page = torch.as_tensor([int(data["block_table"][s, (c - 1) // ps]) for s, (_, c) in enumerate(w.seqs)], device="cuda:0")
    tok_slot = torch.as_tensor([(c - 1) % ps for _, c in w.seqs], device="cuda:0")

    def run(sched, label):
        say("case c5: schedule %s" % label)
        step.y.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(st):
            for _ in range(2):
                layer.forward(step.batch, sched, st)
        st.synchronize()
        new_k = step.k_cache[:, tok_page, :, tok_slot, :].cpu()
        new_v = step.v_cache[:, tok_page, :, :, tok_slot].cpu()
        return step.y.cpu(), new_k, new_v

    lo, hi = [0x0000FFFF] * 8, [0xFFFF0000] * 8
    y0, k0, v0 = run(B.sequential(use_graph=True), "sequential")
    mlp = [B.DYN_OP_GATE_UP, B.DYN_OP_SILU, B.DYN_OP_DOWN]
    scheds = {"k2 partitioned": B.nano_schedule((0, 128, 256), stagger=2, partitions=[1, 2], cu_masks=[lo, hi], use_graph=True),
              "k4 partitioned, mlp merged": B.nano_schedule((0, 64, 128, 192, 256), merged_ops=mlp, stagger=1, partitions=[1, 2, 1, 2],
                                                            streams=[0, 1, 2, 3], cu_masks=[lo, hi], use_graph=True)}
    for label, sched in scheds.items():
        y, kk, vv = run(sched, label)
        assert torch.equal(y.view(torch.uint8), y0.view(torch.uint8)), label
        assert torch.equal(kk.view(torch.uint8), k0.view(torch.uint8)), label
        assert torch.equal(vv.view(torch.uint8), v0.view(torch.uint8)), label
    ids = sample_ids(w, 4)
    say("case c5: oracle on sequences %s through 32 layers" % ids)
    # the step has already appended this token's keys; the oracle overwrites them with its own
    w2, d2 = gen.extract_sequences(w, data, ids)
    y_ref, _, _ = orc.forward(w2, d2)
    err = row_rel_err(as_f64(y0)[d2["rows"]], y_ref)
    say("case c5: max rel err %.3e on %d sampled rows" % (err, len(ids)))
    assert err <= stack_tol(w.shape.dtype, w.shape.n_layers)
