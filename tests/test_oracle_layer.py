"""Pins for the oracle's whole-layer function: an independent composition of fp64 library
routines (torch rms_norm / linear / scaled_dot_product_attention / silu on gathered,
contiguous K and V), and invariants of the layer and of batch splitting."""
import dataclasses

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import oracle as orc
from workloads import gen


def library_layer(sh, wts, data, l=0):
    """Decoder layer from library routines, per sequence, on contiguous gathered K/V.
    Returns y [T, H] fp64 and the per-token new k', v (rounded to the cache type)."""
    H, d, nq, nkv, ps = sh.hidden, sh.head_dim, sh.n_q, sh.n_kv, sh.page_size
    W = {k: v.double() for k, v in wts.items()}
    x = data["x"].double()
    kc, vc = data["k_cache"][l].double(), data["v_cache"][l].double()
    bt, q_start, ctx = data["block_table"], data["q_start"], data["ctx_len"]
    inv = 1.0 / (sh.rope_base ** (torch.arange(0, d, 2, dtype=torch.float64) / d))
    y = torch.zeros_like(x)
    newk, newv = {}, {}
    for s in range(len(ctx)):
        r0, r1, c = int(q_start[s]), int(q_start[s + 1]), int(ctx[s])
        n_new = r1 - r0
        xs = x[r0:r1]
        h1 = F.rms_norm(xs, (H,), W["g_norm1"], sh.eps)
        qkv = F.linear(h1, W["w_qkv"])
        q = qkv[:, :nq * d].view(n_new, nq, d)
        k = qkv[:, nq * d:(nq + nkv) * d].view(n_new, nkv, d)
        v = qkv[:, (nq + nkv) * d:].view(n_new, nkv, d)
        pos = torch.arange(c - n_new, c, dtype=torch.float64)
        ang = pos[:, None] * inv[None, :]
        cos, sin = torch.cat([ang.cos(), ang.cos()], 1)[:, None, :], torch.cat([ang.sin(), ang.sin()], 1)[:, None, :]

        def rot(z):  # rotate-half form of the rotary embedding
            z1, z2 = z[..., :d // 2], z[..., d // 2:]
            return z * cos + torch.cat([-z2, z1], -1) * sin

        q, k = rot(q), rot(k)
        k = k.to(sh.torch_dtype).double()
        v = v.to(sh.torch_dtype).double()
        # contiguous K, V [nkv, c, d]: old entries from pages, the last n_new from this step
        pages = torch.as_tensor(bt[s, :(c + ps - 1) // ps].astype(np.int64))
        Kall = kc[pages].permute(1, 0, 2, 3).reshape(nkv, -1, d)[:, :c].clone()
        Vall = vc[pages].permute(1, 0, 3, 2).reshape(nkv, -1, d)[:, :c].clone()
        Kall[:, c - n_new:] = k.permute(1, 0, 2)
        Vall[:, c - n_new:] = v.permute(1, 0, 2)
        mask = torch.ones(n_new, c, dtype=torch.bool).tril(diagonal=c - n_new)
        o = F.scaled_dot_product_attention(q.permute(1, 0, 2)[None], Kall[None], Vall[None], attn_mask=mask,
                                           enable_gqa=True)[0].permute(1, 0, 2).reshape(n_new, nq * d)
        x2 = xs + F.linear(o, W["w_o"])
        h2 = F.rms_norm(x2, (H,), W["g_norm2"], sh.eps)
        if sh.n_experts == 0:
            gu = F.linear(h2, W["w_gate_up"])
            m = F.linear(F.silu(gu[:, :sh.inter]) * gu[:, sh.inter:], W["w_down"])
        else:
            probs = torch.softmax(F.linear(h2, W["w_router"]), dim=-1)
            top = torch.topk(probs, sh.top_k, dim=-1)
            wgt = top.values / top.values.sum(-1, keepdim=True)
            m = torch.zeros_like(h2)
            for t in range(n_new):
                for j in range(sh.top_k):
                    e = int(top.indices[t, j])
                    gu = F.linear(h2[t], W["w_gate_up"][e])
                    m[t] += wgt[t, j] * F.linear(F.silu(gu[:sh.inter]) * gu[sh.inter:], W["w_down"][e])
        y[r0:r1] = x2 + m
        newk[s], newv[s] = k, v
    return y.numpy(), newk, newv


@pytest.mark.parametrize("name", ["f32_small", "f32_moe_small", "c3_small", "c4_small"])
def test_layer_matches_library_composition(name):
    w = gen.config(name)
    w = dataclasses.replace(w, shape=dataclasses.replace(w.shape, n_layers=1))
    data = gen.generate(w)
    y, kcs, vcs = orc.forward(w, data)
    ref, newk, newv = library_layer(w.shape, data["weights"][0], data)
    assert np.allclose(y, ref, rtol=1e-9, atol=1e-10)
    # appended cache entries: right place, right values (to one unit of the storage type)
    ps = w.shape.page_size
    kc = orc.widen(kcs[0], orc.dtype_code(w.shape.dtype))
    vc = orc.widen(vcs[0], orc.dtype_code(w.shape.dtype))
    tol = 2 ** -7 if w.shape.dtype == "bf16" else 1e-6
    for s, (q, c) in enumerate(w.seqs):
        for i in range(q):
            p = c - q + i
            page, slot = data["block_table"][s, p // ps], p % ps
            assert np.allclose(kc[page, :, slot, :], newk[s][i].numpy(), rtol=tol, atol=tol)
            assert np.allclose(vc[page, :, :, slot], newv[s][i].numpy(), rtol=tol, atol=tol)
    # every other cache slot is untouched
    k0 = orc.to_storage(data["k_cache"][0])
    assert (kcs[0] != k0).sum() <= w.n_tokens * w.shape.n_kv * w.shape.head_dim


def test_zero_output_projections_give_identity():
    w = gen.config("f32_small")
    w = dataclasses.replace(w, shape=dataclasses.replace(w.shape, n_layers=1))
    data = gen.generate(w)
    data["weights"][0]["w_o"].zero_()
    data["weights"][0]["w_down"].zero_()
    y, _, _ = orc.forward(w, data)
    assert np.array_equal(y, data["x"].double().numpy())


@pytest.mark.parametrize("name", ["f32_small", "c5_small", "f32_moe_small"])
def test_batch_split_and_sequence_permutation_leave_rows_unchanged(name):
    w = gen.config(name)
    data = gen.generate(w)
    y, kcs, _ = orc.forward(w, data)
    n = w.n_seqs
    # split into two nano-batches at a sequence boundary: every row keeps its bits
    for ids in (list(range(0, n // 2)), list(range(n // 2, n))):
        w2, d2 = gen.sub_batch(w, data, ids)
        y2, _, _ = orc.forward(w2, d2)
        assert np.array_equal(y2, y[d2["rows"]])
    # permuting the sequences permutes the output rows
    ids = list(np.random.default_rng(0).permutation(n))
    w3, d3 = gen.sub_batch(w, data, ids)
    y3, kcs3, _ = orc.forward(w3, d3)
    assert np.array_equal(y3, y[d3["rows"]])
    assert all(np.array_equal(a, b) for a, b in zip(kcs, kcs3))


def test_identical_experts_reduce_to_dense_and_single_expert():
    w = gen.config("f32_moe_small")
    data = gen.generate(w)
    wt = data["weights"][0]
    wt["w_gate_up"][:] = wt["w_gate_up"][0:1]
    wt["w_down"][:] = wt["w_down"][0:1]
    ro = []
    y_moe, _, _ = orc.forward(w, data, routing_out=ro)
    assert np.allclose(ro[0]["wgt"].sum(axis=1), 1.0, rtol=1e-14)
    dense_shape = dataclasses.replace(w.shape, n_experts=0, top_k=0)
    wd = dataclasses.replace(w, shape=dense_shape)
    dd = dict(data)
    dd["weights"] = [dict(wt, w_gate_up=wt["w_gate_up"][0].contiguous(), w_down=wt["w_down"][0].contiguous())]
    y_dense, _, _ = orc.forward(wd, dd)
    assert np.allclose(y_moe, y_dense, rtol=1e-12, atol=1e-13)
    # E = 1, k = 1 is the dense layer
    w1 = dataclasses.replace(w, shape=dataclasses.replace(w.shape, n_experts=1, top_k=1))
    d1 = dict(data)
    d1["weights"] = [dict(wt, w_gate_up=wt["w_gate_up"][:1].contiguous(), w_down=wt["w_down"][:1].contiguous(),
                          w_router=wt["w_router"][:1].contiguous())]
    y1, _, _ = orc.forward(w1, d1)
    assert np.allclose(y1, y_dense, rtol=1e-12, atol=1e-13)


def test_multi_layer_is_composition_of_single_layers():
    w = gen.config("f32_small")           # 2 layers
    data = gen.generate(w)
    y, _, _ = orc.forward(w, data)
    x = data["x"].double().numpy()
    for l in range(2):
        wts = {k: orc.to_storage(v) for k, v in data["weights"][l].items()}
        x = orc.layer_forward(w.shape, wts, x, data["seq_of_token"], data["pos_of_token"], data["block_table"],
                              orc.to_storage(data["k_cache"][l]).copy(), orc.to_storage(data["v_cache"][l]).copy())
    assert np.array_equal(x, y)
