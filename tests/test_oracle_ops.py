"""Pins for the oracle's operators: closed forms, invariants, brute force and library
routines in fp64.  None of these re-types the oracle's own loops."""
import math

import numpy as np
import pytest
import torch

from oracle import oracle as orc

RNG = np.random.default_rng(1234)


def bf16_words(a: np.ndarray) -> np.ndarray:
    return orc.to_storage(torch.from_numpy(np.asarray(a, dtype=np.float32)).to(torch.bfloat16))


# ---------------------------------------------------------------- RMSNorm
def test_rmsnorm_hand_value():
    # x = (3, 4): mean square 12.5, so out = x / sqrt(12.5)
    out = orc.rmsnorm(np.array([[3.0, 4.0]]), np.ones(2, np.float32), orc.F32, 0.0)
    assert np.allclose(out, np.array([[3.0, 4.0]]) / math.sqrt(12.5), rtol=1e-15)


def test_rmsnorm_unit_rms_and_scale_invariance():
    x = RNG.normal(size=(5, 64)) * 3.0
    g = np.ones(64, np.float32)
    eps = 1e-6
    out = orc.rmsnorm(x, g, orc.F32, eps)
    ms = (x ** 2).mean(axis=1)
    assert np.allclose(np.sqrt((out ** 2).mean(axis=1)), (1.0 + eps / ms) ** -0.5, rtol=1e-13)
    assert np.allclose(orc.rmsnorm(7.0 * x, g, orc.F32, 0.0), orc.rmsnorm(x, g, orc.F32, 0.0), rtol=1e-13)


def test_rmsnorm_matches_library_and_gain_is_per_column():
    x = RNG.normal(size=(4, 48))
    g = RNG.normal(size=48).astype(np.float32)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (48,), torch.from_numpy(g).double(), 1e-5).numpy()
    assert np.allclose(orc.rmsnorm(x, g, orc.F32, 1e-5), ref, rtol=1e-12, atol=1e-14)


def test_rmsnorm_bf16_gain_is_widened_exactly():
    x = RNG.normal(size=(2, 16))
    g = RNG.normal(size=16).astype(np.float32)
    gw = bf16_words(g)
    g_exact = torch.from_numpy(g).to(torch.bfloat16).double().numpy()
    ref = x / np.sqrt((x ** 2).mean(axis=1, keepdims=True) + 1e-6) * g_exact
    assert np.allclose(orc.rmsnorm(x, gw, orc.BF16, 1e-6), ref, rtol=1e-13)


# ---------------------------------------------------------------- linear
def test_linear_matches_matmul_nonsquare():
    x = RNG.normal(size=(3, 37))
    W = RNG.normal(size=(11, 37)).astype(np.float32)
    assert np.allclose(orc.linear(x, W, orc.F32), x @ W.astype(np.float64).T, rtol=1e-12, atol=1e-13)


def test_linear_identity_and_bf16():
    x = RNG.normal(size=(4, 8))
    assert np.array_equal(orc.linear(x, np.eye(8, dtype=np.float32), orc.F32), x)
    W = RNG.normal(size=(5, 8)).astype(np.float32)
    Wb = torch.from_numpy(W).to(torch.bfloat16)
    assert np.allclose(orc.linear(x, orc.to_storage(Wb), orc.BF16), x @ Wb.double().numpy().T, rtol=1e-12, atol=1e-13)


def test_widen_bf16_exact():
    vals = np.array([1.0, -2.5, 3.140625, 1e-3, 65280.0], np.float32)
    tb = torch.from_numpy(vals).to(torch.bfloat16)
    assert np.array_equal(orc.widen(orc.to_storage(tb), orc.BF16), tb.double().numpy())


# ---------------------------------------------------------------- RoPE
def test_rope_position_zero_is_identity():
    z = RNG.normal(size=(3, 2, 8))
    assert np.array_equal(orc.rope(z, np.zeros(3, np.int32), 10000.0), z)


def test_rope_d2_closed_form():
    # d = 2: one pair, theta_0 = 1, a plain rotation by p radians
    z = np.array([[[1.0, 0.0]], [[0.3, -0.7]]])
    pos = np.array([2, 5], np.int32)
    out = orc.rope(z, pos, 10000.0)
    for t, p in enumerate(pos):
        a, b = z[t, 0]
        assert np.allclose(out[t, 0], [a * math.cos(p) - b * math.sin(p), b * math.cos(p) + a * math.sin(p)], rtol=1e-14)


def test_rope_frequencies_and_pairing():
    # unit vector on coordinate i (first half) rotates into coordinates (i, i + d/2) by p * base^(-2i/d)
    d, base, p = 8, 100.0, 3
    for i in range(d // 2):
        z = np.zeros((1, 1, d))
        z[0, 0, i] = 1.0
        out = orc.rope(z, np.array([p], np.int32), base)[0, 0]
        ang = p * base ** (-2.0 * i / d)
        exp = np.zeros(d)
        exp[i], exp[i + d // 2] = math.cos(ang), math.sin(ang)
        assert np.allclose(out, exp, atol=1e-15)


def test_rope_norm_and_relative_position():
    d = 16
    q, k = RNG.normal(size=(1, 1, d)), RNG.normal(size=(1, 1, d))
    dots = []
    for m, n in ((5, 2), (13, 10), (103, 100)):
        qm = orc.rope(q, np.array([m], np.int32), 10000.0)
        kn = orc.rope(k, np.array([n], np.int32), 10000.0)
        assert np.allclose(np.linalg.norm(qm), np.linalg.norm(q), rtol=1e-13)
        for i in range(d // 2):   # each pair keeps its own norm
            assert np.isclose(qm[0, 0, i] ** 2 + qm[0, 0, i + d // 2] ** 2, q[0, 0, i] ** 2 + q[0, 0, i + d // 2] ** 2, rtol=1e-12)
        dots.append(float((qm * kn).sum()))
    assert np.allclose(dots, dots[0], rtol=1e-11)


# ---------------------------------------------------------------- SiLU gate
def test_silu_identities():
    z = np.array([[0.0, 1.5, -1.5, 40.0, -40.0]])
    ones = np.ones_like(z)
    s = orc.silu_mul(np.concatenate([z, ones], axis=1))[0]
    assert s[0] == 0.0
    assert np.isclose(s[1] - s[2], 1.5, rtol=1e-14)          # silu(z) - silu(-z) = z
    assert np.isclose(s[3], 40.0, rtol=1e-14) and abs(s[4]) < 1e-15
    gu = RNG.normal(size=(3, 10))
    ref = (torch.nn.functional.silu(torch.from_numpy(gu[:, :5])) * torch.from_numpy(gu[:, 5:])).numpy()
    assert np.allclose(orc.silu_mul(gu), ref, rtol=1e-13)     # gate is the first half, up the second


# ---------------------------------------------------------------- paged attention
def make_cache(n_seqs, ctxs, n_kv, d, ps, dtype, seed):
    rng = np.random.default_rng(seed)
    pages_per = [(c + ps - 1) // ps for c in ctxs]
    n_pages = sum(pages_per) + 2
    perm = rng.permutation(n_pages).astype(np.int32)
    bt = np.full((n_seqs, max(pages_per)), -12345, np.int32)
    i = 0
    for s, n in enumerate(pages_per):
        bt[s, :n] = perm[i:i + n]
        i += n
    bt[bt == -12345] = 0
    k = rng.normal(size=(n_pages, n_kv, ps, d)).astype(np.float32)
    v = rng.normal(size=(n_pages, n_kv, d, ps)).astype(np.float32)
    if dtype == orc.BF16:
        kb, vb = torch.from_numpy(k).to(torch.bfloat16), torch.from_numpy(v).to(torch.bfloat16)
        return bt, orc.to_storage(kb), orc.to_storage(vb), kb.double().numpy(), vb.double().numpy()
    return bt, k, v, k.astype(np.float64), v.astype(np.float64)


def gather_kv(bt, kf, vf, s, g, n, ps):
    """Contiguous K [n, d] and V [n, d] of sequence s, kv head g, from the paged arrays."""
    K = np.stack([kf[bt[s, j // ps], g, j % ps, :] for j in range(n)])
    V = np.stack([vf[bt[s, j // ps], g, :, j % ps] for j in range(n)])
    return K, V


def brute_attention(q, seq, pos, bt, kf, vf, n_q, n_kv, d, ps):
    T = q.shape[0]
    out = np.zeros((T, n_q * d))
    for t in range(T):
        for h in range(n_q):
            K, V = gather_kv(bt, kf, vf, seq[t], h // (n_q // n_kv), pos[t] + 1, ps)
            s = K @ q[t, h] / math.sqrt(d)
            p = np.exp(s - s.max())
            p /= p.sum()
            out[t, h * d:(h + 1) * d] = p @ V
    return out


def attn_cfg(n_q, n_kv, d, ps, dtype):
    return orc.Config(dtype, 0, n_q, n_kv, d, 0, 0, 0, 1e-6, 10000.0, ps)


@pytest.mark.parametrize("dtype", [orc.F32, orc.BF16])
def test_attention_brute_force_gqa_ragged(dtype):
    n_q, n_kv, d, ps = 6, 2, 8, 4
    ctxs = [1, 4, 5, 11, 16]
    bt, k, v, kf, vf = make_cache(5, ctxs, n_kv, d, ps, dtype, 3)
    # mixed: decode tokens and a multi-token (causal) group for sequence 3
    seq = np.array([0, 1, 2, 3, 3, 3, 4], np.int32)
    pos = np.array([0, 3, 4, 8, 9, 10, 15], np.int32)
    q = RNG.normal(size=(7, n_q, d))
    out, probs = orc.attention(attn_cfg(n_q, n_kv, d, ps, dtype), q, seq, pos, bt, k, v, want_probs=16)
    assert np.allclose(out, brute_attention(q, seq, pos, bt, kf, vf, n_q, n_kv, d, ps), rtol=1e-11, atol=1e-13)
    assert np.allclose(probs.sum(axis=2), 1.0, rtol=1e-13)              # softmax rows sum to one
    for t in range(7):                                                    # nothing beyond the own position
        assert np.all(probs[t, :, pos[t] + 1:] == 0.0)


def test_attention_matches_library_sdpa():
    n_q, n_kv, d, ps, n = 4, 2, 16, 8, 21
    bt, k, v, kf, vf = make_cache(1, [n], n_kv, d, ps, orc.F32, 9)
    q = RNG.normal(size=(1, n_q, d))
    out = orc.attention(attn_cfg(n_q, n_kv, d, ps, orc.F32), q, np.zeros(1, np.int32), np.array([n - 1], np.int32), bt, k, v)
    Ks, Vs = zip(*[gather_kv(bt, kf, vf, 0, g, n, ps) for g in range(n_kv)])
    K = torch.from_numpy(np.stack(Ks))[None]        # [1, n_kv, n, d]
    V = torch.from_numpy(np.stack(Vs))[None]
    Q = torch.from_numpy(q).permute(1, 0, 2)[None]   # [1, n_q, 1, d]
    ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V, enable_gqa=True)[0, :, 0, :].reshape(-1).numpy()
    assert np.allclose(out[0], ref, rtol=1e-11, atol=1e-13)


def test_attention_special_cases():
    n_q, n_kv, d, ps = 4, 2, 8, 4
    bt, k, v, kf, vf = make_cache(2, [1, 9], n_kv, d, ps, orc.F32, 5)
    cfg = attn_cfg(n_q, n_kv, d, ps, orc.F32)
    q = RNG.normal(size=(2, n_q, d))
    seq, pos = np.array([0, 1], np.int32), np.array([0, 8], np.int32)
    out = orc.attention(cfg, q, seq, pos, bt, k, v)
    for h in range(n_q):                                                  # one key: output is its value
        assert np.allclose(out[0, h * d:(h + 1) * d], vf[bt[0, 0], h // 2, :, 0], rtol=1e-15)
    v_same = v.copy()
    row = RNG.normal(size=(n_kv, d)).astype(np.float32)
    v_same[:] = row[None, :, :, None]
    out = orc.attention(cfg, q, seq, pos, bt, k, v_same)                 # equal values: output is that value
    for h in range(n_q):
        assert np.allclose(out[1, h * d:(h + 1) * d], row[h // 2], rtol=1e-13)


def test_attention_gqa_equals_mha_with_replicated_kv_and_page_permutation():
    n_q, n_kv, d, ps = 4, 2, 8, 4
    ctxs = [7, 12]
    bt, k, v, kf, vf = make_cache(2, ctxs, n_kv, d, ps, orc.F32, 6)
    q = RNG.normal(size=(2, n_q, d))
    seq, pos = np.array([0, 1], np.int32), np.array([6, 11], np.int32)
    out = orc.attention(attn_cfg(n_q, n_kv, d, ps, orc.F32), q, seq, pos, bt, k, v)
    k_rep, v_rep = np.repeat(k, 2, axis=1), np.repeat(v, 2, axis=1)
    out_mha = orc.attention(attn_cfg(n_q, n_q, d, ps, orc.F32), q, seq, pos, bt, k_rep, v_rep)
    assert np.array_equal(out, out_mha)
    perm = np.random.default_rng(0).permutation(k.shape[0])
    inv = np.argsort(perm).astype(np.int32)
    out_perm = orc.attention(attn_cfg(n_q, n_kv, d, ps, orc.F32), q, seq, pos, inv[bt], k[perm], v[perm])
    assert np.array_equal(out, out_perm)


def test_prefill_rows_equal_decode_rows():
    # a causal multi-token group gives, per token, what a decode step at that position gives
    n_q, n_kv, d, ps, n = 4, 2, 8, 4, 10
    bt, k, v, _, _ = make_cache(1, [n], n_kv, d, ps, orc.F32, 8)
    cfg = attn_cfg(n_q, n_kv, d, ps, orc.F32)
    q = RNG.normal(size=(n, n_q, d))
    full = orc.attention(cfg, q, np.zeros(n, np.int32), np.arange(n, dtype=np.int32), bt, k, v)
    for t in range(n):
        one = orc.attention(cfg, q[t:t + 1], np.zeros(1, np.int32), np.array([t], np.int32), bt, k, v)
        assert np.array_equal(one[0], full[t])


def test_cache_append_places_and_rounds():
    n_kv, d, ps = 2, 4, 4
    cfg = attn_cfg(2, n_kv, d, ps, orc.BF16)
    bt, k, v, _, _ = make_cache(2, [6, 3], n_kv, d, ps, orc.BF16, 2)
    k0, v0 = k.copy(), v.copy()
    newk, newv = RNG.normal(size=(2, n_kv, d)), RNG.normal(size=(2, n_kv, d))
    seq, pos = np.array([0, 1], np.int32), np.array([5, 2], np.int32)
    orc.cache_append(cfg, newk, newv, seq, pos, bt, k, v)
    changed_k, changed_v = np.argwhere(k != k0), np.argwhere(v != v0)
    for t in range(2):
        page, slot = bt[seq[t], pos[t] // ps], pos[t] % ps
        want_k = orc.to_storage(torch.from_numpy(newk[t].astype(np.float32)).to(torch.bfloat16))
        want_v = orc.to_storage(torch.from_numpy(newv[t].astype(np.float32)).to(torch.bfloat16))
        assert np.array_equal(k[page, :, slot, :], want_k)
        assert np.array_equal(v[page, :, :, slot], want_v)
    pages = {int(bt[seq[t], pos[t] // ps]) for t in range(2)}
    assert set(changed_k[:, 0]) <= pages and set(changed_v[:, 0]) <= pages
    assert len(changed_k) <= 2 * n_kv * d and len(changed_v) <= 2 * n_kv * d


# ---------------------------------------------------------------- router
def test_route_topk_softmax_and_ties():
    H, E = 6, 5
    Wr = np.zeros((E, H), np.float32)
    h = np.zeros((3, H))
    # logits = h[:, :E] because Wr picks coordinates
    for e in range(E):
        Wr[e, e] = 1.0
    h[0, :E] = [0.1, 2.0, -1.0, 1.0, 0.5]
    h[1, :E] = [3.0, 3.0, 3.0, 0.0, 0.0]          # tie: lower indices win
    h[2, :E] = [-5.0, -4.0, -3.0, -2.0, -1.0]
    sel, wgt, logits = orc.route(h, Wr, 2)
    assert np.array_equal(sel, [[1, 3], [0, 1], [4, 3]])
    assert np.allclose(wgt.sum(axis=1), 1.0, rtol=1e-15)
    assert np.allclose(wgt[0], np.array([math.e, 1.0]) / (math.e + 1.0), rtol=1e-14)
    assert np.allclose(wgt[1], [0.5, 0.5]) and np.allclose(logits, h[:, :E])
    full = torch.softmax(torch.from_numpy(logits), dim=1).numpy()       # softmax over all, renormalised
    renorm = np.take_along_axis(full, sel.astype(np.int64), axis=1)
    assert np.allclose(wgt, renorm / renorm.sum(axis=1, keepdims=True), rtol=1e-13)
    sel2, wgt2, _ = orc.route(h, Wr, 2, forced_sel=np.array([[3, 1], [2, 0], [0, 1]], np.int32))
    assert np.array_equal(sel2, [[3, 1], [2, 0], [0, 1]])
    assert np.allclose(wgt2[0], np.array([1.0, math.e]) / (math.e + 1.0), rtol=1e-14)
