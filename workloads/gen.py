"""Seeded synthetic inputs for the decoder-layer forward step.

This module is shared by the CPU oracle's tests and by the HIP path's tests and
benchmark.  It holds no arithmetic of the method: it only draws random numbers,
rounds stored values to their storage type and lays them out in the documented
tensor formats.

Tensor formats (all row-major, the last index fastest):

  x            [n_tokens, hidden]
  w_qkv        [(n_q + 2 n_kv) * d, hidden]   rows: all q heads, then k heads, then v heads
  w_o          [hidden, n_q * d]
  w_gate_up    [2 * inter, hidden]            rows: gate rows, then up rows   (dense MLP)
               [E, 2 * inter, hidden]                                          (MoE)
  w_down       [hidden, inter]   /  [E, hidden, inter]
  w_router     [E, hidden]   (fp32 in every configuration)
  g_norm1/2    [hidden]
  k_cache      [n_pages, n_kv, page_size, d]  a page holds page_size consecutive positions
  v_cache      [n_pages, n_kv, d, page_size]  (V is stored position-fastest inside a page)
  block_table  [n_seqs, max_pages_per_seq]    int32 physical page of logical page j
  seq_of_token, pos_of_token [n_tokens] int32;  q_start [n_seqs+1];  ctx_len [n_seqs]

Every weight matrix is stored "output-major": y = x @ W^T.  ctx_len counts the keys a
sequence attends to after this step's tokens have been appended.

Workload shapes follow the paper's evaluation section only in shape (Llama-3-8B layer
sizes, batches of hundreds of sequences with contexts of 0.5k-8k tokens, a prefill
chunk mixed with decodes); values are N(0, 0.02^2) weights, N(0, 1) activations and
cache entries, unit norm gains.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np
import torch


@dataclass(frozen=True)
class LayerShape:
    dtype: str            # "f32" | "bf16"
    hidden: int
    n_q: int
    n_kv: int
    head_dim: int
    inter: int
    n_layers: int = 1
    n_experts: int = 0
    top_k: int = 0
    eps: float = 1e-6
    rope_base: float = 10000.0
    page_size: int = 16

    @property
    def qkv_rows(self) -> int:
        return (self.n_q + 2 * self.n_kv) * self.head_dim

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


@dataclass(frozen=True)
class Workload:
    name: str
    shape: LayerShape
    # one entry per sequence: (q_len, ctx_len) with ctx_len >= q_len; the q_len new
    # tokens occupy positions ctx_len - q_len .. ctx_len - 1.
    seqs: Tuple[Tuple[int, int], ...]
    seed: int = 0
    nano_rows: Tuple[int, ...] = ()      # default token-row cut points [0, ..., n_tokens]

    @property
    def n_tokens(self) -> int:
        return sum(q for q, _ in self.seqs)

    @property
    def n_seqs(self) -> int:
        return len(self.seqs)


LLAMA3_8B = LayerShape("bf16", 4096, 32, 8, 128, 14336)
MOE_8X = dataclasses.replace(LLAMA3_8B, n_experts=8, top_k=2)


def _uniform_ctx(seed: int, n: int, lo: int, hi: int) -> List[int]:
    rng = np.random.default_rng(seed)
    return [int(v) for v in rng.integers(lo, hi + 1, size=n)]


def mixed(prefill_tokens: int, n_decode: int, decode_ctx: int, shape: LayerShape = LLAMA3_8B, seed: int = 0) -> Workload:
    """One prefill chunk with no prior context followed by n_decode single-token sequences
    that all attend decode_ctx keys (the shape family of configuration 3); either part may
    be absent.  Default cut: the prefill / decode boundary."""
    seqs = (((prefill_tokens, prefill_tokens),) if prefill_tokens else ()) + tuple((1, decode_ctx) for _ in range(n_decode))
    T = prefill_tokens + n_decode
    return Workload("mix_p%d_d%dx%d" % (prefill_tokens, n_decode, decode_ctx), shape, seqs, seed,
                    (0, prefill_tokens, T) if prefill_tokens and n_decode else (0, T))


def config(name: str) -> Workload:
    """The named workloads: c1..c5 are the five benchmark configurations, the *_small
    ones are reduced shapes the CPU oracle finishes in seconds."""
    if name == "c1":
        sh = LayerShape("f32", 256, 4, 4, 64, 1024)
        return Workload("c1", sh, tuple((1, 128) for _ in range(4)), 0, (0, 2, 4))
    if name == "c2":
        ctx = _uniform_ctx(0, 128, 512, 4096)
        return Workload("c2", LLAMA3_8B, tuple((1, c) for c in ctx), 0, (0, 64, 128))
    if name == "c3":
        seqs = ((2048, 2048),) + tuple((1, 2048) for _ in range(64))
        return Workload("c3", LLAMA3_8B, seqs, 0, (0, 2048, 2112))
    if name == "c4":
        return Workload("c4", MOE_8X, tuple((1, 1024) for _ in range(256)), 0, (0, 128, 256))
    if name == "c5":
        ctx = _uniform_ctx(0, 256, 1024, 8192)
        sh = dataclasses.replace(LLAMA3_8B, n_layers=32)
        return Workload("c5", sh, tuple((1, c) for c in ctx), 0, (0, 128, 256))
    if name == "c5_layer":      # one layer of c5 (same sequences): quick operator-level measurements of the 256-row decode regime
        ctx = _uniform_ctx(0, 256, 1024, 8192)
        return Workload("c5_layer", LLAMA3_8B, tuple((1, c) for c in ctx), 0, (0, 128, 256))
    if name == "d300":          # full layer shape at 300 rows: the 384-row projection tile next to 256-row tiles when split
        ctx = _uniform_ctx(20, 300, 1, 300)
        return Workload("d300", LLAMA3_8B, tuple((1, c) for c in ctx), 20, (0, 150, 300))
    if name == "d600":          # 600 rows of the full layer shape: two 256 x 256 m tiles and the last 88 rows in a launch of their own
        ctx = _uniform_ctx(21, 600, 1, 200)
        return Workload("d600", LLAMA3_8B, tuple((1, c) for c in ctx), 21, (0, 300, 600))
    if name == "d1100":         # 1100 rows of the full layer shape: down as two 512-row tiles + 76 rows, gate/up as four wide m tiles + 76 rows
        ctx = _uniform_ctx(22, 1100, 1, 120)
        return Workload("d1100", LLAMA3_8B, tuple((1, c) for c in ctx), 22, (0, 500, 1100))
    if name == "c2_small":
        sh = LayerShape("bf16", 512, 8, 2, 128, 1536)
        ctx = _uniform_ctx(1, 13, 1, 700)
        return Workload("c2_small", sh, tuple((1, c) for c in ctx), 1, (0, 6, 13))
    if name == "c3_small":
        sh = LayerShape("bf16", 512, 8, 2, 128, 1536)
        seqs = ((150, 150), (1, 77), (37, 90), (1, 300), (1, 1))
        return Workload("c3_small", sh, seqs, 2, (0, 150, 190))
    if name == "c3_mid":        # enough rows for the many-row GEMM path, a long prefill chunk next to decodes
        sh = LayerShape("bf16", 1024, 8, 2, 128, 2048)
        seqs = ((2700, 2700),) + tuple((1, c) for c in _uniform_ctx(8, 20, 1, 600)) + ((96, 130),)
        return Workload("c3_mid", sh, seqs, 8, (0, 2700, 2816))
    if name == "c4_small":
        sh = LayerShape("bf16", 512, 8, 2, 128, 1024, n_experts=8, top_k=2)
        ctx = _uniform_ctx(3, 40, 1, 200)
        return Workload("c4_small", sh, tuple((1, c) for c in ctx), 3, (0, 17, 40))
    if name == "c5_small":
        sh = LayerShape("bf16", 512, 8, 2, 128, 1536, n_layers=3)
        ctx = _uniform_ctx(4, 24, 1, 520)
        return Workload("c5_small", sh, tuple((1, c) for c in ctx), 4, (0, 5, 11, 18, 24))
    if name == "stack_mixed":   # three layers over prefill chunks and decodes: later layers walk layer 0's attention work lists
        sh = LayerShape("bf16", 512, 8, 2, 128, 1024, n_layers=3)
        seqs = ((90, 1300), (1, 700), (1, 20), (40, 40), (1, 1), (1, 1025), (6, 300))
        return Workload("stack_mixed", sh, seqs, 17, (0, 92, 140))
    if name == "pf_long":       # a prefill chunk after 2300 cached positions: several 1024-position chunks per query block
        sh = LayerShape("bf16", 512, 8, 2, 128, 1024)
        seqs = ((200, 2500), (1, 1100), (70, 70), (1, 33), (3, 1027))
        return Workload("pf_long", sh, seqs, 9, (0, 200, 275))
    if name == "pf_deep":       # prefill chunks behind 8..66 thousand cached positions: split-KV chunks of 2048, 4096 and 8192 positions,
                                # and a sequence whose blocks straddle the 8192-key step (1024- and 2048-position chunks side by side)
        sh = LayerShape("bf16", 512, 8, 2, 128, 1024)
        seqs = ((100, 9000), (1, 8200), (30, 17000), (70, 8230), (3, 66000), (1, 40))
        return Workload("pf_deep", sh, seqs, 23, (0, 101, 205))
    if name == "dec_deep":      # decodes behind 16 to 70 thousand cached positions: 64, 65, 79 and 274 split-KV chunks (two-level merge above 64)
        sh = LayerShape("bf16", 512, 8, 2, 128, 1024)
        seqs = ((1, 20000), (1, 70000), (1, 16384), (1, 16385), (1, 300), (5, 130))
        return Workload("dec_deep", sh, seqs, 27, (0, 2, 10))
    if name == "pf_g8":         # eight q heads per kv head: two tokens per 16-column set, 32-token query blocks
        sh = LayerShape("bf16", 1024, 8, 1, 128, 1024)
        seqs = ((45, 45), (1, 300), (33, 1090), (1, 1))
        return Workload("pf_g8", sh, seqs, 10, (0, 46, 80))
    if name == "pf_mha":        # one q head per kv head: sixteen tokens per set, 256-token query blocks
        sh = LayerShape("bf16", 512, 4, 4, 128, 1024)
        seqs = ((300, 300), (1, 77), (20, 400))
        return Workload("pf_mha", sh, seqs, 11, (0, 300, 321))
    if name == "pf_g16":        # sixteen q heads on one kv head: one token per 16-column set
        sh = LayerShape("bf16", 512, 16, 1, 128, 512)
        seqs = ((21, 21), (1, 500), (1, 16), (18, 1040), (1, 1), (1, 257))
        return Workload("pf_g16", sh, seqs, 18, (0, 22, 43))
    if name == "pf_g2":         # two q heads per kv head: eight tokens per set, 128-token query blocks
        sh = LayerShape("bf16", 512, 4, 2, 128, 512)
        seqs = ((1, 333), (140, 140), (1, 17), (70, 1200), (1, 1024))
        return Workload("pf_g2", sh, seqs, 19, (0, 141, 213))
    if name == "pf_480":        # 385..512 rows: one 512-row tile per (n tile, plane) of the projections with planes
        sh = LayerShape("bf16", 1024, 8, 2, 128, 2048)
        seqs = ((440, 440),) + tuple((1, c) for c in _uniform_ctx(12, 30, 1, 500)) + ((10, 700),)
        return Workload("pf_480", sh, seqs, 12, (0, 440, 480))
    if name == "pf_640":        # 513..1024 rows: two tall tiles
        sh = LayerShape("bf16", 1024, 8, 2, 128, 2048)
        seqs = ((300, 300), (290, 1400)) + tuple((1, c) for c in _uniform_ctx(13, 50, 1, 400))
        return Workload("pf_640", sh, seqs, 13, (0, 590, 640))
    if name == "bf16_hd64":     # head_dim 64: outside the matrix-core attention kernels, the generic path in bf16
        sh = LayerShape("bf16", 256, 4, 2, 64, 512)
        seqs = ((23, 23), (1, 70), (1, 200), (9, 41), (1, 1))
        return Workload("bf16_hd64", sh, seqs, 14, (0, 24, 35))
    if name == "bf16_ps32":     # 32-position pages with head_dim 128: also the generic attention path
        sh = LayerShape("bf16", 512, 4, 2, 128, 512, page_size=32)
        seqs = ((1, 33), (40, 100), (1, 64), (1, 129))
        return Workload("bf16_ps32", sh, seqs, 15, (0, 41, 43))
    if name == "bf16_max":      # the largest head_dim and expert count the layer accepts, 64-position pages
        sh = LayerShape("bf16", 256, 2, 1, 256, 128, n_experts=16, top_k=4, page_size=64)
        seqs = ((1, 65), (17, 17), (1, 300), (5, 130), (1, 1), (1, 64))
        return Workload("bf16_max", sh, seqs, 16, (0, 18, 26))
    if name == "moe_mid":       # about 150 rows per expert: one 256-row tile per expert and n tile
        sh = LayerShape("bf16", 512, 8, 2, 128, 1024, n_experts=4, top_k=2)
        return Workload("moe_mid", sh, tuple((1, c) for c in _uniform_ctx(24, 300, 1, 60)), 24, (0, 140, 300))
    if name == "moe_many_a":    # about 350 rows per expert: 256 x 256 tiles for the gated gate/up, planes for down
        sh = LayerShape("bf16", 512, 8, 2, 128, 1024, n_experts=4, top_k=2)
        return Workload("moe_many_a", sh, tuple((1, c) for c in _uniform_ctx(25, 700, 1, 40)), 25, (0, 300, 700))
    if name == "moe_many_b":    # the other way round: gate/up with planes (not gated), 256 x 256 tiles for down
        sh = LayerShape("bf16", 1024, 8, 2, 128, 512, n_experts=4, top_k=2)
        return Workload("moe_many_b", sh, tuple((1, c) for c in _uniform_ctx(26, 700, 1, 40)), 26, (0, 300, 700))
    if name == "shallow_a":     # contractions of one and two 64-deep stages (hidden 128, MLP width 64) under the 256-row tall tile
        sh = LayerShape("bf16", 128, 1, 1, 128, 64)
        return Workload("shallow_a", sh, tuple((1, c) for c in _uniform_ctx(28, 200, 1, 40)), 28, (0, 130, 200))
    if name == "shallow_b":     # the same depths under the 384-row tall tile, a prefill chunk among the rows
        sh = LayerShape("bf16", 128, 1, 1, 128, 64)
        seqs = ((150, 150),) + tuple((1, c) for c in _uniform_ctx(29, 190, 1, 40))
        return Workload("shallow_b", sh, seqs, 29, (0, 150, 340))
    if name == "shallow_wide":  # two stages deep under the 256 x 256 tile (gate/up 1536 x 8192 x 128), 64 stages for down
        sh = LayerShape("bf16", 128, 1, 1, 128, 4096)
        return Workload("shallow_wide", sh, tuple((1, c) for c in _uniform_ctx(30, 1536, 1, 8)), 30, (0, 768, 1536))
    if name == "f32_small":
        sh = LayerShape("f32", 128, 4, 2, 32, 320, n_layers=2)
        seqs = ((9, 9), (1, 40), (1, 17), (5, 21), (1, 1))
        return Workload("f32_small", sh, seqs, 5, (0, 9, 17))
    if name == "f32_moe_small":
        sh = LayerShape("f32", 128, 4, 2, 32, 192, n_experts=4, top_k=2)
        ctx = _uniform_ctx(6, 11, 1, 50)
        return Workload("f32_moe_small", sh, tuple((1, c) for c in ctx), 6, (0, 4, 11))
    raise KeyError(name)


def round_to(t: torch.Tensor, dtype: str) -> torch.Tensor:
    """Round fp32 values to the storage type (round-to-nearest-even for bf16)."""
    return t.to(torch.bfloat16) if dtype == "bf16" else t.to(torch.float32)


def metadata(w: Workload, page_seed: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Token/sequence index arrays and a block table with randomly permuted physical pages."""
    ps = w.shape.page_size
    seq_of_token, pos_of_token, q_start, ctx_len = [], [], [0], []
    for s, (q, c) in enumerate(w.seqs):
        assert 1 <= q <= c
        for i in range(q):
            seq_of_token.append(s)
            pos_of_token.append(c - q + i)
        q_start.append(q_start[-1] + q)
        ctx_len.append(c)
    pages_per_seq = [(c + ps - 1) // ps for _, c in w.seqs]
    max_pages = max(pages_per_seq)
    n_pages = sum(pages_per_seq) + 3                       # a few spare pages never referenced
    rng = np.random.default_rng((w.seed if page_seed is None else page_seed) + 7919)
    perm = rng.permutation(n_pages).astype(np.int32)
    bt = np.zeros((w.n_seqs, max_pages), dtype=np.int32)
    nxt = 0
    for s, n in enumerate(pages_per_seq):
        bt[s, :n] = perm[nxt:nxt + n]
        nxt += n
    return dict(
        seq_of_token=np.asarray(seq_of_token, dtype=np.int32),
        pos_of_token=np.asarray(pos_of_token, dtype=np.int32),
        q_start=np.asarray(q_start, dtype=np.int32),
        ctx_len=np.asarray(ctx_len, dtype=np.int32),
        block_table=bt, n_pages=n_pages, max_pages_per_seq=max_pages,
    )


def _normal(gen: torch.Generator, shape, std: float, dtype: str, device="cpu") -> torch.Tensor:
    t = torch.empty(shape, dtype=torch.float32, device=device)
    t.normal_(0.0, std, generator=gen)
    return round_to(t, dtype)


def layer_weights(sh: LayerShape, gen: torch.Generator, device="cpu") -> Dict[str, torch.Tensor]:
    H, I, E = sh.hidden, sh.inter, sh.n_experts
    wts = {
        "w_qkv": _normal(gen, (sh.qkv_rows, H), 0.02, sh.dtype, device),
        "w_o": _normal(gen, (H, sh.n_q * sh.head_dim), 0.02, sh.dtype, device),
        "g_norm1": round_to(torch.ones(H, device=device), sh.dtype),
        "g_norm2": round_to(torch.ones(H, device=device), sh.dtype),
    }
    if E:
        wts["w_gate_up"] = _normal(gen, (E, 2 * I, H), 0.02, sh.dtype, device)
        wts["w_down"] = _normal(gen, (E, H, I), 0.02, sh.dtype, device)
        wts["w_router"] = _normal(gen, (E, H), H ** -0.5, "f32", device)
    else:
        wts["w_gate_up"] = _normal(gen, (2 * I, H), 0.02, sh.dtype, device)
        wts["w_down"] = _normal(gen, (H, I), 0.02, sh.dtype, device)
    return wts


def generate(w: Workload, device="cpu", stacked: bool = False, place=None) -> Dict[str, object]:
    """All tensors of one step: per-layer weights, per-layer caches, x and the metadata.

    With device="cpu" the torch CPU generator is used; a GPU device draws directly in
    device memory (needed only for the 32-layer configuration whose caches exceed host
    memory); the two do not produce the same numbers.  stacked=True returns each cache as
    one [n_layers, ...] tensor filled layer by layer instead of a list of layer tensors.
    place: a callable that gets everything generated before the caches (weights, x, metadata)
    and the two pool shapes and returns two lists of per-layer tensors to fill in place, for a
    caller that decides where each layer's pools go; the values are those of stacked=True."""
    sh = w.shape
    gen = torch.Generator(device=device)
    gen.manual_seed(w.seed)
    md = metadata(w)
    out: Dict[str, object] = dict(md)
    out["weights"] = [layer_weights(sh, gen, device) for _ in range(sh.n_layers)]
    out["x"] = _normal(gen, (w.n_tokens, sh.hidden), 1.0, sh.dtype, device)
    k_shape = (md["n_pages"], sh.n_kv, sh.page_size, sh.head_dim)
    v_shape = (md["n_pages"], sh.n_kv, sh.head_dim, sh.page_size)
    if stacked or place is not None:
        if place is not None:
            kc, vc = place(out, k_shape, v_shape)
        else:
            kc = torch.empty((sh.n_layers,) + k_shape, dtype=sh.torch_dtype, device=device)
            vc = torch.empty((sh.n_layers,) + v_shape, dtype=sh.torch_dtype, device=device)
        chunk = max(1, md["n_pages"] // 8)          # keeps the fp32 staging buffers small
        for l in range(sh.n_layers):
            for p0 in range(0, md["n_pages"], chunk):
                p1 = min(md["n_pages"], p0 + chunk)
                kc[l][p0:p1] = _normal(gen, (p1 - p0,) + k_shape[1:], 1.0, sh.dtype, device)
                vc[l][p0:p1] = _normal(gen, (p1 - p0,) + v_shape[1:], 1.0, sh.dtype, device)
    else:
        kc, vc = [], []
        for _ in range(sh.n_layers):
            kc.append(_normal(gen, k_shape, 1.0, sh.dtype, device))
            vc.append(_normal(gen, v_shape, 1.0, sh.dtype, device))
    out["k_cache"], out["v_cache"] = kc, vc
    return out


def extract_sequences(w: Workload, data: Dict[str, object], seq_ids: List[int]) -> Tuple[Workload, Dict[str, object]]:
    """Host copy of the same step restricted to some sequences, with their cache pages
    gathered into small per-layer caches and the block table renumbered.  For workloads
    generated in device memory whose caches do not fit on the host."""
    ps = w.shape.page_size
    w2 = dataclasses.replace(w, name=w.name + "_sub", seqs=tuple(w.seqs[s] for s in seq_ids), nano_rows=())
    md = metadata(w2)
    q_start = data["q_start"]
    rows = np.concatenate([np.arange(q_start[s], q_start[s + 1]) for s in seq_ids])
    pages, bt = [], np.zeros((len(seq_ids), md["max_pages_per_seq"]), dtype=np.int32)
    for i, s in enumerate(seq_ids):
        n = (w.seqs[s][1] + ps - 1) // ps
        bt[i, :n] = np.arange(len(pages), len(pages) + n)
        pages.extend(int(p) for p in data["block_table"][s, :n])
    idx = torch.as_tensor(pages, dtype=torch.long, device=data["x"].device)
    d2: Dict[str, object] = dict(md)
    d2["block_table"] = bt
    d2["n_pages"] = len(pages)
    d2["rows"] = rows
    d2["x"] = data["x"][torch.as_tensor(rows, dtype=torch.long, device=data["x"].device)].cpu().contiguous()
    d2["weights"] = [{k: v.cpu() for k, v in lw.items()} for lw in data["weights"]]
    d2["k_cache"] = [data["k_cache"][l][idx].cpu().contiguous() for l in range(w.shape.n_layers)]
    d2["v_cache"] = [data["v_cache"][l][idx].cpu().contiguous() for l in range(w.shape.n_layers)]
    return w2, d2


def sub_batch(w: Workload, data: Dict[str, object], seq_ids: List[int]) -> Tuple[Workload, Dict[str, object]]:
    """The same step restricted to some sequences (rows are independent per sequence).
    The caches and block-table rows are shared with the full batch, x rows are gathered."""
    q_start = data["q_start"]
    rows = np.concatenate([np.arange(q_start[s], q_start[s + 1]) for s in seq_ids])
    w2 = dataclasses.replace(w, name=w.name + "_sub", seqs=tuple(w.seqs[s] for s in seq_ids), nano_rows=())
    md = metadata(w2)
    d2 = dict(data)
    for k in ("seq_of_token", "pos_of_token", "q_start", "ctx_len"):
        d2[k] = md[k]
    d2["block_table"] = np.ascontiguousarray(data["block_table"][seq_ids])
    d2["x"] = data["x"][torch.as_tensor(rows, dtype=torch.long)].contiguous()
    d2["rows"] = rows
    return w2, d2
