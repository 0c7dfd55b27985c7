"""ctypes front end of the CPU oracle (oracle/dyn_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg; never by the product package.  Argument marshalling only - all
arithmetic is in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, List, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dyn_oracle.c")
_LIB = os.path.join(_HERE, "libdynoracle.so")

F32, BF16 = 0, 1


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


class Config(C.Structure):
    _fields_ = [("dtype", C.c_int), ("hidden", C.c_int), ("n_q", C.c_int), ("n_kv", C.c_int),
                ("head_dim", C.c_int), ("inter", C.c_int), ("n_experts", C.c_int), ("top_k", C.c_int),
                ("eps", C.c_double), ("rope_base", C.c_double), ("page_size", C.c_int)]


class Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("w_qkv", "w_o", "w_gate_up", "w_down", "g_norm1", "g_norm2", "w_router")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_layer_forward.restype = C.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def dtype_code(name: str) -> int:
    return BF16 if name == "bf16" else F32


def to_storage(t) -> np.ndarray:
    """torch CPU tensor (fp32 or bf16) -> contiguous numpy array of its storage words."""
    import torch
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def widen(a: np.ndarray, dtype: int) -> np.ndarray:
    out = np.empty(a.shape, dtype=np.float64)
    lib().orc_widen(_p(a), C.c_int(dtype), C.c_size_t(a.size), _p(out))
    return out


def make_config(sh) -> Config:
    return Config(dtype_code(sh.dtype), sh.hidden, sh.n_q, sh.n_kv, sh.head_dim, sh.inter,
                  sh.n_experts, sh.top_k, sh.eps, sh.rope_base, sh.page_size)


def rmsnorm(x: np.ndarray, g: np.ndarray, dtype: int, eps: float) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty_like(x)
    lib().orc_rmsnorm(_p(x), _p(g), C.c_int(dtype), C.c_int(x.shape[0]), C.c_int(x.shape[1]), C.c_double(eps), _p(out))
    return out


def linear(x: np.ndarray, W: np.ndarray, dtype: int) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    N, K = W.shape
    assert x.shape[1] == K
    out = np.empty((x.shape[0], N), dtype=np.float64)
    lib().orc_linear(_p(x), _p(W), C.c_int(dtype), C.c_int(x.shape[0]), C.c_int(K), C.c_int(N), _p(out))
    return out


def rope(z: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """z [T, n_heads, d] fp64 -> rotated copy."""
    z = np.array(z, dtype=np.float64, order="C")
    T, nh, d = z.shape
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    lib().orc_rope(_p(z), C.c_size_t(nh * d), _p(pos), C.c_int(T), C.c_int(nh), C.c_int(d), C.c_double(base))
    return z


def silu_mul(gu: np.ndarray) -> np.ndarray:
    gu = np.ascontiguousarray(gu, dtype=np.float64)
    T, I2 = gu.shape
    out = np.empty((T, I2 // 2), dtype=np.float64)
    lib().orc_silu_mul(_p(gu), C.c_int(T), C.c_int(I2 // 2), _p(out))
    return out


def cache_append(cfg: Config, k: np.ndarray, v: np.ndarray, seq_of_token, pos_of_token, block_table,
                 k_cache: np.ndarray, v_cache: np.ndarray) -> None:
    """k, v [T, n_kv, d] fp64; caches are modified in place."""
    k = np.ascontiguousarray(k, dtype=np.float64)
    v = np.ascontiguousarray(v, dtype=np.float64)
    T = k.shape[0]
    lib().orc_cache_append(C.byref(cfg), _p(k), _p(v), C.c_size_t(cfg.n_kv * cfg.head_dim), C.c_int(T),
                           _p(seq_of_token), _p(pos_of_token), _p(block_table), C.c_int(block_table.shape[1]),
                           _p(k_cache), _p(v_cache))


def attention(cfg: Config, q: np.ndarray, seq_of_token, pos_of_token, block_table,
              k_cache: np.ndarray, v_cache: np.ndarray, want_probs: int = 0):
    """q [T, n_q, d] fp64 -> out [T, n_q*d] (and probs [T, n_q, want_probs] if asked)."""
    q = np.ascontiguousarray(q, dtype=np.float64)
    T = q.shape[0]
    out = np.empty((T, cfg.n_q * cfg.head_dim), dtype=np.float64)
    probs = np.zeros((T, cfg.n_q, want_probs), dtype=np.float64) if want_probs else None
    lib().orc_attention(C.byref(cfg), _p(q), C.c_size_t(cfg.n_q * cfg.head_dim), C.c_int(T),
                        _p(seq_of_token), _p(pos_of_token), _p(block_table), C.c_int(block_table.shape[1]),
                        _p(k_cache), _p(v_cache), _p(out), _p(probs), C.c_int(want_probs))
    return (out, probs) if want_probs else out


def route(h: np.ndarray, w_router: np.ndarray, top_k: int, forced_sel: Optional[np.ndarray] = None):
    h = np.ascontiguousarray(h, dtype=np.float64)
    T, H = h.shape
    E = w_router.shape[0]
    sel = np.empty((T, top_k), dtype=np.int32)
    wgt = np.empty((T, top_k), dtype=np.float64)
    logits = np.empty((T, E), dtype=np.float64)
    lib().orc_route(_p(h), _p(w_router), C.c_int(T), C.c_int(H), C.c_int(E), C.c_int(top_k),
                    _p(forced_sel), _p(sel), _p(wgt), _p(logits))
    return sel, wgt, logits


def layer_forward(sh, wts: Dict[str, np.ndarray], x: np.ndarray, seq_of_token, pos_of_token, block_table,
                  k_cache: np.ndarray, v_cache: np.ndarray, forced_sel: Optional[np.ndarray] = None,
                  routing_out: Optional[dict] = None) -> np.ndarray:
    """One layer.  wts / caches are storage-word arrays (see to_storage); x is fp64 [T, hidden].
    The caches are updated in place.  Returns y fp64."""
    cfg = make_config(sh)
    w = Weights(*[_p(wts.get(n)) for n in ("w_qkv", "w_o", "w_gate_up", "w_down", "g_norm1", "g_norm2", "w_router")])
    x = np.ascontiguousarray(x, dtype=np.float64)
    T = x.shape[0]
    y = np.empty_like(x)
    sel = wgt = logits = None
    if sh.n_experts:
        sel = np.empty((T, sh.top_k), dtype=np.int32)
        wgt = np.empty((T, sh.top_k), dtype=np.float64)
        logits = np.empty((T, sh.n_experts), dtype=np.float64)
        if forced_sel is not None:
            forced_sel = np.ascontiguousarray(forced_sel, dtype=np.int32)
    seq_of_token = np.ascontiguousarray(seq_of_token, dtype=np.int32)
    pos_of_token = np.ascontiguousarray(pos_of_token, dtype=np.int32)
    block_table = np.ascontiguousarray(block_table, dtype=np.int32)
    rc = lib().orc_layer_forward(C.byref(cfg), C.byref(w), C.c_int(T), _p(x), _p(seq_of_token), _p(pos_of_token),
                                 _p(block_table), C.c_int(block_table.shape[1]), _p(k_cache), _p(v_cache),
                                 _p(y), _p(forced_sel), _p(sel), _p(wgt), _p(logits))
    if rc != 0:
        raise ValueError("oracle rejected the configuration")
    if routing_out is not None and sh.n_experts:
        routing_out.update(sel=sel, wgt=wgt, logits=logits)
    return y


def forward(w, data: dict, forced_sel: Optional[List[np.ndarray]] = None, routing_out: Optional[list] = None):
    """All layers of a generated workload (workloads.gen.generate output).
    Returns (y fp64, k_caches, v_caches) where the caches are updated copies (storage words)."""
    sh = w.shape
    dt = dtype_code(sh.dtype)
    x = widen(to_storage(data["x"]), dt)
    kcs, vcs = [], []
    for l in range(sh.n_layers):
        wts = {k: to_storage(v) for k, v in data["weights"][l].items()}
        kc = to_storage(data["k_cache"][l]).copy()
        vc = to_storage(data["v_cache"][l]).copy()
        ro = {} if routing_out is not None else None
        x = layer_forward(sh, wts, x, data["seq_of_token"], data["pos_of_token"], data["block_table"], kc, vc,
                          None if forced_sel is None else forced_sel[l], ro)
        if routing_out is not None:
            routing_out.append(ro)
        kcs.append(kc)
        vcs.append(vc)
    return x, kcs, vcs
