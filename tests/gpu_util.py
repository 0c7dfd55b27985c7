"""Helpers shared by the GPU tests: run a generated step through the C-ABI library and
compare with the oracle."""
import sys

import numpy as np
import torch

from oracle import oracle as orc
from paper_2605_21603_amd import binding as B
from workloads import gen

TOL = {"f32": 1e-4, "bf16": 2e-2}


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def row_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max over rows of max_i |got - ref| / max_i |ref| (element-wise relative error is
    meaningless next to zeros)."""
    num = np.abs(got - ref).max(axis=1)
    den = np.abs(ref).max(axis=1)
    return float((num / den).max())


def to_device_weights(data, device="cuda:0"):
    return [{k: v.to(device) for k, v in lw.items()} for lw in data["weights"]]


class GpuRun:
    def __init__(self, w, data, device="cuda:0", kv_chunk_positions=0):
        self.w, self.data = w, data
        self.weights = to_device_weights(data, device)
        self.layer = B.DynLayer(B.make_config(w.shape, kv_chunk_positions), self.weights)
        self.device = device

    def run(self, sched, stream=None, repeat=1):
        """Fresh copies of x and the caches, one forward (or `repeat` forwards on the same
        buffers, for graph replays).  Returns y, k_cache, v_cache as CPU tensors."""
        step = B.DeviceStep(self.layer, self.data, self.device)
        st = stream or torch.cuda.Stream()
        with torch.cuda.stream(st):
            for _ in range(repeat):
                self.layer.forward(step.batch, sched, st)
        st.synchronize()
        torch.cuda.synchronize()
        return step.y.cpu(), step.k_cache.cpu(), step.v_cache.cpu()


def as_f64(t: torch.Tensor) -> np.ndarray:
    return t.double().numpy()


def check_against_oracle(w, data, y, kc, vc, rows=None):
    """y / caches from the GPU against the oracle on the same inputs.  Returns the error."""
    routing = [] if w.shape.n_experts else None
    y_ref, kcs, vcs = orc.forward(w, data, routing_out=routing)
    dt = orc.dtype_code(w.shape.dtype)
    y_got = as_f64(y)
    if routing and w.shape.n_layers == 1:
        # Two routings are both correct where the router's k-th and (k+1)-th logits nearly tie.
        # Rows that miss the tolerance with such a tie are re-checked against the other selection.
        bad = np.abs(y_got - y_ref).max(axis=1) / np.abs(y_ref).max(axis=1) > TOL[w.shape.dtype]
        logits, sel = routing[0]["logits"], routing[0]["sel"]
        srt = np.sort(logits, axis=1)[:, ::-1]
        margin = srt[:, w.shape.top_k - 1] - srt[:, w.shape.top_k]
        for t in np.nonzero(bad)[0]:
            assert margin[t] < 1e-3, "row %d misses tolerance without a near tie (margin %.3e)" % (t, margin[t])
            forced = sel.copy()
            forced[t, -1] = np.argsort(-logits[t])[w.shape.top_k]
            y_alt, _, _ = orc.forward(w, data, forced_sel=[forced])
            y_ref[t] = y_alt[t]
    err = row_rel_err(y_got, y_ref)
    assert err <= TOL[w.shape.dtype], "max rel err %.3e" % err
    ps = w.shape.page_size
    for l in range(w.shape.n_layers):
        k_ref, v_ref = orc.widen(kcs[l], dt), orc.widen(vcs[l], dt)
        k_got, v_got = as_f64(kc[l]), as_f64(vc[l])
        k_old, v_old = as_f64(data["k_cache"][l]), as_f64(data["v_cache"][l])
        touched_k = np.zeros(k_got.shape, bool)
        touched_v = np.zeros(v_got.shape, bool)
        for s, (q, c) in enumerate(w.seqs):
            for p in range(c - q, c):
                page, slot = data["block_table"][s, p // ps], p % ps
                touched_k[page, :, slot, :] = True
                touched_v[page, :, :, slot] = True
        # untouched entries keep their bits, appended ones agree to the storage rounding
        assert np.array_equal(k_got[~touched_k], k_old[~touched_k])
        assert np.array_equal(v_got[~touched_v], v_old[~touched_v])
        tol = TOL[w.shape.dtype]
        for got, ref, m in ((k_got, k_ref, touched_k), (v_got, v_ref, touched_v)):
            scale = np.abs(ref[m]).max()
            assert np.abs(got[m] - ref[m]).max() <= tol * scale
    return err
