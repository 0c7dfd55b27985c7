"""Measured placement of the K and V cache pools in HBM.  Caller-side helper: it decides where
caller-owned buffers go and computes nothing of the layer.

The attention launch of a layer streams that layer's K pool and V pool together, page by page,
and on MI355X its rate depends on which regions of HBM the two pools lie in: for one
Llama-3-8B-shaped layer at batch 256 (2.3 GiB per pool) the same launch takes 827-849, 857-885 or
940-957 us depending on the pair of regions, in blocks of 32 or 64 GiB that follow the physical
backing of the allocation (a bare reader sees only a third of that contrast, so the launch itself
is the probe).  Two pools allocated one after the other early in a process land in the slowest
class.  So: take one large arena, time the real attention launch with the pools at pairs of arena
chunks, and give every layer the fastest pair that still has room.  The library takes the result
through k_cache_layers / v_cache_layers of the batch."""
from typing import Dict, List, Sequence, Tuple

import torch

from . import binding as B

GiB = 1 << 30


class Arena:
    """One allocation cut into chunks of chunk_bytes; a chunk holds whole pools ("slots")."""

    def __init__(self, n_chunks: int, chunk_bytes: int, device="cuda:0"):
        self.n_chunks, self.chunk_bytes = n_chunks, chunk_bytes
        self.reserved_tail = 0              # bytes at the end of every chunk kept free of pools (a workspace may go there)
        self.buf = torch.empty(n_chunks * chunk_bytes, dtype=torch.uint8, device=device)

    def fill_random(self, seed: int = 1) -> None:
        """N(0, 1) bf16 values everywhere (one 512 MiB block repeated): the probe reads pools at
        places that hold no cache yet, and what it reads should cost what real values cost."""
        g = torch.Generator(device=self.buf.device)
        g.manual_seed(seed)
        blk = torch.empty(256 << 20, dtype=torch.float32, device=self.buf.device).normal_(generator=g).to(torch.bfloat16).view(torch.uint8)
        for o in range(0, self.buf.numel(), blk.numel()):
            n = min(blk.numel(), self.buf.numel() - o)
            self.buf[o:o + n].copy_(blk[:n])

    def view(self, chunk: int, slot: int, slot_bytes: int, shape, dtype) -> torch.Tensor:
        off = chunk * self.chunk_bytes + slot * slot_bytes
        n = 1
        for d in shape:
            n *= d
        e = torch.empty(0, dtype=dtype).element_size()
        assert slot * slot_bytes + n * e <= self.chunk_bytes - self.reserved_tail
        return self.buf[off:off + n * e].view(dtype).view(shape)


def slot_bytes_of(k_shape, dtype) -> int:
    n = 1
    for d in k_shape:
        n *= d
    b = n * torch.empty(0, dtype=dtype).element_size()
    return (b + 255) & ~255


def measure_pairs(layer1: "B.DynLayer", data: dict, arena: Arena, k_shape, v_shape, dtype, stream, reps: int = 2,
                  workspace: "torch.Tensor" = None) -> Dict[Tuple[int, int], float]:
    """Attention launch time (us, by the library's own per-dispatch events) of the one-layer model
    `layer1` on the step in `data`, with the K pool at the start of chunk i and the V pool at the
    start of chunk j (i < j), or right behind the K pool in the same chunk (i == j).
    workspace: the buffer the timed step will use.  The attention kernel writes its split-KV
    partials there, a third stream next to the two pools, and which region that buffer lies in
    moves the launch by 4-5 % (one Llama-3-8B layer at batch 128, chunks of 256 positions: 215-219
    us with pools and workspace in three different regions' classes, 227-230 us when the workspace
    shares a class with a pool): measure with the buffer that will be used."""
    sb = slot_bytes_of(k_shape, dtype)
    k0 = arena.view(0, 0, sb, k_shape, dtype)
    v0 = arena.view(0, 1, sb, v_shape, dtype)
    step = B.DeviceStep(layer1, dict(data, k_cache=[k0], v_cache=[v0]), placed=True, workspace=workspace)
    base = arena.buf.data_ptr()
    sched = B.sequential()
    layer1.set_profiling(True)
    times = {}
    try:
        for i in range(arena.n_chunks):
            for j in range(i, arena.n_chunks):
                step._k_ptrs[0] = base + i * arena.chunk_bytes
                step._v_ptrs[0] = base + j * arena.chunk_bytes + (sb if i == j else 0)
                ts = []
                with torch.cuda.stream(stream):
                    for r in range(reps + 1):
                        layer1.forward(step.batch, sched, stream)
                        stream.synchronize()
                        if r == 0:
                            continue
                        for rec in layer1.slot_times():
                            if rec["op"] == B.DYN_OP_ATTN:
                                ts.append(rec["main_stop_ms"] - rec["main_start_ms"])
                times[(i, j)] = 1e3 * sum(ts) / len(ts)
    finally:
        layer1.set_profiling(False)
    return times


def measure_workspace(layer1: "B.DynLayer", data: dict, arena: Arena, k_shape, v_shape, dtype, ws_bytes: int, stream,
                      reps: int = 3) -> Dict[int, float]:
    """Time (us) of everything but attention in the one-layer step - the projections write their
    split-K planes to the workspace while they stream their weights - with the workspace in the
    last ws_bytes of each arena chunk (pools at the first and the last chunk).  Weights in the
    workspace's region cost the projections 2-3 %, an expert-grouped down projection 10 %."""
    sb = slot_bytes_of(k_shape, dtype)
    k0 = arena.view(0, 0, sb, k_shape, dtype)
    v0 = arena.view(arena.n_chunks - 1, 0, sb, v_shape, dtype)
    sched = B.sequential()
    out = {}
    for c in range(arena.n_chunks):
        ws = workspace_view(arena, c, ws_bytes)
        step = B.DeviceStep(layer1, dict(data, k_cache=[k0], v_cache=[v0]), placed=True, workspace=ws)
        layer1.set_profiling(True)
        ts = []
        try:
            with torch.cuda.stream(stream):
                for r in range(reps + 1):
                    layer1.forward(step.batch, sched, stream)
                    stream.synchronize()
                    if r == 0:
                        continue
                    ts.append(sum(rec["stop_ms"] - rec["start_ms"] for rec in layer1.slot_times() if rec["op"] != B.DYN_OP_ATTN))
        finally:
            layer1.set_profiling(False)
        out[c] = 1e3 * sum(ts) / len(ts)
    return out


def workspace_view(arena: Arena, chunk: int, ws_bytes: int) -> torch.Tensor:
    """The last ws_bytes (rounded up to 4 KiB) of a chunk."""
    n = (ws_bytes + 4095) & ~4095
    end = (chunk + 1) * arena.chunk_bytes
    return arena.buf[end - n:end]


def assign(times: Dict[Tuple[int, int], float], n_layers: int, slots_per_chunk: int, n_chunks: int) -> List[Tuple[int, int, int, int, float]]:
    """Every layer gets a K slot and a V slot.  Fastest pairs first, as many layers per pair as both
    chunks still have slots for; then pairs of layers trade partners while that lowers the sum
    (two layers on (i, j) and (k, l) become (i, k), (j, l) or (i, l), (j, k): every chunk keeps its
    number of used slots) - without it the greedy pass can spend the slots of good partners on each
    other and leave the last layers a pair of the slowest class.
    Returns per layer (K chunk, K slot, V chunk, V slot, probed us)."""
    def cost(i, j):
        return times[(i, j) if i <= j else (j, i)]

    free = [slots_per_chunk] * n_chunks
    pairs = []
    for (i, j), _ in sorted(times.items(), key=lambda kv: kv[1]):
        while len(pairs) < n_layers and (free[i] >= 2 if i == j else free[i] >= 1 and free[j] >= 1):
            free[i] -= 1
            free[j] -= 1
            pairs.append((i, j))
        if len(pairs) == n_layers:
            break
    if len(pairs) < n_layers:
        raise RuntimeError("the arena has room for %d of %d layers" % (len(pairs), n_layers))
    improved = True
    while improved:
        improved = False
        # a layer moves to a pair with free slots
        for a in range(len(pairs)):
            i, j = pairs[a]
            free[i] += 1
            free[j] += 1
            best, best_c = (i, j), cost(i, j)
            for (k, l), t in times.items():
                if t < best_c - 1e-9 and (free[k] >= 2 if k == l else free[k] >= 1 and free[l] >= 1):
                    best, best_c = (k, l), t
            if best != (i, j):
                improved = True
            pairs[a] = best
            free[best[0]] -= 1
            free[best[1]] -= 1
        # two layers trade partners
        for a in range(len(pairs)):
            for b in range(a + 1, len(pairs)):
                (i, j), (k, l) = pairs[a], pairs[b]
                now = cost(i, j) + cost(k, l)
                for (p, q), (r, u) in (((i, k), (j, l)), ((i, l), (j, k))):
                    if (min(p, q), max(p, q)) in times and (min(r, u), max(r, u)) in times and cost(p, q) + cost(r, u) < now - 1e-9:
                        pairs[a], pairs[b] = (p, q), (r, u)
                        now = cost(p, q) + cost(r, u)
                        (i, j), (k, l) = pairs[a], pairs[b]
                        improved = True
    used = [0] * n_chunks
    out = []
    for i, j in sorted(pairs, key=lambda pq: cost(*pq)):
        ks = used[i]
        used[i] += 1
        vs = used[j]
        used[j] += 1
        out.append((i, ks, j, vs, cost(i, j)))
    return out


def rule_chunk(ctx_len: Sequence[int], q_len: Sequence[int], n_kv: int, n_waves: int = 2048) -> int:
    """kv_chunk_positions by rule: 1024 positions when the decode sequences of the batch make at
    least eight work items per persistent wave at 256 (so that a quarter as many still keep every
    wave supplied), else the library's 256.  Measured (MI355X, pools placed): batch 256 at contexts
    1024..8192 (18 items per wave at 256): attention dispatch 884-887 us at 256, 868-873 at 1024,
    871 at 2048; batch 128 at 512..4096 (4.8 per wave): 246-250, 252-255, 261-267 us."""
    items = sum((c + 255) // 256 for c, q in zip(ctx_len, q_len) if q == 1) * n_kv
    return 1024 if items >= 8 * n_waves else 256


def choose_chunk(make_layer1, data: dict, k0: torch.Tensor, v0: torch.Tensor, candidates: Sequence[int], stream, reps: int = 4,
                 workspace: "torch.Tensor" = None) -> Tuple[int, Dict[int, float]]:
    """Split-KV chunk size of decode attention (kv_chunk_positions of the configuration) by
    measurement: the whole attention dispatch (work lists, attention kernels, merge) of a one-layer
    handle per candidate, on the step in `data` with its layer-0 pools k0 / v0 where they will be.
    make_layer1(chunk) returns the handle.  Returns the fastest candidate and every candidate's us."""
    out = {}
    for chunk in candidates:
        layer1 = make_layer1(chunk)
        step = B.DeviceStep(layer1, dict(data, k_cache=[k0], v_cache=[v0]), placed=True, workspace=workspace)
        sched = B.sequential()
        layer1.set_profiling(True)
        ts = []
        try:
            with torch.cuda.stream(stream):
                for r in range(reps + 1):
                    layer1.forward(step.batch, sched, stream)
                    stream.synchronize()
                    if r == 0:
                        continue
                    for rec in layer1.slot_times():
                        if rec["op"] == B.DYN_OP_ATTN:
                            ts.append(rec["stop_ms"] - rec["start_ms"])
        finally:
            layer1.set_profiling(False)
        out[chunk] = 1e3 * sum(ts) / len(ts)
        layer1.close()
    best = min(out, key=lambda c: out[c])
    return best, out


def place_layers(arena: Arena, plan: Sequence[Tuple[int, int, int, int, float]], k_shape, v_shape, dtype):
    sb = slot_bytes_of(k_shape, dtype)
    ks = [arena.view(kc, ksl, sb, k_shape, dtype) for kc, ksl, _, _, _ in plan]
    vs = [arena.view(vc, vsl, sb, v_shape, dtype) for _, _, vc, vsl, _ in plan]
    return ks, vs


def summary(times: Dict[Tuple[int, int], float], plan) -> dict:
    all_t = sorted(times.values())
    chosen = [p[4] for p in plan]
    return {"pairs_probed": len(all_t), "probe_us_fastest": all_t[0], "probe_us_median": all_t[len(all_t) // 2],
            "probe_us_slowest": all_t[-1], "chosen_us_mean": sum(chosen) / len(chosen), "chosen_us_worst": max(chosen),
            "pairs": [[p[0], p[2]] for p in plan]}
