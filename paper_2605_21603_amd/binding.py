"""ctypes binding of libdynlayer.so.  Argument marshalling only: every step of the layer
runs in the library's HIP kernels.  PyTorch supplies device memory and streams."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch  # must be imported before the library so both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("DYNLAYER_LIB") or os.path.join(_HERE, "libdynlayer.so")   # the in-tree build unless another build is named

DYN_OK, DYN_ERR_INVALID_ARG, DYN_ERR_UNSUPPORTED, DYN_ERR_SCHEDULE, DYN_ERR_WORKSPACE, DYN_ERR_HIP = range(6)
DYN_F32, DYN_BF16 = 0, 1
(DYN_OP_NORM1, DYN_OP_QKV, DYN_OP_ROPE_KV, DYN_OP_ATTN, DYN_OP_OPROJ, DYN_OP_NORM2, DYN_OP_ROUTE, DYN_OP_GATE_UP,
 DYN_OP_SILU, DYN_OP_DOWN) = range(10)
DYN_N_OPS = 10
DYN_SCHED_SEQUENTIAL, DYN_SCHED_EXPLICIT = 0, 1
DYN_MAX_NANO, DYN_MAX_STREAMS, DYN_MAX_PARTITIONS = 8, 8, 4
DYN_NOALLOC_MAX_WORKSPACE = 96 << 20
DYN_FORM_SEQUENTIAL, DYN_FORM_SPLIT, DYN_FORM_MLP_MERGED, DYN_FORM_ATTN_SPLIT, DYN_FORM_MLP_SPLIT = 0, 1, 2, 3, 4
FORM_NAMES = ["sequential", "split", "mlp_merged", "attn_split", "mlp_split"]
OP_NAMES = ["norm1", "qkv", "rope_kv", "attn", "oproj", "norm2", "route", "gate_up", "silu", "down"]
DENSE_CHAIN = [DYN_OP_NORM1, DYN_OP_QKV, DYN_OP_ROPE_KV, DYN_OP_ATTN, DYN_OP_OPROJ, DYN_OP_NORM2, DYN_OP_GATE_UP,
               DYN_OP_SILU, DYN_OP_DOWN]
MOE_CHAIN = DENSE_CHAIN[:6] + [DYN_OP_ROUTE] + DENSE_CHAIN[6:]


class dyn_layer_config(C.Structure):
    _fields_ = [("dtype", C.c_int), ("n_layers", C.c_int), ("hidden", C.c_int), ("n_q_heads", C.c_int),
                ("n_kv_heads", C.c_int), ("head_dim", C.c_int), ("mlp_inter", C.c_int), ("n_experts", C.c_int),
                ("top_k", C.c_int), ("rms_eps", C.c_float), ("rope_base", C.c_float), ("page_size", C.c_int),
                ("kv_chunk_positions", C.c_int)]


class dyn_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("w_qkv", "w_o", "w_gate_up", "w_down", "g_norm1", "g_norm2", "w_router")]


class dyn_batch(C.Structure):
    _fields_ = [("n_tokens", C.c_int), ("n_seqs", C.c_int), ("x", C.c_void_p), ("y", C.c_void_p),
                ("seq_of_token", C.c_void_p), ("pos_of_token", C.c_void_p), ("block_table", C.c_void_p),
                ("max_pages_per_seq", C.c_int), ("q_start_host", C.c_void_p), ("k_cache", C.c_void_p),
                ("v_cache", C.c_void_p), ("kv_layer_stride", C.c_size_t), ("workspace", C.c_void_p),
                ("workspace_bytes", C.c_size_t), ("k_cache_layers", C.c_void_p), ("v_cache_layers", C.c_void_p)]


class dyn_slot(C.Structure):
    _fields_ = [("op", C.c_uint8), ("nano", C.c_uint8), ("n_nano", C.c_uint8), ("stream", C.c_uint8),
                ("partition", C.c_uint8)]


class dyn_schedule(C.Structure):
    _fields_ = [("mode", C.c_int), ("k", C.c_int), ("nano_rows", C.c_void_p), ("n_streams", C.c_int),
                ("n_partitions", C.c_int), ("cu_masks", C.c_void_p), ("cu_mask_words", C.c_int), ("n_slots", C.c_int),
                ("slots", C.c_void_p), ("use_graph", C.c_int)]


class dyn_policy_choice(C.Structure):
    _fields_ = [("split", C.c_int), ("cut_row", C.c_int), ("est_sequential_us", C.c_float), ("est_split_us", C.c_float)]


class dyn_memory_report(C.Structure):
    _fields_ = [("workspace_bytes", C.c_size_t), ("peak_live_bytes", C.c_size_t), ("peak_live_bytes_sequential", C.c_size_t),
                ("peak_at_dispatch", C.c_int), ("n_regions", C.c_int), ("max_ref_count", C.c_int), ("n_resharded", C.c_int),
                ("workspace_bytes_schedule", C.c_size_t)]

    def as_dict(self) -> dict:
        return {n: getattr(self, n) for n, _ in self._fields_}


class dyn_region(C.Structure):
    _fields_ = [("kind", C.c_int), ("slot", C.c_int), ("stream", C.c_int), ("offset", C.c_size_t), ("bytes", C.c_size_t),
                ("live_slots", C.c_uint64 * 2)]


REGION_NAMES = ["h", "qkv", "attn", "x2", "gu", "act", "routing", "xa", "xb", "plan", "planes", "part_o", "part_ml", "lists",
                "moe_planes"]


class dyn_tune_candidate(C.Structure):
    _fields_ = [("k", C.c_int), ("rows", C.c_int32 * (DYN_MAX_NANO + 1)), ("form", C.c_int), ("stagger", C.c_int),
                ("cus_first", C.c_int), ("us", C.c_float)]

    def as_dict(self) -> dict:
        return {"k": self.k, "rows": [self.rows[i] for i in range(self.k + 1)], "form": FORM_NAMES[self.form],
                "stagger": self.stagger, "cus_first": self.cus_first, "us": self.us}


class dyn_tune_options(C.Structure):
    _fields_ = [("max_k", C.c_int), ("partitions", C.c_int), ("n_cus", C.c_int), ("warmup", C.c_int), ("iters", C.c_int),
                ("use_graph", C.c_int), ("min_gain", C.c_float)]


class dyn_tune_result(C.Structure):
    _fields_ = [("best", dyn_tune_candidate), ("us_sequential", C.c_float), ("n_tried", C.c_int), ("n_skipped", C.c_int)]


class dyn_slot_time(C.Structure):
    _fields_ = [("layer", C.c_int), ("op", C.c_int), ("nano", C.c_int), ("n_nano", C.c_int), ("stream", C.c_int),
                ("partition", C.c_int), ("start_ms", C.c_float), ("main_start_ms", C.c_float), ("main_stop_ms", C.c_float),
                ("stop_ms", C.c_float)]


EXPORTS = ["dyn_layer_create", "dyn_layer_destroy", "dyn_layer_workspace_bytes", "dyn_schedule_validate",
           "dyn_layer_prepare", "dyn_layer_release_graphs", "dyn_layer_forward", "dyn_layer_forward_noalloc", "dyn_layer_set_profiling", "dyn_layer_get_slot_times", "dyn_last_error",
           "dyn_scheduler_create", "dyn_scheduler_destroy", "dyn_scheduler_split", "dyn_scheduler_set_partitions",
           "dyn_scheduler_get_ready_ops", "dyn_scheduler_execute", "dyn_scheduler_finish", "dyn_policy_auto",
           "dyn_tune_candidates", "dyn_tune_record", "dyn_tune", "dyn_schedule_memory", "dyn_schedule_workspace_bytes",
           "dyn_schedule_regions", "dyn_probe_hbm_read", "dyn_probe_mfma_loop"]

_lib = None


def lib() -> C.CDLL:
    """The loaded library.  There is no fallback: a missing build is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libdynlayer.so is not built: run `python -m paper_2605_21603_amd.build`")
        l = C.CDLL(LIB_PATH)
        l.dyn_last_error.restype = C.c_char_p
        l.dyn_layer_workspace_bytes.restype = C.c_size_t
        l.dyn_layer_workspace_bytes.argtypes = [C.c_void_p, C.c_int, C.c_int]
        l.dyn_layer_create.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        l.dyn_layer_destroy.argtypes = [C.c_void_p]
        l.dyn_layer_destroy.restype = None
        l.dyn_schedule_validate.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        l.dyn_layer_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        l.dyn_layer_prepare.argtypes = [C.c_void_p, C.c_void_p]
        l.dyn_layer_release_graphs.argtypes = [C.c_void_p]
        l.dyn_layer_forward_noalloc.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        l.dyn_probe_hbm_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        l.dyn_probe_mfma_loop.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        l.dyn_layer_set_profiling.argtypes = [C.c_void_p, C.c_int]
        l.dyn_layer_get_slot_times.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
        l.dyn_scheduler_create.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        l.dyn_scheduler_destroy.argtypes = [C.c_void_p]
        l.dyn_scheduler_destroy.restype = None
        l.dyn_scheduler_split.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
        l.dyn_scheduler_set_partitions.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int]
        l.dyn_scheduler_get_ready_ops.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int]
        l.dyn_scheduler_execute.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int]
        l.dyn_scheduler_finish.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
        l.dyn_policy_auto.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        l.dyn_schedule_memory.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        l.dyn_schedule_workspace_bytes.restype = C.c_size_t
        l.dyn_schedule_workspace_bytes.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        l.dyn_schedule_regions.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
        l.dyn_tune_candidates.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int]
        l.dyn_tune_record.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        l.dyn_tune.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                               C.c_void_p, C.c_void_p, C.c_int]
        _lib = l
    return _lib


class DynError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__("dynlayer status %d: %s" % (status, msg))
        self.status = status


def _check(status: int) -> None:
    if status != DYN_OK:
        raise DynError(status, lib().dyn_last_error().decode())


def dyn_last_error() -> str:
    return lib().dyn_last_error().decode()


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, torch.Tensor):
        assert t.is_contiguous()
        return t.data_ptr()
    if isinstance(t, np.ndarray):
        assert t.flags["C_CONTIGUOUS"]
        return t.ctypes.data
    return int(t)


@dataclass
class Schedule:
    """Host-side schedule descriptor; slots are (op, nano, n_nano, stream, partition)."""
    mode: int = DYN_SCHED_SEQUENTIAL
    nano_rows: Sequence[int] = ()
    slots: Sequence[Sequence[int]] = ()
    n_streams: int = 1
    cu_masks: Sequence[Sequence[int]] = ()     # one row of uint32 words per masked partition
    use_graph: bool = False
    _keep: list = field(default_factory=list, repr=False)

    def to_c(self) -> dyn_schedule:
        rows = np.ascontiguousarray(self.nano_rows, dtype=np.int32)
        slots = (dyn_slot * max(1, len(self.slots)))(*[dyn_slot(*s) for s in self.slots])
        masks = np.ascontiguousarray(self.cu_masks, dtype=np.uint32).reshape(len(self.cu_masks), -1) \
            if len(self.cu_masks) else np.zeros((0, 0), np.uint32)
        self._keep = [rows, slots, masks]
        return dyn_schedule(self.mode, max(0, len(rows) - 1), _ptr(rows) if len(rows) else None, self.n_streams,
                            len(self.cu_masks), _ptr(masks) if len(self.cu_masks) else None,
                            masks.shape[1] if len(self.cu_masks) else 0, len(self.slots),
                            C.cast(slots, C.c_void_p).value if len(self.slots) else None, int(self.use_graph))


def sequential(use_graph: bool = False) -> Schedule:
    return Schedule(DYN_SCHED_SEQUENTIAL, use_graph=use_graph)


def nano_schedule(nano_rows: Sequence[int], chain: Sequence[int] = DENSE_CHAIN, merged_ops: Sequence[int] = (),
                  streams: Optional[Sequence[int]] = None, partitions: Optional[Sequence[int]] = None,
                  cu_masks: Sequence[Sequence[int]] = (), use_graph: bool = False, stagger: int = 0,
                  op_partitions: Optional[dict] = None) -> Schedule:
    """Split-and-overlap schedule in the style of the paper's batch-splitting strategies:
    micro-batch b runs its operators on stream streams[b]; operators in merged_ops are
    dispatched once for all micro-batches (merge form) on stream 0.  Issue order interleaves
    the micro-batches operator by operator, micro-batch b lagging `stagger` operators behind
    micro-batch b-1, so that a memory-bound operator of one meets a GEMM of the other.
    partitions gives each micro-batch a CU partition; op_partitions ({operator: partition})
    overrides it per operator class, e.g. every micro-batch's attention on one partition and
    the projections on another."""
    k = len(nano_rows) - 1
    streams = list(streams) if streams is not None else list(range(k))
    partitions = list(partitions) if partitions is not None else [0] * k
    slots, pos, n, tick = [], [0] * k, len(chain), 0
    while min(pos) < n:
        for b in range(k):
            if pos[b] >= n or tick < b * stagger:
                continue
            op = chain[pos[b]]
            if op not in merged_ops:
                slots.append((op, b, 1, streams[b], (op_partitions or {}).get(op, partitions[b])))
                pos[b] += 1
            elif all(p == pos[b] for p in pos):      # the last micro-batch has arrived: merge form
                slots.append((op, 0, k, 0, 0))
                pos = [p + 1 for p in pos]
        tick += 1
    return Schedule(DYN_SCHED_EXPLICIT, list(nano_rows), slots, max(streams) + 1, cu_masks, use_graph)


class RecordedSchedule:
    """A dyn_schedule filled in by the library's scheduler; it borrows the scheduler's
    arrays, so it keeps the scheduler alive.  Accepted wherever a Schedule is."""

    def __init__(self, scheduler: "Scheduler", c_sched: dyn_schedule):
        self._scheduler = scheduler
        self._c = c_sched

    def to_c(self) -> dyn_schedule:
        return self._c

    @property
    def slots(self) -> List[tuple]:
        arr = C.cast(self._c.slots, C.POINTER(dyn_slot))
        return [(arr[i].op, arr[i].nano, arr[i].n_nano, arr[i].stream, arr[i].partition) for i in range(self._c.n_slots)]

    @property
    def nano_rows(self) -> List[int]:
        arr = C.cast(self._c.nano_rows, C.POINTER(C.c_int32))
        return [arr[i] for i in range(self._c.k + 1)]


class Scheduler:
    """The library's schedule recorder: split / get_ready_ops / execute / finish.  A
    strategy is a short program over these calls; every call is checked by the library."""

    def __init__(self, cfg: dyn_layer_config, q_start: Sequence[int]):
        self._q = np.ascontiguousarray(q_start, dtype=np.int32)
        self._h = C.c_void_p()
        _check(lib().dyn_scheduler_create(C.byref(cfg), int(self._q[-1]), len(self._q) - 1, _ptr(self._q), C.byref(self._h)))

    def close(self):
        if self._h:
            lib().dyn_scheduler_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def split(self, sizes: Sequence[int]) -> None:
        a = np.ascontiguousarray(sizes, dtype=np.int32)
        _check(lib().dyn_scheduler_split(self._h, len(a), _ptr(a)))

    def set_partitions(self, cu_masks: Sequence[Sequence[int]]) -> None:
        m = np.ascontiguousarray(cu_masks, dtype=np.uint32).reshape(len(cu_masks), -1) if len(cu_masks) else np.zeros((0, 1), np.uint32)
        _check(lib().dyn_scheduler_set_partitions(self._h, m.shape[0], _ptr(m) if m.shape[0] else None, m.shape[1] if m.shape[0] else 0))

    def get_ready_ops(self, nano: int) -> List[int]:
        buf = (C.c_uint8 * DYN_N_OPS)()
        n = lib().dyn_scheduler_get_ready_ops(self._h, nano, buf, DYN_N_OPS)
        if n < 0:
            raise DynError(DYN_ERR_INVALID_ARG, dyn_last_error())
        return [buf[i] for i in range(n)]

    def execute(self, pairs: Sequence[Sequence[int]], stream: int = 0, partition: int = 0) -> None:
        """pairs: (operator, micro-batch) tuples."""
        ops = (C.c_uint8 * max(1, len(pairs)))(*[p[0] for p in pairs])
        nanos = (C.c_uint8 * max(1, len(pairs)))(*[p[1] for p in pairs])
        _check(lib().dyn_scheduler_execute(self._h, len(pairs), ops, nanos, stream, partition))

    def finish(self, use_graph: bool = False) -> RecordedSchedule:
        c = dyn_schedule()
        _check(lib().dyn_scheduler_finish(self._h, int(use_graph), C.byref(c)))
        return RecordedSchedule(self, c)

    def auto(self, ctx_len: Sequence[int], use_graph: bool = False):
        """The built-in policy: returns (schedule, choice dict)."""
        ctx = np.ascontiguousarray(ctx_len, dtype=np.int32)
        c, ch = dyn_schedule(), dyn_policy_choice()
        _check(lib().dyn_policy_auto(self._h, _ptr(ctx), int(use_graph), C.byref(c), C.byref(ch)))
        return RecordedSchedule(self, c), {"split": bool(ch.split), "cut_row": ch.cut_row,
                                           "est_sequential_us": ch.est_sequential_us, "est_split_us": ch.est_split_us}


    # ---- measured tuning of micro-batch sizes and CU partitions
    @staticmethod
    def _tune_options(max_k, partitions, n_cus, warmup, iters, use_graph, min_gain) -> dyn_tune_options:
        return dyn_tune_options(int(max_k), int(partitions), int(n_cus), int(warmup), int(iters), int(use_graph), float(min_gain))

    def tune_candidates(self, ctx_len: Optional[Sequence[int]] = None, max_k: int = 2, partitions: int = 0,
                        n_cus: int = 0) -> List[dyn_tune_candidate]:
        """The candidate schedules the tuner would time for this batch structure (host only)."""
        ctx = np.ascontiguousarray(ctx_len, dtype=np.int32) if ctx_len is not None else None
        opt = self._tune_options(max_k, partitions, n_cus, 0, 0, 0, -1.0)
        n = lib().dyn_tune_candidates(self._h, _ptr(ctx) if ctx is not None else None, C.byref(opt), None, 0)
        if n < 0:
            raise DynError(DYN_ERR_INVALID_ARG, dyn_last_error())
        table = (dyn_tune_candidate * max(n, 1))()
        lib().dyn_tune_candidates(self._h, _ptr(ctx) if ctx is not None else None, C.byref(opt), table, n)
        return [table[i] for i in range(n)]

    def tune_record(self, cand: dyn_tune_candidate, n_cus: int = 0, use_graph: bool = False) -> RecordedSchedule:
        """Records one candidate (host only)."""
        c = dyn_schedule()
        _check(lib().dyn_tune_record(self._h, C.byref(cand), int(n_cus), int(use_graph), C.byref(c)))
        return RecordedSchedule(self, c)

    def tune(self, layer: "DynLayer", batch, stream, ctx_len: Optional[Sequence[int]] = None, max_k: int = 2,
             partitions: int = 0, warmup: int = 0, iters: int = 0, use_graph: bool = True, min_gain: float = -1.0):
        """Times every candidate on the device (eager launches; use_graph marks the recorded schedule only) and
        records the fastest: returns (schedule, result dict, table of candidate dicts).  batch is a dyn_batch;
        stream a torch stream."""
        ctx = np.ascontiguousarray(ctx_len, dtype=np.int32) if ctx_len is not None else None
        opt = self._tune_options(max_k, partitions, 0, warmup, iters, use_graph, min_gain)
        cap = 256
        table = (dyn_tune_candidate * cap)()
        c, res = dyn_schedule(), dyn_tune_result()
        _check(lib().dyn_tune(layer.handle, C.byref(batch), _ptr(ctx) if ctx is not None else None, C.byref(opt),
                              C.c_void_p(stream.cuda_stream), self._h, C.byref(c), C.byref(res), table, cap))
        n = min(cap, res.n_tried + res.n_skipped)
        return (RecordedSchedule(self, c),
                {"best": res.best.as_dict(), "us_sequential": res.us_sequential, "n_tried": res.n_tried,
                 "n_skipped": res.n_skipped},
                [table[i].as_dict() for i in range(n)])


class DynLayer:
    """Owns a dyn_layer handle and keeps the weight tensors alive."""

    def __init__(self, cfg: dyn_layer_config, weights: List[Dict[str, torch.Tensor]]):
        self.cfg = cfg
        self.weights = weights
        arr = (dyn_layer_weights * len(weights))()
        for i, w in enumerate(weights):
            arr[i] = dyn_layer_weights(*[_ptr(w.get(n)) for n in
                                         ("w_qkv", "w_o", "w_gate_up", "w_down", "g_norm1", "g_norm2", "w_router")])
        self._warr = arr
        h = C.c_void_p()
        _check(lib().dyn_layer_create(C.addressof(cfg), C.cast(arr, C.c_void_p), C.addressof(h)))
        self.handle = h

    def close(self):
        if self.handle:
            lib().dyn_layer_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def workspace_bytes(self, max_tokens: int, max_pages_per_seq: int) -> int:
        return lib().dyn_layer_workspace_bytes(self.handle, max_tokens, max_pages_per_seq)

    def validate(self, batch: dyn_batch, sched: Schedule) -> None:
        sc = sched.to_c()
        _check(lib().dyn_schedule_validate(self.handle, C.addressof(batch), C.addressof(sc)))

    def memory(self, batch: dyn_batch, sched: Schedule) -> dict:
        """Static data-flow analysis of a schedule (host only): reference counts, reshard points
        and the peak of live intermediate bytes next to the sequential order's."""
        sc = sched.to_c()
        rep = dyn_memory_report()
        _check(lib().dyn_schedule_memory(self.handle, C.addressof(batch), C.addressof(sc), C.byref(rep)))
        return rep.as_dict()

    def schedule_workspace_bytes(self, batch: dyn_batch, sched: Schedule) -> int:
        """Workspace bytes a forward of this batch shape with this schedule needs (host only)."""
        sc = sched.to_c()
        return lib().dyn_schedule_workspace_bytes(self.handle, C.addressof(batch), C.addressof(sc))

    def schedule_regions(self, batch: dyn_batch, sched: Schedule) -> List[dict]:
        """The regions of that layout: kind, slot, offset, bytes, set of issue slots during which it is alive."""
        sc = sched.to_c()
        n = C.c_int(0)
        _check(lib().dyn_schedule_regions(self.handle, C.addressof(batch), C.addressof(sc), None, 0, C.addressof(n)))
        arr = (dyn_region * max(1, n.value))()
        _check(lib().dyn_schedule_regions(self.handle, C.addressof(batch), C.addressof(sc), C.cast(arr, C.c_void_p), n.value, C.addressof(n)))
        return [dict(kind=REGION_NAMES[a.kind], slot=a.slot, stream=a.stream, offset=a.offset, bytes=a.bytes,
                     live=a.live_slots[0] | (a.live_slots[1] << 64)) for a in arr[:n.value]]

    def prepare(self, sched: Schedule) -> None:
        """Creates the schedule's side streams now (synchronises the device for CU-masked ones)."""
        sc = sched.to_c()
        _check(lib().dyn_layer_prepare(self.handle, C.addressof(sc)))

    def release_graphs(self) -> None:
        """Waits for and destroys every captured graph of the handle."""
        _check(lib().dyn_layer_release_graphs(self.handle))

    def forward(self, batch: dyn_batch, sched: Schedule, stream: Optional[torch.cuda.Stream] = None) -> None:
        sc = sched.to_c()
        s = stream if stream is not None else torch.cuda.current_stream()
        _check(lib().dyn_layer_forward(self.handle, C.addressof(batch), C.addressof(sc), C.c_void_p(s.cuda_stream)))

    def forward_noalloc(self, batch: dyn_batch, stream: Optional[torch.cuda.Stream] = None) -> None:
        """Sequential forward on the library's static workspace (batch.workspace is ignored)."""
        s = stream if stream is not None else torch.cuda.current_stream()
        _check(lib().dyn_layer_forward_noalloc(self.handle, C.addressof(batch), C.c_void_p(s.cuda_stream)))

    def set_profiling(self, on: bool) -> None:
        _check(lib().dyn_layer_set_profiling(self.handle, int(on)))

    def slot_times(self) -> List[dict]:
        n = C.c_int(0)
        _check(lib().dyn_layer_get_slot_times(self.handle, None, 0, C.addressof(n)))
        arr = (dyn_slot_time * max(1, n.value))()
        _check(lib().dyn_layer_get_slot_times(self.handle, C.cast(arr, C.c_void_p), n.value, C.addressof(n)))
        return [dict(layer=a.layer, op=a.op, nano=a.nano, n_nano=a.n_nano, stream=a.stream, partition=a.partition,
                     start_ms=a.start_ms, main_start_ms=a.main_start_ms, main_stop_ms=a.main_stop_ms,
                     stop_ms=a.stop_ms) for a in arr[:n.value]]


def probe_hbm_read(buf: torch.Tensor, nbytes: int, sink: torch.Tensor, stream: torch.cuda.Stream) -> None:
    """One launch of the library's read-only streaming kernel over the first nbytes of buf."""
    assert sink.numel() * sink.element_size() >= 32768
    _check(lib().dyn_probe_hbm_read(_ptr(buf), nbytes, _ptr(sink), C.c_void_p(stream.cuda_stream)))


def probe_mfma_loop(buf: torch.Tensor, n_stages: int, sink: torch.Tensor, stream: torch.cuda.Stream) -> float:
    """One launch of the library's matrix-core probe on the operands in buf (>= 16 MiB); returns its FLOP count."""
    flops = C.c_double(0.0)
    _check(lib().dyn_probe_mfma_loop(_ptr(buf), buf.numel() * buf.element_size(), n_stages, _ptr(sink),
                                     sink.numel() * sink.element_size(), C.c_void_p(stream.cuda_stream), C.byref(flops)))
    return flops.value


def make_config(sh, kv_chunk_positions: int = 0) -> dyn_layer_config:
    """From a workloads.gen.LayerShape-like object.  kv_chunk_positions: the split-KV chunk of
    decode attention (0: the library's default of 256 positions)."""
    return dyn_layer_config(DYN_BF16 if sh.dtype == "bf16" else DYN_F32, sh.n_layers, sh.hidden, sh.n_q, sh.n_kv,
                            sh.head_dim, sh.inter, sh.n_experts, sh.top_k, sh.eps, sh.rope_base, sh.page_size,
                            kv_chunk_positions)


class DeviceStep:
    """Device copies of one generated step (workloads.gen.generate output) and the dyn_batch
    describing them.  Layer caches are stacked so that kv_layer_stride is uniform, unless the
    caller has placed them layer by layer."""

    def __init__(self, layer: DynLayer, data: dict, device="cuda:0", sched: Optional["Schedule"] = None, guard: int = 0,
                 placed: bool = False, workspace: Optional[torch.Tensor] = None):
        """sched: size the workspace for this schedule alone (dyn_schedule_workspace_bytes) instead of
        for any schedule; guard: extra bytes behind the workspace that the library is not told about;
        placed: data["k_cache"] / data["v_cache"] are lists of per-layer device tensors that stay
        where they are (k_cache_layers / v_cache_layers of the batch) instead of being stacked;
        workspace: a device byte tensor to use (at least the needed bytes + 256) instead of a new one."""
        dev = torch.device(device)
        self.x = data["x"].to(dev)
        self.y = torch.empty_like(self.x)
        self.k_layers = self.v_layers = None
        if placed:
            self.k_layers, self.v_layers = list(data["k_cache"]), list(data["v_cache"])
            assert all(t.is_cuda and t.is_contiguous() for t in self.k_layers + self.v_layers)
            self.k_cache, self.v_cache = self.k_layers[0], self.v_layers[0]
        else:
            self.k_cache = torch.stack([k.to(dev) for k in data["k_cache"]]) if isinstance(data["k_cache"], list) else data["k_cache"]
            self.v_cache = torch.stack([v.to(dev) for v in data["v_cache"]]) if isinstance(data["v_cache"], list) else data["v_cache"]
        self.seq_of_token = torch.from_numpy(data["seq_of_token"]).to(dev)
        self.pos_of_token = torch.from_numpy(data["pos_of_token"]).to(dev)
        self.block_table = torch.from_numpy(np.ascontiguousarray(data["block_table"])).to(dev)
        self.q_start_host = np.ascontiguousarray(data["q_start"], dtype=np.int32)
        n_tokens, n_seqs = self.x.shape[0], len(self.q_start_host) - 1
        max_pages = int(data["block_table"].shape[1])
        stride = 0 if placed else self.k_cache[0].numel() * self.k_cache.element_size()
        self.batch = dyn_batch(n_tokens, n_seqs, _ptr(self.x), _ptr(self.y), _ptr(self.seq_of_token),
                               _ptr(self.pos_of_token), _ptr(self.block_table), max_pages, _ptr(self.q_start_host),
                               _ptr(self.k_cache), _ptr(self.v_cache), stride, None, 0)
        if placed:
            self._k_ptrs = (C.c_void_p * len(self.k_layers))(*[t.data_ptr() for t in self.k_layers])
            self._v_ptrs = (C.c_void_p * len(self.v_layers))(*[t.data_ptr() for t in self.v_layers])
            self.batch.k_cache_layers = C.cast(self._k_ptrs, C.c_void_p)
            self.batch.v_cache_layers = C.cast(self._v_ptrs, C.c_void_p)
        nbytes = layer.workspace_bytes(n_tokens, max_pages) if sched is None else layer.schedule_workspace_bytes(self.batch, sched)
        if workspace is not None:
            assert workspace.is_cuda and workspace.dtype == torch.uint8 and workspace.numel() >= nbytes + 256 + guard
            self.workspace = workspace
        else:
            self.workspace = torch.empty(nbytes + 256 + guard, dtype=torch.uint8, device=dev)
        ws_ptr = (self.workspace.data_ptr() + 255) & ~255
        self.workspace_offset = ws_ptr - self.workspace.data_ptr()
        self.batch.workspace = ws_ptr
        self.batch.workspace_bytes = nbytes
        # uploads were queued on torch's current stream; forwards run on other, non-blocking
        # streams, so wait here until the inputs have landed
        torch.cuda.synchronize(dev)
