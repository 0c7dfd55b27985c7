"""Host-side checks of bench.py's bookkeeping (no GPU): the algorithmic bytes and FLOPs its roofline figures divide by,
the committed counter figures, and the single-GPU contract."""
import json
import os
import subprocess
import sys

import bench
from workloads import gen

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_algorithmic_bytes_and_flops_are_the_layer_shapes_own_arithmetic():
    """Restated from the layer's dimensions rather than from bench.py's expressions: 4096 B per cached position and
    layer (K and V, 8 kv heads x 128 x 2 B), 436.2 MB and 436.2 MFLOP per token of projections for the Llama-3-8B
    layer, 16384 FLOP of attention per (query, key) pair."""
    for name in ("c2", "c5"):
        w = gen.config(name)
        cached = sum(c for _, c in w.seqs)
        assert w.shape.n_kv * w.shape.head_dim * 2 * 2 == 4096
        assert bench.attention_bytes(w) == 4096 * cached + 2 * w.n_tokens * 4096 * 2        # + q in and o out, 4096 bf16 each
        params = 4096 * 6144 + 4096 * 4096 + 4096 * 28672 + 14336 * 4096
        assert params == 218103808
        byts, flops = bench.layer_bytes_flops(w)
        L = w.shape.n_layers
        act = w.n_tokens * 2 * (2 * 4096 * 4 + 2 * 6144 + 2 * 4096 + 3 * 2 * 14336)
        assert byts == L * (params * 2 + bench.attention_bytes(w) + act)
        assert flops == L * (2 * params * w.n_tokens + 16384 * cached)                      # one query per sequence: pairs = cached positions
    assert bench.attention_bytes(gen.config("c5")) == 4995624960
    assert bench.attention_bytes(gen.config("c2")) == 1230270464
    gb, gf = bench.gate_up_bytes_flops(gen.config("c3"))
    assert gf == 2 * 2112 * 4096 * 28672 == 496068722688
    assert gb == 28672 * 4096 * 2 + 2112 * 4096 * 2 + 2112 * 14336 * 2


def test_committed_counter_figures_belong_to_the_attention_kernel_as_it_is():
    """bench.py withholds `roofline.traffic` when the kernel's source no longer is the one the counters were read on;
    a change to that source has to come with a new counter run, and this is where that shows."""
    h = bench.source_hash(bench.ATTN_SOURCE)
    for wl, t in bench.ROCPROF_TRAFFIC.items():
        assert t["source_sha256_16"] == h, "re-run the counters for %s (profiles/) and update bench.ROCPROF_TRAFFIC" % wl
        assert os.path.exists(os.path.join(ROOT, t["source"].split(" ")[0]))
        # the fetched bytes are within a few percent of the algorithmic ones: no wasted re-reads
        assert 1.0 <= t["bytes"] / bench.attention_bytes(gen.config(wl)) < 1.06


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE, stderr=subprocess.PIPE,
                       text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in (p.stderr + p.stdout)
    assert not any(l.startswith("{") and "metric" in json.loads(l) for l in p.stdout.splitlines() if l.startswith("{"))
