"""Host side of libdynlayer on the CPU under AddressSanitizer + UndefinedBehaviorSanitizer.

Every source of the library is compiled for the host only (hipcc --cuda-host-only: the kernels
become launch stubs) and linked against tests/host_sim/hip_stub.cpp, a stand-in for the HIP
runtime that keeps streams, events, graphs and executables as host objects, completes nothing
before the host waits for it, and reports every misuse (use after destroy, a wait on a stale
capture event, an executable destroyed while its launch may still run, work left unjoined at
the end of a capture, ...).  tests/host_sim/replay.cpp then drives the call sequences that
matter for object lifetimes: a tuning run - also with four micro-batches, which the device
search itself refuses after a fault inside hipGraphLaunch on the GPU - a run that overflows the
graph cache without host waits, and a mix of eager, profiled, captured, CU-masked and
allocation-free forwards.  Nothing here needs a GPU."""
import json
import os
import subprocess

import pytest

from workloads import gen

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SIM = os.path.join(HERE, "host_sim")
BUILD = os.path.join(SIM, "_build")
CSRC = os.path.join(ROOT, "paper_2605_21603_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANGXX = "/opt/rocm/lib/llvm/bin/clang++"
# host pass only; each sanitizer flag goes to the host compiler
HOST_FLAGS = ["-O1", "-g", "--cuda-host-only", "-std=c++17", "-fPIC", "-x", "hip", "-fno-omit-frame-pointer",
              "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
              "-Xarch_host", "-fno-sanitize-recover=undefined"]


def _build():
    from paper_2605_21603_amd.build import SOURCES
    os.makedirs(BUILD, exist_ok=True)
    jobs = []
    srcs = [os.path.join(CSRC, s) for s in SOURCES] + [os.path.join(SIM, "hip_stub.cpp"), os.path.join(SIM, "replay.cpp")]
    objs = []
    for src in srcs:
        obj = os.path.join(BUILD, os.path.splitext(os.path.basename(src))[0] + ".o")
        objs.append(obj)
        jobs.append((src, subprocess.Popen([HIPCC] + HOST_FLAGS + ["-c", src, "-o", obj], stdout=subprocess.PIPE,
                                           stderr=subprocess.STDOUT, text=True)))
    for src, p in jobs:
        out, _ = p.communicate()
        assert p.returncode == 0, "host-only build of %s failed:\n%s" % (src, out)
    # the host pass refers to the device code object of each source by a symbol the device pass would define
    fatbins = set()
    for obj in objs:
        for line in subprocess.check_output(["nm", "-u", obj], text=True).splitlines():
            name = line.split()[-1]
            if name.startswith("__hip_fatbin"):
                fatbins.add(name)
    shim = os.path.join(BUILD, "fatbin_symbols.c")
    with open(shim, "w") as f:
        f.write("".join("const char %s[8] = {0};\n" % n for n in sorted(fatbins)))
    exe = os.path.join(BUILD, "replay")
    subprocess.check_call([CLANGXX, "-fsanitize=address,undefined", "-o", exe] + objs + ["-x", "c", shim])
    return exe


@pytest.fixture(scope="module")
def replay():
    if not os.path.exists(HIPCC) or not os.path.exists(CLANGXX):
        pytest.skip("no ROCm toolchain")
    return _build()


def _shape_file(name):
    w = gen.config(name)
    sh = w.shape
    path = os.path.join(BUILD, "shape_%s.txt" % name)
    with open(path, "w") as f:
        f.write("%d %d %d %d %d %d %d %d %d %d %d\n" % (1 if sh.dtype == "bf16" else 0, sh.n_layers, sh.hidden, sh.n_q, sh.n_kv,
                                                      sh.head_dim, sh.inter, sh.n_experts, sh.top_k, sh.page_size, w.n_seqs))
        f.write("".join("%d %d\n" % (q, c) for q, c in w.seqs))
    return path


def _run(exe, name, *mode):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)          # the sanitizer runtime has to come first in the process
    p = subprocess.run([exe, _shape_file(name)] + [str(m) for m in mode], stdout=subprocess.PIPE, stderr=subprocess.PIPE,
                       text=True, env=env, timeout=600)
    assert p.returncode == 0, "replay %s %s: exit %d\n%s\n%s" % (name, mode, p.returncode, p.stdout, p.stderr[-6000:])
    assert "ERROR: AddressSanitizer" not in p.stderr and "runtime error" not in p.stderr, p.stderr[-6000:]
    stats = json.loads(p.stdout.strip().splitlines()[-1])
    assert stats["violations"] == 0 and stats["failures"] == 0
    assert stats["live_events"] == 0 and stats["live_graphs"] == 0 and stats["live_execs"] == 0
    assert stats["masked_streams_destroyed"] == 0          # CU-masked streams are never destroyed
    return stats


def test_the_stand_in_detects_each_misuse_it_is_there_for(replay):
    """Every kind of misuse is committed once against the stand-in directly and must be counted:
    a checker that sees nothing proves nothing."""
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0")
    env.pop("LD_PRELOAD", None)
    p = subprocess.run([replay, "selftest"], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, env=env, timeout=120)
    assert p.returncode == 0, p.stdout + p.stderr[-4000:]
    out = json.loads(p.stdout.strip().splitlines()[-1])
    assert out["missed"] == 0 and out["violations"] >= 14


def test_tuning_run_with_four_micro_batches_keeps_every_object_alive_while_used(replay):
    """The sequence that ended in a segmentation fault inside hipGraphLaunch on the GPU: 13
    tokens, candidates with up to four micro-batches, one CU-share pair, one warm-up and three
    timed runs of three replays each.  (The candidates on CU partitions, captured like the others
    at the time, are issued eagerly now: 38 graphs instead of 51.)"""
    stats = _run(replay, "c2_small", "tune", 4, 1, 1, 3)
    assert stats["captures"] == stats["instantiations"] >= 38
    assert stats["execs_destroyed"] == stats["instantiations"]
    assert stats["max_live_execs"] <= 17 and stats["max_live_side_branches"] <= 20
    assert stats["empty_branches"] == 0                      # no stream is forked into a capture without launching in it


@pytest.mark.parametrize("name,max_k,partitions", [("c2_small", 3, 1), ("c2_small", 2, 3), ("c3_small", 2, 3), ("c4_small", 3, 0), ("c5_small", 3, 1), ("c5_small", 2, 1)])
def test_tuning_runs(replay, name, max_k, partitions):
    stats = _run(replay, name, "tune", max_k, partitions, 1, 2)
    assert stats["graph_launches"] > 0 and stats["execs_destroyed"] == stats["instantiations"]


@pytest.mark.parametrize("name", ["c2_small", "c5_small"])
def test_graph_cache_overflow_without_host_waits(replay, name):
    """Executables evicted while their last replay has not completed are destroyed only after it has."""
    stats = _run(replay, name, "evict")
    assert stats["instantiations"] > 40 and stats["execs_destroyed"] == stats["instantiations"]
    # 16 cached + at most 8 evicted ones waiting for their last replay + the one being added
    assert stats["max_live_execs"] <= 25 and stats["max_live_side_branches"] <= 25


@pytest.mark.parametrize("name", ["c2_small", "c3_small", "c4_small", "f32_small", "stack_mixed"])
def test_mixed_eager_profiled_captured_masked_and_allocation_free_forwards(replay, name):
    stats = _run(replay, name, "mixed")
    assert stats["kernel_launches"] > 1000


@pytest.mark.parametrize("name,k,stagger,mem_cus", [("c5_small", 2, 2, 160), ("c5_small", 4, 2, 192), ("c4_small", 2, 4, 128)])
def test_partitions_by_operator_class_are_issued_eagerly(replay, name, k, stagger, mem_cus):
    """Every micro-batch's attention on one CU partition and its other operators on another, so
    consecutive operators of a micro-batch change streams; use_graph is set, and nothing may be
    captured, because a replayed graph would drop the masks."""
    stats = _run(replay, name, "opclass", k, stagger, mem_cus, 1)
    assert stats["captures"] == 0 and stats["graph_launches"] == 0 and stats["kernel_launches"] > 100
