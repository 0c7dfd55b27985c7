"""GPU tests of the measured tuner (unequal micro-batch sizes and CU shares, the knobs of
Section 2.1): whatever it picks reproduces the sequential step bit for bit and matches the
oracle, every candidate was timed, and the winner is the fastest of the table or the
sequential order when no overlapped schedule earns its margin."""
import sys

import pytest
import torch

from paper_2605_21603_amd import binding as B
from workloads import gen

from gpu_util import GpuRun, check_against_oracle

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, file=sys.stderr, flush=True)


# The searches below once timed every candidate as a HIP graph (capture, replay, destroy, dozens per search) and ended
# in a segmentation fault inside the runtime three times - with four micro-batches at the 50th graph of a process, with
# three late in the full suite, at last with two - without a cause that could be shown in this library (its host side
# replays clean under sanitizers on the CPU: tests/test_host_sanitizer.py).  That code path is gone: dyn_tune times its
# candidates with eager launches and captures nothing, so these cases run what every other eager test runs.
def test_tuning_with_four_micro_batches():
    _tune_and_check("c2_small", 4, 1)


@pytest.mark.parametrize("name,max_k,partitions", [("c2_small", 3, 0), ("c5_small", 3, 1)])
def test_tuning_with_three_micro_batches(name, max_k, partitions):
    _tune_and_check(name, max_k, partitions)


def test_device_search_rejects_more_than_four_micro_batches():
    w = gen.config("c2_small")
    data = gen.generate(w)
    run = GpuRun(w, data)
    md = gen.metadata(w)
    step = B.DeviceStep(run.layer, data, run.device)
    sch = B.Scheduler(B.make_config(w.shape), md["q_start"])
    with pytest.raises(B.DynError) as e:
        sch.tune(run.layer, step.batch, torch.cuda.Stream(), ctx_len=md["ctx_len"], max_k=5)
    assert e.value.status == B.DYN_ERR_INVALID_ARG


@pytest.mark.parametrize("name,max_k,partitions", [("c2_small", 2, 1), ("c3_small", 2, 1), ("c4_small", 2, 0),
                                                   ("c5_small", 2, 0)])
def test_tuned_schedule_is_bit_exact_and_the_table_is_consistent(name, max_k, partitions):
    _tune_and_check(name, max_k, partitions)


def _tune_and_check(name, max_k, partitions):
    w = gen.config(name)
    data = gen.generate(w)
    run = GpuRun(w, data)
    md = gen.metadata(w)
    say("case %s: sequential" % name)
    y0, k0, v0 = run.run(B.sequential())
    check_against_oracle(w, data, y0, k0, v0)
    step = B.DeviceStep(run.layer, data, run.device)
    sch = B.Scheduler(B.make_config(w.shape), md["q_start"])
    st = torch.cuda.Stream()
    say("case %s: tuning" % name)
    sched, res, table = sch.tune(run.layer, step.batch, st, ctx_len=md["ctx_len"], max_k=max_k, partitions=partitions,
                                 warmup=1, iters=3, use_graph=True, min_gain=0.02)
    torch.cuda.synchronize()
    say("case %s: best %s of %d tried, %d skipped, sequential %.1f us" % (name, res["best"], res["n_tried"],
                                                                          res["n_skipped"], res["us_sequential"]))
    expected = sch.tune_candidates(md["ctx_len"], max_k=max_k, partitions=partitions)
    assert res["n_tried"] + res["n_skipped"] == len(expected) == len(table)
    assert table[0]["form"] == "sequential" and table[0]["us"] == res["us_sequential"] > 0
    timed = [c for c in table if c["us"] > 0]
    assert len(timed) == res["n_tried"] and res["n_tried"] >= 1 + (len(expected) - 1) // 2
    fastest = min(timed, key=lambda c: c["us"])
    if fastest["us"] <= 0.98 * res["us_sequential"]:
        assert res["best"]["us"] == fastest["us"]
    else:
        assert res["best"]["form"] == "sequential"
    # the tuning forwards wrote the same result every time: the buffers hold the step's output
    assert torch.equal(step.y.cpu().view(torch.uint8), y0.view(torch.uint8))
    # the recorded winner, on fresh buffers
    assert sched.nano_rows == res["best"]["rows"]
    y, kc, vc = run.run(sched, repeat=2)
    assert torch.equal(y.view(torch.uint8), y0.view(torch.uint8))
    assert torch.equal(kc.view(torch.uint8), k0.view(torch.uint8))
    assert torch.equal(vc.view(torch.uint8), v0.view(torch.uint8))


def test_every_overlapped_form_of_the_table_is_bit_exact_on_a_prefill_decode_mix():
    """The tuner's candidates themselves, one per (form, partitioned or not), eager."""
    w = gen.config("c3_small")
    data = gen.generate(w)
    run = GpuRun(w, data)
    md = gen.metadata(w)
    y0, k0, v0 = run.run(B.sequential())
    sch = B.Scheduler(B.make_config(w.shape), md["q_start"])
    seen = set()
    for c in sch.tune_candidates(md["ctx_len"], max_k=2, partitions=1):
        key = (c.form, c.cus_first > 0)
        if key in seen:
            continue
        seen.add(key)
        say("candidate %s" % c.as_dict())
        y, kc, vc = run.run(sch.tune_record(c, n_cus=256))
        assert torch.equal(y.view(torch.uint8), y0.view(torch.uint8)), c.as_dict()
        assert torch.equal(kc.view(torch.uint8), k0.view(torch.uint8)), c.as_dict()
        assert torch.equal(vc.view(torch.uint8), v0.view(torch.uint8)), c.as_dict()
    assert len(seen) == 7
