"""GPU tests of schedules recorded through the programmable scheduling calls (Section 3.2.2,
Figure 6): strategies written as short programs over split / get_ready_ops / execute run
on the device and reproduce the sequential step bit for bit, against the oracle within
tolerance; the built-in policy's choice does too."""
import sys

import pytest
import torch

from paper_2605_21603_amd import binding as B
from workloads import gen

from gpu_util import GpuRun, check_against_oracle

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, file=sys.stderr, flush=True)


def round_robin(sch, k):
    while True:
        issued = False
        for b in range(k):
            ready = sch.get_ready_ops(b)
            if ready:
                sch.execute([(ready[0], b)], stream=b)
                issued = True
        if not issued:
            return


def attention_split_mlp_merged(sch, k, chain):
    """Micro-batches run up to the second norm on their own streams, one operator apart
    (so one's attention meets another's projections); the MLP runs once for all of them:
    no second read of the MLP weights."""
    head = [op for op in chain if op < B.DYN_OP_ROUTE]
    tail = [op for op in chain if op >= B.DYN_OP_ROUTE]
    for step in range(len(head) + k - 1):
        for b in range(k):
            i = step - b
            if 0 <= i < len(head):
                assert sch.get_ready_ops(b) == [head[i]]
                sch.execute([(head[i], b)], stream=b)
    for op in tail:
        sch.execute([(op, b) for b in range(k)], stream=0)


def sizes_of(w):
    r = list(w.nano_rows)
    return [r[i + 1] - r[i] for i in range(len(r) - 1)]


@pytest.mark.parametrize("name", ["c1", "c2_small", "c3_small", "c4_small", "c5_small"])
def test_recorded_strategies_are_bit_exact_and_match_the_oracle(name):
    w = gen.config(name)
    data = gen.generate(w)
    run = GpuRun(w, data)
    say("case %s: sequential" % name)
    y0, k0, v0 = run.run(B.sequential())
    check_against_oracle(w, data, y0, k0, v0)
    chain = B.MOE_CHAIN if w.shape.n_experts else B.DENSE_CHAIN
    k = len(w.nano_rows) - 1
    md = gen.metadata(w)
    recorded = {}
    sch = B.Scheduler(B.make_config(w.shape), md["q_start"])
    sch.split(sizes_of(w))
    round_robin(sch, k)
    recorded["round robin"] = sch.finish()
    sch2 = B.Scheduler(B.make_config(w.shape), md["q_start"])
    sch2.split(sizes_of(w))
    attention_split_mlp_merged(sch2, k, chain)
    recorded["attention split, MLP merged, graph"] = sch2.finish(use_graph=True)
    sch3 = B.Scheduler(B.make_config(w.shape), md["q_start"])
    recorded["policy"], choice = sch3.auto(md["ctx_len"])
    say("case %s: policy chose %s" % (name, choice))
    for label, sched in recorded.items():
        say("case %s: %s" % (name, label))
        y, kc, vc = run.run(sched, repeat=2 if "graph" in label else 1)
        assert torch.equal(y.view(torch.uint8), y0.view(torch.uint8)), label
        assert torch.equal(kc.view(torch.uint8), k0.view(torch.uint8)), label
        assert torch.equal(vc.view(torch.uint8), v0.view(torch.uint8)), label


def test_policy_choice_and_forced_split_of_a_prefill_decode_mix_are_bit_exact():
    """A long prefill chunk beside decodes at a reduced hidden size: the schedule the policy
    records (whichever way it decides) and a forced two-stream split at the prefill / decode
    boundary, both as HIP graphs or eager, against the sequential order."""
    w = gen.config("c3_mid")
    data = gen.generate(w)
    run = GpuRun(w, data)
    md = gen.metadata(w)
    sch = B.Scheduler(B.make_config(w.shape), md["q_start"])
    sched, choice = sch.auto(md["ctx_len"], use_graph=True)
    say("c3_mid: policy chose %s" % choice)
    y0, k0, v0 = run.run(B.sequential())
    y, kc, vc = run.run(sched, repeat=2)
    assert torch.equal(y.view(torch.uint8), y0.view(torch.uint8))
    assert torch.equal(kc.view(torch.uint8), k0.view(torch.uint8))
    assert torch.equal(vc.view(torch.uint8), v0.view(torch.uint8))
    # whatever the policy chose, a forced split at the prefill / decode boundary is legal and exact
    cut = next(int(md["q_start"][i]) for i in range(1, w.n_seqs)
               if (md["q_start"][i] - md["q_start"][i - 1] > 1) != (md["q_start"][i + 1] - md["q_start"][i] > 1))
    sch.split([cut, w.n_tokens - cut])
    round_robin(sch, 2)
    y, kc, vc = run.run(sch.finish())
    assert torch.equal(y.view(torch.uint8), y0.view(torch.uint8))
    assert torch.equal(kc.view(torch.uint8), k0.view(torch.uint8))
