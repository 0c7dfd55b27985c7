"""The assignment step of the measured cache placement (pure host logic; the probing itself
needs a GPU and is covered by the benchmark's GPU test)."""
import pytest

from paper_2605_21603_amd import placement as P


def test_fastest_pairs_first_then_partners_are_traded():
    times = {(0, 0): 950.0, (0, 1): 870.0, (0, 2): 830.0, (1, 1): 950.0, (1, 2): 868.0, (2, 2): 940.0}
    plan = P.assign(times, n_layers=4, slots_per_chunk=3, n_chunks=3)
    # greedy alone: three layers on (0, 2), which fills both chunks, and the fourth on (1, 1) at 950; trading partners
    # with one of the three gives (0, 2), (0, 2), (1, 2), (0, 1)
    assert sorted(p[4] for p in plan) == [830.0, 830.0, 868.0, 870.0]
    assert sorted(tuple(sorted((p[0], p[2]))) for p in plan) == [(0, 1), (0, 2), (0, 2), (1, 2)]


def test_slots_are_distinct_and_inside_their_chunks():
    times = {(i, j): 800.0 + 10 * abs(i - j) + (100 if i == j else 0) for i in range(4) for j in range(i, 4)}
    plan = P.assign(times, n_layers=10, slots_per_chunk=6, n_chunks=4)
    used = set()
    for kc, ks, vc, vs, _ in plan:
        assert 0 <= ks < 6 and 0 <= vs < 6
        assert (kc, ks) not in used and (vc, vs) not in used and (kc, ks) != (vc, vs)
        used.add((kc, ks))
        used.add((vc, vs))
    assert len(used) == 20


def test_not_enough_room_is_an_error():
    with pytest.raises(RuntimeError):
        P.assign({(0, 0): 1.0, (0, 1): 1.0, (1, 1): 1.0}, n_layers=3, slots_per_chunk=2, n_chunks=2)


def test_slot_size_is_rounded_to_256_bytes():
    import torch
    assert P.slot_bytes_of((3, 2, 16, 8), torch.bfloat16) == 1536
    assert P.slot_bytes_of((3, 2, 16, 9), torch.bfloat16) == 1792


def test_layers_trade_partners_instead_of_ending_in_the_slowest_class():
    """Chunk classes a (0, 1), b (2), c (3, 4): a with b is fast, c with c slow, everything else in
    the middle.  Greedy alone pairs the a chunks' left-over slots with each other and leaves the
    last layers (c, c); after the exchange pass no layer is in the slowest class."""
    cls = {0: "a", 1: "a", 2: "b", 3: "c", 4: "c"}
    def t(i, j):
        x, y = sorted((cls[i], cls[j]))
        return {("a", "b"): 830.0, ("c", "c"): 950.0}.get((x, y), 868.0 + 0.01 * (i + j))
    times = {(i, j): t(i, j) for i in range(5) for j in range(i, 5)}
    plan = P.assign(times, n_layers=12, slots_per_chunk=6, n_chunks=5)
    costs = sorted(p[4] for p in plan)
    assert costs[:6] == [830.0] * 6              # chunk 2 has six slots: six layers in the fast class
    assert max(costs) < 900.0                    # and nobody in the slowest
    used = {}
    for kc, ks, vc, vs, _ in plan:
        for c, s_ in ((kc, ks), (vc, vs)):
            assert (c, s_) not in used and 0 <= s_ < 6
            used[(c, s_)] = 1


def test_chunk_rule_follows_the_decode_work_items_per_wave():
    from workloads import gen
    for name, want in (("c5", 1024), ("c2", 256), ("c3", 256), ("c4", 256), ("c2_small", 256)):
        w = gen.config(name)
        assert P.rule_chunk([c for _, c in w.seqs], [q for q, _ in w.seqs], w.shape.n_kv) == want, name
    # a prefill chunk's tokens are not decode work items
    assert P.rule_chunk([8192] * 4, [4096] * 4, 8) == 256
