"""The assignment step of the measured cache placement (pure host logic; the probing itself
needs a GPU and is covered by the benchmark's GPU test)."""
import pytest

from paper_2605_21603_amd import placement as P


def test_fastest_pairs_first_within_each_chunks_capacity():
    times = {(0, 0): 950.0, (0, 1): 870.0, (0, 2): 830.0, (1, 1): 950.0, (1, 2): 868.0, (2, 2): 940.0}
    plan = P.assign(times, n_layers=4, slots_per_chunk=3, n_chunks=3)
    # three layers fit the fastest pair (0, 2), which fills both chunks; chunk 1 then hosts one layer with two of its slots
    assert [(p[0], p[2]) for p in plan[:3]] == [(0, 2)] * 3
    assert [p[4] for p in plan[:3]] == [830.0] * 3
    assert (plan[3][0], plan[3][2]) == (1, 1) and plan[3][1] != plan[3][3] and plan[3][4] == 950.0


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
