"""Pins of the storage-allocation oracle (Section 4.2): instances solved by inspection, an
independent exact method (first fit over every placement order), bounds, special cases."""
import itertools

import numpy as np
import pytest

from oracle import memo_dsa_oracle as do


def _first_fit_all_orders(req):
    """Independent exact method: an optimal plan sorted by address is reproduced by placing the
    requests in that order, each at the lowest address free of its time-overlapping predecessors."""
    best = None
    for order in itertools.permutations(range(len(req))):
        addr = {}
        for i in order:
            s, a, b = req[i]
            busy = sorted((addr[j], addr[j] + req[j][0]) for j in addr if req[j][1] < b and a < req[j][2])
            x = 0
            for lo, hi in busy:
                if x + s <= lo:
                    break
                x = max(x, hi)
            addr[i] = x
        peak = max(addr[i] + req[i][0] for i in addr)
        best = peak if best is None else min(best, peak)
    return best


def test_instances_solved_by_inspection():
    # two tensors alive together must be stacked; a third that only meets the first reuses the second's room
    assert do.solve_exact([(4, 0, 2), (3, 0, 1), (3, 1, 2)])[0] == 7
    # disjoint lifespans share one address
    peak, addr = do.solve_exact([(5, 0, 1), (9, 1, 2), (2, 2, 3)])
    assert peak == 9 and addr == [0, 0, 0]
    # everything alive at once: the peak is the sum
    assert do.solve_exact([(1, 0, 5), (2, 0, 5), (3, 0, 5), (4, 0, 5)])[0] == 10
    # a long-lived small tensor between two big short ones: it goes to one end, not the middle
    req = [(1, 0, 4), (3, 0, 2), (3, 2, 4)]
    peak, addr = do.solve_exact(req)
    assert peak == 4 and do.check_plan(req, addr) == 4
    assert do.solve_exact([])[0] == 0


def test_overlap_uses_half_open_lifespans():
    # [0,2) and [2,4) do not overlap: freed memory is reusable at the very tick it is freed
    assert do.overlapping_pairs([(1, 0, 2), (1, 2, 4)]) == []
    assert do.overlapping_pairs([(1, 0, 3), (1, 2, 4)]) == [(0, 1)]


@pytest.mark.parametrize("seed", range(25))
def test_two_exact_methods_agree_and_respect_the_bounds(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 6))
    req = []
    for _ in range(n):
        a = int(rng.integers(0, 5))
        req.append((int(rng.integers(1, 9)), a, int(rng.integers(a + 1, 8))))
    peak, addr = do.solve_exact(req)
    assert do.check_plan(req, addr) == peak
    assert peak == _first_fit_all_orders(req)
    assert do.load_lower_bound(req) <= peak <= sum(r[0] for r in req)


def test_unit_sizes_need_exactly_the_largest_clique():
    # interval graphs are perfect: with unit sizes the optimum is the largest number alive at once
    rng = np.random.default_rng(99)
    for _ in range(10):
        req = []
        for _ in range(5):
            a = int(rng.integers(0, 5))
            req.append((1, a, int(rng.integers(a + 1, 8))))
        assert do.solve_exact(req)[0] == do.load_lower_bound(req)


def test_check_plan_rejects_overlap():
    with pytest.raises(AssertionError):
        do.check_plan([(4, 0, 2), (4, 1, 3)], [0, 2])
    assert do.check_plan([(4, 0, 2), (4, 2, 3)], [0, 2]) == 6


def test_trace_to_requests():
    ev = [("malloc", "a", 8), ("malloc", "b", 4), ("free", "a", 8), ("malloc", "c", 2), ("free", "c", 2)]
    req, ids = do.trace_to_requests(ev)
    assert ids == ["a", "b", "c"]
    assert req == [(8, 0, 2), (4, 1, 5), (2, 3, 4)]        # b is never freed: alive to the end
    with pytest.raises(ValueError):
        do.trace_to_requests([("free", "x", 1)])
    with pytest.raises(ValueError):
        do.trace_to_requests([("malloc", "x", 1), ("free", "x", 2)])


def test_bilevel_small_example_by_inspection():
    # one layer's forward: two transient tensors alive together (3 + 2) then a third of 4 alone -> 5;
    # backward: a single tensor of 6.  Three layers: forward passes at ticks 1,2,3, backward at 5,4,... 
    fwd = [(3, 0, 2), (2, 1, 2), (4, 2, 3)]
    bwd = [(6, 0, 1)]
    # outside the layers: a loss buffer of 7 alive only between the passes (tick 4)
    plan = do.bilevel(fwd, bwd, [1, 2, 3], [7, 6, 5], [(7, 4, 5)])
    assert plan["fwd_peak"] == 5 and plan["bwd_peak"] == 6
    # every pass and the loss buffer are disjoint in time: all share address 0, the peak is 7
    assert plan["peak"] == 7
    assert plan["fwd_base"] == [0, 0, 0] and plan["bwd_base"] == [0, 0, 0] and plan["outer_addr"] == [0]
    # an embedding buffer of 10 alive from the start through every forward pass sits beside them
    plan = do.bilevel(fwd, bwd, [1, 2, 3], [7, 6, 5], [(7, 4, 5), (10, 0, 4)])
    assert plan["peak"] == 15
    assert do.check_plan(plan["level2_requests"], plan["outer_addr"] + plan["fwd_base"] + plan["bwd_base"]) == 15
    # ... and if it also lives through the loss and the backward passes, the loss buffer decides: 10 + 7
    plan = do.bilevel(fwd, bwd, [1, 2, 3], [7, 6, 5], [(7, 4, 5), (10, 0, 8)])
    assert plan["peak"] == 17
    # the flat problem (every tensor of every layer as its own request) cannot do better than the
    # two-level plan here, and the two-level plan is never below the flat optimum
    flat = [(10, 0, 24), (7, 12, 15)]
    for l in range(3):
        flat += [(sz, 3 * (l + 1) + a, 3 * (l + 1) + b) for sz, a, b in fwd]
    for k, l in enumerate((2, 1, 0)):
        flat += [(6, 15 + 3 * k, 16 + 3 * k)]
    assert do.load_lower_bound(flat) <= 17
