"""The storage-allocation planner of the library (Section 4.2) against the oracle: the exact
search reaches the optimum of the enumerated mixed-integer programme, plans are valid, the
two-level composition matches, a node budget degrades to a valid plan.  CPU only."""
import ctypes
import time

import numpy as np
import pytest

from oracle import memo_dsa_oracle as do
from paper_2407_12117_amd import binding as mb


def _random_requests(rng, n, tmax=8, smax=9):
    req = []
    for _ in range(n):
        a = int(rng.integers(0, tmax - 1))
        req.append((int(rng.integers(1, smax + 1)), a, int(rng.integers(a + 1, tmax + 1))))
    return req


@pytest.mark.parametrize("seed", range(40))
def test_exact_search_reaches_the_mip_optimum(seed):
    rng = np.random.default_rng(seed)
    req = _random_requests(rng, int(rng.integers(1, 7)))
    peak, addr, proven = mb.memo_dsa_plan(req)
    assert proven
    assert do.check_plan(req, addr) == peak
    assert peak == do.solve_exact(req)[0]


def test_instances_solved_by_inspection():
    assert mb.memo_dsa_plan([(4, 0, 2), (3, 0, 1), (3, 1, 2)])[0] == 7
    assert mb.memo_dsa_plan([(5, 0, 1), (9, 1, 2), (2, 2, 3)])[:2] == (9, [0, 0, 0])
    assert mb.memo_dsa_plan([(1, 0, 5), (2, 0, 5), (3, 0, 5), (4, 0, 5)])[0] == 10
    assert mb.memo_dsa_plan([(1, 0, 4), (3, 0, 2), (3, 2, 4)])[0] == 4
    assert mb.memo_dsa_plan([]) == (0, [], True)


def test_alignment_rounds_sizes_and_addresses():
    req = [(100, 0, 2), (300, 0, 2), (10, 1, 3)]
    peak, addr, _ = mb.memo_dsa_plan(req, align=256)
    assert all(a % 256 == 0 for a in addr)
    rounded = [((s + 255) // 256 * 256, a, b) for s, a, b in req]
    assert do.check_plan(rounded, addr) == peak == do.solve_exact(rounded)[0]


@pytest.mark.parametrize("seed", range(5))
def test_larger_instances_are_valid_and_between_the_bounds(seed):
    rng = np.random.default_rng(100 + seed)
    req = _random_requests(rng, 40, tmax=30, smax=64)
    peak, addr, proven = mb.memo_dsa_plan(req, node_limit=200_000)
    assert do.check_plan(req, addr) == peak
    assert do.load_lower_bound(req) <= peak <= sum(r[0] for r in req)
    # never worse than what an allocator that sees the requests in program order would do
    order = sorted(range(len(req)), key=lambda i: req[i][1])
    online = {}
    for i in order:
        busy = sorted((online[j], online[j] + req[j][0]) for j in online
                      if req[j][1] < req[i][2] and req[i][1] < req[j][2])
        x = 0
        for lo, hi in busy:
            if x + req[i][0] <= lo:
                break
            x = max(x, hi)
        online[i] = x
    assert peak <= max(online[i] + req[i][0] for i in online)
    if proven:
        assert peak >= do.load_lower_bound(req)


def test_node_budget_of_zero_still_returns_a_valid_plan():
    rng = np.random.default_rng(7)
    req = _random_requests(rng, 12, tmax=10)
    peak, addr, proven = mb.memo_dsa_plan(req, node_limit=0)
    assert do.check_plan(req, addr) == peak
    full = mb.memo_dsa_plan(req)
    assert full[0] <= peak
    assert proven == (peak == do.load_lower_bound(req))


def test_trace_conversion_matches_oracle():
    ev = [("malloc", 1, 8), ("malloc", 2, 4), ("free", 1, 8), ("malloc", 3, 2), ("free", 3, 2), ("malloc", 1, 16)]
    req, ids = mb.memo_trace_to_requests(ev)
    # the oracle wants unique names: the second life of id 1 is called "d" there
    oreq, oids = do.trace_to_requests([("malloc", "a", 8), ("malloc", "b", 4), ("free", "a", 8), ("malloc", "c", 2),
                                       ("free", "c", 2), ("malloc", "d", 16)])
    assert req == oreq and ids == [1, 2, 3, 1]             # an id may be reused after its free
    for bad in ([("free", 1, 8)], [("malloc", 1, 8), ("malloc", 1, 8)], [("malloc", 1, 8), ("free", 1, 4)]):
        with pytest.raises(mb.MemoError) as e:
            mb.memo_trace_to_requests(bad)
        assert e.value.status == mb.MEMO_ERR_INVALID_ARG


@pytest.mark.parametrize("seed", range(8))
def test_bilevel_matches_oracle(seed):
    rng = np.random.default_rng(200 + seed)
    fwd = _random_requests(rng, int(rng.integers(1, 6)), tmax=6)
    bwd = _random_requests(rng, int(rng.integers(1, 6)), tmax=6)
    nl = int(rng.integers(1, 4))
    fwd_ticks = list(range(1, 1 + nl))
    bwd_ticks = list(range(2 * nl + 1, nl + 1, -1))
    outer = _random_requests(rng, int(rng.integers(0, 3)), tmax=2 * nl + 3, smax=20)
    got = mb.memo_dsa_plan_bilevel(fwd, bwd, fwd_ticks, bwd_ticks, outer)
    want = do.bilevel(fwd, bwd, fwd_ticks, bwd_ticks, outer)
    assert got["optimal"]
    assert (got["peak"], got["fwd_peak"], got["bwd_peak"]) == (want["peak"], want["fwd_peak"], want["bwd_peak"])
    assert do.check_plan(fwd, got["fwd_offsets"]) == got["fwd_peak"]
    assert do.check_plan(bwd, got["bwd_offsets"]) == got["bwd_peak"]
    assert do.check_plan(want["level2_requests"], got["outer_addr"] + got["fwd_base"] + got["bwd_base"]) == got["peak"]


def test_bilevel_examples_by_inspection():
    fwd, bwd = [(3, 0, 2), (2, 1, 2), (4, 2, 3)], [(6, 0, 1)]
    p = mb.memo_dsa_plan_bilevel(fwd, bwd, [1, 2, 3], [7, 6, 5], [(7, 4, 5)])
    assert (p["fwd_peak"], p["bwd_peak"], p["peak"]) == (5, 6, 7)
    assert p["fwd_base"] == [0, 0, 0] and p["bwd_base"] == [0, 0, 0]
    assert mb.memo_dsa_plan_bilevel(fwd, bwd, [1, 2, 3], [7, 6, 5], [(7, 4, 5), (10, 0, 4)])["peak"] == 15
    assert mb.memo_dsa_plan_bilevel(fwd, bwd, [1, 2, 3], [7, 6, 5], [(7, 4, 5), (10, 0, 8)])["peak"] == 17


def test_planner_rejects_bad_arguments():
    L = mb.lib()
    req = (mb.MemoDsaRequest * 2)()
    req[0].size, req[0].start, req[0].end = 4, 0, 2
    req[1].size, req[1].start, req[1].end = 4, 1, 3
    addr = (ctypes.c_int64 * 2)()
    peak = ctypes.c_int64(0)
    ok = lambda n=2, r=req, al=1, nl=10, a=addr, p=ctypes.byref(peak): L.memo_dsa_plan(n, r, al, nl, a, p, None)
    assert ok() == mb.MEMO_OK and peak.value == 8
    assert ok(n=-1) == mb.MEMO_ERR_INVALID_ARG
    assert ok(r=None) == mb.MEMO_ERR_INVALID_ARG
    assert ok(al=3) == mb.MEMO_ERR_INVALID_ARG
    assert ok(al=0) == mb.MEMO_ERR_INVALID_ARG
    assert ok(nl=-1) == mb.MEMO_ERR_INVALID_ARG
    assert ok(p=None) == mb.MEMO_ERR_INVALID_ARG
    req[1].end = 1
    assert ok() == mb.MEMO_ERR_INVALID_ARG               # empty lifespan
    req[1].end = 3
    req[0].size = -1
    assert ok() == mb.MEMO_ERR_INVALID_ARG


def test_layer_sized_instance_is_planned_quickly():
    """A transformer layer's forward-sized problem (a few dozen transient tensors with nested and
    chained lifespans) is planned within the node budget in well under a second."""
    rng = np.random.default_rng(5)
    req, t = [], 0
    for block in range(8):                               # eight operator groups
        base = t
        for k in range(int(rng.integers(2, 5))):
            req.append((int(rng.integers(1, 33)) << 20, base + k, base + k + int(rng.integers(1, 4))))
        t += 4
    t0 = time.perf_counter()
    peak, addr, proven = mb.memo_dsa_plan(req, align=512, node_limit=500_000)
    assert time.perf_counter() - t0 < 5.0
    rounded = [((s + 511) // 512 * 512, a, b) for s, a, b in req]
    assert do.check_plan(rounded, addr) == peak
    assert peak >= do.load_lower_bound(rounded)


def test_synthetic_transformer_layer_sequence():
    """A stand-in for the profiled request sequence of one layer (sizes in units of one
    b*s*h/TP tensor, 1 GiB at 1M tokens): the two-level plan reaches the load bound where an
    allocator that serves the requests in program order, lowest address first, fragments."""
    U = 1 << 30
    fwd = [(1, 0, 2), (3, 1, 4), (1, 2, 3), (0.0625, 2, 5), (1, 4, 6), (1, 5, 7), (1, 6, 8), (4, 7, 10),
           (4, 8, 10), (0.5, 8, 9), (4, 9, 11), (1, 10, 12), (1, 11, 12)]
    bwd = [(1, 0, 2), (4, 1, 3), (4, 2, 5), (4, 3, 5), (1, 4, 6), (1, 5, 7), (3, 6, 9), (1, 7, 8), (3, 8, 10),
           (1, 9, 11), (0.0625, 9, 10), (1, 10, 11)]
    f = [(int(s * U), a, b) for s, a, b in fwd]
    b_ = [(int(s * U), a, b) for s, a, b in bwd]
    nl = 32
    outer = [(2 * U, 0, 1), (8 * U, nl + 1, nl + 2), (2 * U, 2 * nl + 2, 2 * nl + 3)]
    p = mb.memo_dsa_plan_bilevel(f, b_, list(range(1, nl + 1)), list(range(2 * nl + 1, nl + 1, -1)), outer, align=512)
    assert p["optimal"]
    assert p["fwd_peak"] == do.load_lower_bound(f) == 12 * U
    assert p["bwd_peak"] == do.load_lower_bound(b_) == 9 * U
    assert p["peak"] == 12 * U                     # every layer pass reuses the same 12 GiB
    assert len(set(p["fwd_base"])) == 1 and len(set(p["bwd_base"])) == 1

    def program_order_first_fit(req):
        addr = {}
        for i in sorted(range(len(req)), key=lambda i: req[i][1]):
            busy = sorted((addr[j], addr[j] + req[j][0]) for j in addr
                          if req[j][1] < req[i][2] and req[i][1] < req[j][2])
            x = 0
            for lo, hi in busy:
                if x + req[i][0] <= lo:
                    break
                x = max(x, hi)
            addr[i] = x
        return max(addr[i] + req[i][0] for i in addr)
    assert program_order_first_fit(f) == 13 * U
