"""Pins of the rounding-buffer schedule oracle (Section 4.1 / Figure 5, Section 4.3.4).

The oracle is pinned against things it does not compute itself: a schedule worked out by
hand (tests/golden/schedule_n4.txt), hand-computed packing offsets, the statement of
what a backward pass must find (expected_seen: definition, no schedule involved), every
execution order the waits allow, mutations that drop one wait, and closed forms of the
exposed copy time derived on paper.
"""
import os

import numpy as np
import pytest

from oracle import memo_sched_oracle as so

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "schedule_n4.txt")


def _producer(dev_bytes, seed=7):
    def produce(layer):
        rng = np.random.default_rng(seed * 1000 + layer)
        a = rng.integers(0, 255, dev_bytes, dtype=np.uint8)
        a[a == 0xEE] = 0x11      # keep the poison value out of the payload
        return a
    return produce


def test_hand_schedule_n4():
    want = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        head, waits = line.split(":")
        op, queue, buf = head.split()
        want.append((op[0], int(op[1:]), queue, int(buf),
                     sorted((w[0], int(w[1:])) for w in waits.split())))
    got = [(k, l, q, l % 2, sorted(w)) for k, l, q, w in so.schedule_ops(4)]
    assert got == want


def test_buffer_plan_hand_numbers():
    slots, dev, host = so.buffer_plan(10, [(100, 1.0), (60, 0.5), (7, 0.3)])
    assert [s["dev_offset"] for s in slots] == [0, 1024, 1792]
    assert [s["host_offset"] for s in slots] == [0, 1024, 1536]
    assert [s["k_swapped"] for s in slots] == [10, 5, 3]
    assert [s["bytes_swapped"] for s in slots] == [1000, 300, 21]
    assert (dev, host) == (2048, 1792)


def test_buffer_plan_paper_layer_sizes():
    # Section 4.1: the skeletal tensors of one layer hold 16*b*s*h elements, of which the
    # layer input and the attention output are one b*s*h each.  One GPU's share at tensor
    # parallel degree 8 of the 7B model (h = 4096) at s = 2^20 in 16-bit: 16 tensors of
    # 2^20 x 1 KiB = 16 GiB per layer, 2 + 14*alpha GiB swapped.
    S = 1 << 20
    for alpha in (0.0, 0.25, 1.0):
        tensors = [(1024, 1.0), (1024, 1.0)] + [(1024, alpha)] * 14
        _, dev, host = so.buffer_plan(S, tensors)
        assert dev == 16 << 30
        assert host == int((2 + 14 * alpha) * (1 << 30))
        assert so.host_store_bytes(32, host) == 30 * host


@pytest.mark.parametrize("n_layers", [1, 2, 3, 4, 5, 8])
def test_replay_in_issue_order_matches_definition(n_layers):
    S, tensors = 12, [(40, 1.0), (24, 0.5), (9, 0.0), (16, 0.9)]
    _, dev, _ = so.buffer_plan(S, tensors)
    prod = _producer(dev)
    seen = so.replay_bytes(n_layers, S, tensors, prod)
    want = so.expected_seen(n_layers, S, tensors, prod)
    assert sorted(seen) == list(range(n_layers))
    for layer in range(n_layers):
        assert np.array_equal(seen[layer], want[layer]), layer


@pytest.mark.parametrize("n_layers", [3, 4, 6, 9])
def test_every_allowed_order_gives_the_same_bytes(n_layers):
    S, tensors = 8, [(32, 1.0), (16, 0.5), (8, 0.25)]
    _, dev, _ = so.buffer_plan(S, tensors)
    prod = _producer(dev, seed=n_layers)
    want = so.expected_seen(n_layers, S, tensors, prod)
    ops = so.schedule_ops(n_layers)
    rng = np.random.default_rng(11)
    for order in so.valid_orders(ops, rng, 200):
        seen = so.replay_bytes(n_layers, S, tensors, prod, order=order, ops=ops)
        for layer in range(n_layers):
            assert np.array_equal(seen[layer], want[layer])


@pytest.mark.parametrize("drop", ["F<-O", "O<-F", "I<-B", "B<-I"])
def test_each_stated_wait_is_needed(drop):
    """Dropping any one kind of wait lets some allowed order corrupt a buffer."""
    n_layers, S, tensors = 6, 8, [(32, 1.0), (16, 0.5)]
    _, dev, _ = so.buffer_plan(S, tensors)
    prod = _producer(dev, seed=3)
    want = so.expected_seen(n_layers, S, tensors, prod)
    kind, dep = drop.split("<-")
    ops = [(k, l, q, [w for w in waits if not (k == kind and w[0] == dep)])
           for k, l, q, waits in so.schedule_ops(n_layers)]
    rng = np.random.default_rng(5)
    broken = 0
    for order in so.valid_orders(ops, rng, 300):
        seen = so.replay_bytes(n_layers, S, tensors, prod, order=order, ops=ops)
        broken += any(not np.array_equal(seen[l], want[l]) for l in range(n_layers))
    assert broken > 0


def test_timeline_no_copies_is_plain_sum():
    t = so.timeline(7, 3.0, 5.0, 0.0, 0.0)
    assert t["makespan"] == pytest.approx(7 * 8.0)
    assert t["exposed"] == pytest.approx(0.0)


@pytest.mark.parametrize("n_layers", [3, 4, 5, 12, 32])
def test_timeline_closed_form(n_layers):
    # On paper: a copy longer than the pass it hides behind delays every swapped layer by
    # the difference, forward and backward independently; shorter copies are free.
    rng = np.random.default_rng(n_layers)
    for _ in range(50):
        tf, tb, to, ti = rng.uniform(0.1, 4.0, 4)
        t = so.timeline(n_layers, tf, tb, to, ti)
        want = (n_layers - 2) * (max(0.0, to - tf) + max(0.0, ti - tb))
        assert t["exposed"] == pytest.approx(want, abs=1e-9)
        assert t["compute"] == pytest.approx(n_layers * (tf + tb))


def test_timeline_small_depths_never_swap():
    for n in (1, 2):
        t = so.timeline(n, 1.0, 2.0, 50.0, 50.0)
        assert t["exposed"] == pytest.approx(0.0)


def test_timeline_recompute_counts_as_compute():
    t = so.timeline(6, 1.0, 2.0, 0.5, 0.5, t_recompute=0.25)
    assert t["compute"] == pytest.approx(6 * 3.0 + 4 * 0.25)
    assert t["exposed"] == pytest.approx(0.0)


def test_timeline_respects_every_wait():
    t = so.timeline(9, 1.0, 1.5, 2.3, 0.7)
    for kind, layer, _, waits in so.schedule_ops(9):
        for w in waits:
            assert t["start"][(kind, layer)] >= t["end"][w] - 1e-12
