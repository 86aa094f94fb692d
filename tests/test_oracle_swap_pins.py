"""Pins of the oracle's token-split bookkeeping (Section 4.1) and alpha choice."""
import math
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ALPHAS = [t / 8 for t in range(9)] + [0.9]


def _golden_numbers(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                key, val = line.split()
                out[key] = float(val)
    return out


def test_split_counts_for_the_workloads(oracle):
    # values worked out by hand from floor(alpha*S)
    assert oracle.split_tokens(1024, 0.5) == 512
    assert oracle.split_tokens(32768, 0.75) == 24576
    assert oracle.split_tokens(131072, 1.0) == 131072
    assert oracle.split_tokens(262144, 0.9) == 235929      # 235929.6 rounds down
    assert oracle.split_tokens(1048576, 1.0) == 1048576
    assert oracle.split_tokens(7, 0.0) == 0
    assert oracle.split_tokens(0, 0.5) == 0


@pytest.mark.parametrize("bad", [-0.01, 1.0000001, float("nan"), float("inf"), -float("inf")])
def test_split_rejects_bad_alpha(oracle, bad):
    assert oracle.split_tokens(100, bad) == -1
    assert oracle.swap_plan(100, 8, bad) is None


def test_split_rejects_bad_sizes(oracle):
    assert oracle.split_tokens(-1, 0.5) == -1
    assert oracle.swap_plan(10, 0, 0.5) is None
    assert oracle.swap_plan(10, -4, 0.5) is None


@pytest.mark.parametrize("alpha", ALPHAS)
@pytest.mark.parametrize("S,row_bytes", [(1024, 1024), (1000, 24), (1, 8), (262144, 10240)])
def test_plan_partitions_the_tokens(oracle, alpha, S, row_bytes):
    p = oracle.swap_plan(S, row_bytes, alpha)
    assert p["k_swapped"] + p["n_recompute"] == S
    assert p["bytes_swapped"] + p["bytes_dropped"] == S * row_bytes
    assert p["recompute_byte_offset"] == p["bytes_swapped"] == p["k_swapped"] * row_bytes
    assert 0 <= p["k_swapped"] <= S
    assert p["k_swapped"] <= alpha * S < p["k_swapped"] + 1 or alpha == 1.0
    if alpha == 0.0:
        assert p["bytes_swapped"] == 0
    if alpha == 1.0:
        assert p["n_recompute"] == 0


def test_paper_skeletal_byte_count(oracle):
    # Section 3.2: 16*b*s*h elements per layer -> 4096 GB for 7B at 1M tokens in half precision;
    # Section 4.1: the attention output is 6.25 % of it.  Offloading everything (alpha = 1) of a
    # [s, 16*h] half-precision tensor per layer must reproduce the printed total.
    g = _golden_numbers("skeletal_bytes_7b_1m.txt")
    row_bytes = int(g["skeletal_elems_per_token_over_h"] * g["h"] * g["bytes_per_elem"])
    p = oracle.swap_plan(int(g["s"]), row_bytes, 1.0)
    assert p["bytes_swapped"] * int(g["layers"]) == int(g["total_GiB"]) * 2 ** 30
    attn_row_bytes = int(g["h"] * g["bytes_per_elem"])
    pa = oracle.swap_plan(int(g["s"]), attn_row_bytes, 1.0)
    assert pa["bytes_swapped"] / p["bytes_swapped"] == g["attn_output_fraction"]


@pytest.mark.parametrize("alpha", ALPHAS)
def test_round_trip_is_byte_identical_and_leaves_dropped_rows_alone(oracle, alpha):
    S, row_bytes = 203, 40
    rng = np.random.default_rng(5)
    act = rng.integers(0, 256, size=S * row_bytes, dtype=np.uint8)
    host = np.full(S * row_bytes + 16, 0xEE, dtype=np.uint8)
    k = oracle.split_tokens(S, alpha)
    n = oracle.swap_out(act, row_bytes, alpha, host)
    assert n == k * row_bytes
    assert np.array_equal(host[:n], act[:n])
    assert (host[n:] == 0xEE).all()                 # nothing written past the swapped bytes
    restored = np.full_like(act, 0x5A)              # poison: dropped rows must stay poisoned
    m = oracle.swap_in(restored, row_bytes, alpha, host)
    assert m == n
    assert np.array_equal(restored[:n], act[:n])
    assert (restored[n:] == 0x5A).all()


def test_host_capacity_error(oracle):
    S, row_bytes = 64, 16
    act = np.zeros(S * row_bytes, dtype=np.uint8)
    host = np.zeros(S * row_bytes // 2 - 1, dtype=np.uint8)
    assert oracle.swap_out(act, row_bytes, 0.5, host) == -2
    assert oracle.swap_in(act, row_bytes, 0.5, host) == -2
    host = np.zeros(S * row_bytes // 2, dtype=np.uint8)
    assert oracle.swap_out(act, row_bytes, 0.5, host) == S * row_bytes // 2


# ------------------------------------------------------------------ alpha (Section 4.1)
def test_alpha_grid_cases_worked_by_hand(oracle):
    # (S_in + S_attn + a*S_oth)/B <= T  and (n-2)(...) <= M
    # 1) both slack at a = 1
    assert oracle.alpha_grid(1, 1, 14, bandwidth=32, t_layer=1.0, n_layers=32, m_cpu=1e9, steps=8) == 1.0
    # 2) time binds: 2 + 14a <= 9  -> a <= 0.5
    assert oracle.alpha_grid(1, 1, 14, bandwidth=1, t_layer=9.0, n_layers=32, m_cpu=1e9, steps=8) == 0.5
    # 3) host memory binds: 30 (2 + 14a) <= 165 -> a <= 0.25
    assert oracle.alpha_grid(1, 1, 14, bandwidth=1e9, t_layer=1.0, n_layers=32, m_cpu=165, steps=8) == 0.25
    # 4) infeasible even at a = 0
    assert oracle.alpha_grid(1, 1, 14, bandwidth=1, t_layer=1.0, n_layers=32, m_cpu=1e9, steps=8) == -1.0
    # 5) two layers: the (n-2) factor removes the memory constraint
    assert oracle.alpha_grid(1, 1, 14, bandwidth=1e9, t_layer=1.0, n_layers=2, m_cpu=0.0, steps=8) == 1.0
