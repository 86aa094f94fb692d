"""Pins of the CPU oracle against things other than itself (no GPU needed).

Each test names the mistake it is there to catch.  The oracle states Section 2.1.3's
attention definition and its derivative; Section 4.1's token split.
"""
import math
import os

import numpy as np
import pytest
import torch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _parse_golden(name):
    vals = {}
    env = {"ln3": math.log(3.0), "ln4": math.log(4.0)}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            vals[parts[0]] = [eval(p, {"__builtins__": {}}, env) for p in parts[1:]]
    return vals


# ---------------------------------------------------------------- hand example
def test_hand_example(oracle):
    g = _parse_golden("hand_example_s2.txt")
    t = lambda n: np.array(g[n], dtype=np.float64).reshape(1, 2, 1, 1)
    o, lse = oracle.attn_fwd(t("q"), t("k"), t("v"), 1.0)
    dq, dk, dv = oracle.attn_bwd(t("q"), t("k"), t("v"), t("dO"), 1.0)
    np.testing.assert_allclose(o.ravel(), g["O"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(lse.ravel(), g["LSE"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(dq.ravel(), g["dQ"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(dk.ravel(), g["dK"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(dv.ravel(), g["dV"], rtol=0, atol=1e-14)


# ------------------------------------------- brute force with an explicit SxS matrix
def _brute_forward(q, k, v, scale):
    """Independent statement: build the full SxS score matrix per head, mask the
    strict upper triangle, normalise each row, multiply by V."""
    B, S, H, d = q.shape
    o = np.zeros_like(q)
    lse = np.zeros((B, H, S))
    for b in range(B):
        for h in range(H):
            Sm = np.zeros((S, S))
            for i in range(S):
                for j in range(S):
                    Sm[i, j] = scale * sum(q[b, i, h, c] * k[b, j, h, c] for c in range(d))
            for i in range(S):
                w = [math.exp(Sm[i, j]) for j in range(i + 1)]
                tot = sum(w)
                lse[b, h, i] = math.log(tot)
                for c in range(d):
                    o[b, i, h, c] = sum(w[j] * v[b, j, h, c] for j in range(i + 1)) / tot
    return o, lse


def test_forward_vs_bruteforce(oracle):
    # catches: wrong mask bound, wrong head/batch stride, scale misplaced
    q, k, v = (_rand((2, 9, 3, 4), s) for s in (1, 2, 3))
    o, lse = oracle.attn_fwd(q, k, v, 0.37)
    ob, lb = _brute_forward(q, k, v, 0.37)
    np.testing.assert_allclose(o, ob, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, lb, rtol=1e-12, atol=1e-13)


# --------------------------------------------- library routine: torch fp64 + autograd
def _torch_reference(q, k, v, d_o, scale):
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    # [B,S,H,d] -> [B,H,S,d]
    o = torch.nn.functional.scaled_dot_product_attention(
        tq.transpose(1, 2), tk.transpose(1, 2), tv.transpose(1, 2), is_causal=True, scale=scale)
    o = o.transpose(1, 2)
    (o * torch.tensor(d_o)).sum().backward()
    return o.detach().numpy(), tq.grad.numpy(), tk.grad.numpy(), tv.grad.numpy()


@pytest.mark.parametrize("shape", [(2, 40, 3, 8), (1, 130, 2, 16)])
def test_fwd_bwd_vs_torch_autograd(oracle, shape):
    # catches: transposed operands, dropped term in dS, wrong sign, missing scale in dQ/dK
    q, k, v, d_o = (_rand(shape, s) for s in (11, 12, 13, 14))
    scale = 1.0 / math.sqrt(shape[3]) * 1.3
    o, _ = oracle.attn_fwd(q, k, v, scale)
    dq, dk, dv = oracle.attn_bwd(q, k, v, d_o, scale)
    ro, rdq, rdk, rdv = _torch_reference(q, k, v, d_o, scale)
    for a, b in ((o, ro), (dq, rdq), (dk, rdk), (dv, rdv)):
        np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-12)


# --------------------------------------------------------------- finite differences
def test_gradients_vs_finite_differences(oracle):
    shape = (1, 12, 2, 3)
    q, k, v, d_o = (_rand(shape, s) for s in (21, 22, 23, 24))
    scale = 0.61
    dq, dk, dv = oracle.attn_bwd(q, k, v, d_o, scale)

    def loss(q_, k_, v_):
        o, _ = oracle.attn_fwd(q_, k_, v_, scale)
        return float((o * d_o).sum())

    eps = 1e-6
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps
            xm[idx] -= eps
            args_p = {"q": (xp, k, v), "k": (q, xp, v), "v": (q, k, xp)}[name]
            args_m = {"q": (xm, k, v), "k": (q, xm, v), "v": (q, k, xm)}[name]
            num[idx] = (loss(*args_p) - loss(*args_m)) / (2 * eps)
        err = np.linalg.norm(num - g) / np.linalg.norm(g)
        assert err < 1e-6, (name, err)


# ------------------------------------------------------------ invariants, closed forms
def test_rows_of_softmax_sum_to_one(oracle):
    q, k = _rand((1, 65, 2, 8), 31), _rand((1, 65, 2, 8), 32)
    v = np.ones((1, 65, 2, 8))
    o, _ = oracle.attn_fwd(q, k, v, 0.5)
    np.testing.assert_allclose(o, 1.0, rtol=0, atol=1e-14)


def test_zero_queries_closed_form(oracle):
    # Q = 0 -> uniform weights 1/(i+1): O_i = prefix mean of V, LSE_i = ln(i+1),
    # dK = 0, dV_j = sum_{i>=j} dO_i/(i+1)
    S, d = 77, 5
    k, v, d_o = (_rand((1, S, 1, d), s) for s in (41, 42, 43))
    q = np.zeros_like(k)
    o, lse = oracle.attn_fwd(q, k, v, 0.7)
    n = np.arange(1, S + 1, dtype=np.float64)
    np.testing.assert_allclose(o[0, :, 0, :], np.cumsum(v[0, :, 0, :], axis=0) / n[:, None],
                               rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse[0, 0], np.log(n), rtol=1e-13, atol=1e-13)
    dq, dk, dv = oracle.attn_bwd(q, k, v, d_o, 0.7)
    np.testing.assert_allclose(dk, 0.0, atol=1e-14)
    w = d_o[0, :, 0, :] / n[:, None]
    suffix = np.cumsum(w[::-1], axis=0)[::-1]
    np.testing.assert_allclose(dv[0, :, 0, :], suffix, rtol=1e-12, atol=1e-13)
    # dQ_i = scale/(i+1) [ (sum_{j<=i} k_j v_j^T) dO_i - D_i sum_{j<=i} k_j ]
    K, V, G = k[0, :, 0, :], v[0, :, 0, :], d_o[0, :, 0, :]
    kv = np.cumsum(K[:, :, None] * V[:, None, :], axis=0)
    ksum = np.cumsum(K, axis=0)
    D = (G * o[0, :, 0, :]).sum(axis=1)
    expect = 0.7 / n[:, None] * (np.einsum("icd,id->ic", kv, G) - D[:, None] * ksum)
    np.testing.assert_allclose(dq[0, :, 0, :], expect, rtol=1e-11, atol=1e-13)


def test_zero_keys_closed_form(oracle):
    # K = 0 -> same uniform weights, dQ = 0,
    # dK_j = scale [ (sum_{i>=j} q_i dO_i^T/(i+1)) v_j - sum_{i>=j} D_i q_i/(i+1) ]
    S, d = 53, 4
    q, v, d_o = (_rand((1, S, 1, d), s) for s in (51, 52, 53))
    k = np.zeros_like(q)
    o, _ = oracle.attn_fwd(q, k, v, 0.9)
    dq, dk, _ = oracle.attn_bwd(q, k, v, d_o, 0.9)
    np.testing.assert_allclose(dq, 0.0, atol=1e-14)
    n = np.arange(1, S + 1, dtype=np.float64)
    Q, V, G, O = q[0, :, 0, :], v[0, :, 0, :], d_o[0, :, 0, :], o[0, :, 0, :]
    D = (G * O).sum(axis=1)
    qg = (Q[:, :, None] * G[:, None, :]) / n[:, None, None]
    qg_suffix = np.cumsum(qg[::-1], axis=0)[::-1]
    dq_suffix = np.cumsum(((D / n)[:, None] * Q)[::-1], axis=0)[::-1]
    expect = 0.9 * (np.einsum("jcd,jd->jc", qg_suffix, V) - dq_suffix)
    np.testing.assert_allclose(dk[0, :, 0, :], expect, rtol=1e-11, atol=1e-13)


def test_gradient_invariants(oracle):
    # sum_j dV_j = sum_i dO_i (rows of P sum to 1); sum q.dQ = sum k.dK per head
    # (the scores are invariant under q -> c q, k -> k / c)
    shape = (2, 64, 3, 8)
    q, k, v, d_o = (_rand(shape, s) for s in (61, 62, 63, 64))
    dq, dk, dv = oracle.attn_bwd(q, k, v, d_o, 0.35)
    np.testing.assert_allclose(dv.sum(axis=1), d_o.sum(axis=1), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose((q * dq).sum(axis=(1, 3)), (k * dk).sum(axis=(1, 3)),
                               rtol=1e-10, atol=1e-12)


def test_causality_bitwise(oracle):
    # changing keys/values after position i must leave O_i, LSE_i bit-identical
    shape = (1, 50, 2, 6)
    q, k, v = (_rand(shape, s) for s in (71, 72, 73))
    o1, l1 = oracle.attn_fwd(q, k, v, 0.4)
    k2, v2 = k.copy(), v.copy()
    k2[:, 30:] += 5.0
    v2[:, 30:] -= 3.0
    o2, l2 = oracle.attn_fwd(q, k2, v2, 0.4)
    assert np.array_equal(o1[:, :30], o2[:, :30])
    assert np.array_equal(l1[:, :, :30], l2[:, :, :30])
    assert not np.array_equal(o1[:, 30:], o2[:, 30:])


def test_large_scores_do_not_overflow(oracle):
    # the row maximum is subtracted before exponentiation
    q = np.full((1, 4, 1, 2), 40.0)
    k = np.full((1, 4, 1, 2), 40.0)
    v = _rand((1, 4, 1, 2), 81)
    o, lse = oracle.attn_fwd(q, k, v, 1.0)
    assert np.isfinite(o).all() and np.isfinite(lse).all()
    np.testing.assert_allclose(lse[0, 0], 3200.0 + np.log(np.arange(1, 5)), rtol=1e-14)


# ---------------------------------------------------- sampled entry points = dense ones
def test_sampled_rows_and_tail_columns_match_dense(oracle):
    B, S, H, d = 2, 96, 3, 8
    q, k, v, d_o = (_rand((B, S, H, d), s) for s in (91, 92, 93, 94))
    scale = 0.3
    o, lse = oracle.attn_fwd(q, k, v, scale)
    dq, dk, dv = oracle.attn_bwd(q, k, v, d_o, scale)
    rows = np.array([0, 1, 31, 32, 95], dtype=np.int64)
    b, h = 1, 2
    qs, ks, vs, gs = (x[b, :, h, :] for x in (q, k, v, d_o))
    o_r, lse_r, delta_r, dq_r = oracle.head_rows(qs, ks, vs, gs, rows, scale)
    assert np.array_equal(o_r, o[b, rows, h, :])
    assert np.array_equal(lse_r, lse[b, h, rows])
    assert np.array_equal(dq_r, dq[b, rows, h, :])
    np.testing.assert_allclose(delta_r, (gs[rows] * o_r).sum(axis=1), rtol=1e-13)
    j0 = 70
    dk_t, dv_t = oracle.head_dkdv_tail(qs, ks, vs, gs, j0, scale)
    assert np.array_equal(dk_t, dk[b, j0:, h, :])
    assert np.array_equal(dv_t, dv[b, j0:, h, :])
    o_only, lse_only, none1, none2 = oracle.head_rows(qs, ks, vs, None, rows, scale)
    assert np.array_equal(o_only, o_r) and np.array_equal(lse_only, lse_r)
    assert none1 is None and none2 is None
