"""CPU-only checks of the C-ABI library: it loads, exports what include/memo.h declares,
rejects bad arguments before touching a GPU, and its host-side bookkeeping (token split,
swap plan, alpha) is bit-identical to the oracle's."""
import ctypes
import os
import re

import pytest

from paper_2407_12117_amd import binding as mb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ALPHAS = [t / 8 for t in range(9)] + [0.9, 0.3, 1e-9, 0.999999]


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "memo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(memo_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = mb.lib()
    names = _declared_symbols()
    assert set(names) == set(mb.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_status_strings():
    for s in range(6):
        assert len(mb.status_str(s)) > 0


@pytest.mark.parametrize("S", [0, 1, 7, 1000, 1024, 32768, 262144, 1048576])
@pytest.mark.parametrize("alpha", ALPHAS)
def test_split_matches_oracle(oracle, S, alpha):
    assert mb.memo_split_tokens(S, alpha) == oracle.split_tokens(S, alpha)


@pytest.mark.parametrize("bad", [-0.01, 1.0000001, float("nan"), float("inf"), -float("inf")])
def test_split_rejects_bad_alpha(bad):
    assert mb.memo_split_tokens(100, bad) == -1
    with pytest.raises(mb.MemoError) as e:
        mb.memo_swap_plan_make(100, 8, bad)
    assert e.value.status == mb.MEMO_ERR_INVALID_ARG


@pytest.mark.parametrize("S,row_bytes", [(1024, 1024), (32768, 8192), (131072, 8192),
                                         (262144, 10240), (1048576, 8192), (1000, 24)])
@pytest.mark.parametrize("alpha", ALPHAS)
def test_plan_matches_oracle(oracle, S, row_bytes, alpha):
    got = mb.memo_swap_plan_make(S, row_bytes, alpha)
    want = oracle.swap_plan(S, row_bytes, alpha)
    for key, val in want.items():
        assert got[key] == val, key
    assert got["S"] == S and got["row_bytes"] == row_bytes


def test_plan_rejects_bad_sizes():
    for S, rb in ((10, 0), (10, -8), (-1, 8)):
        with pytest.raises(mb.MemoError):
            mb.memo_swap_plan_make(S, rb, 0.5)


def _desc(**kw):
    base = dict(B=1, H=1, d=128, S=256, dtype=mb.MEMO_BF16, scale=0.1, stride_b=256 * 128,
                stride_s=128, stride_h=128, causal=1, flags=0)
    base.update(kw)
    return mb.MemoAttnDesc(**base)


@pytest.mark.parametrize("kw,status", [
    (dict(S=0), mb.MEMO_ERR_INVALID_ARG),
    (dict(B=0), mb.MEMO_ERR_INVALID_ARG),
    (dict(scale=float("nan")), mb.MEMO_ERR_INVALID_ARG),
    (dict(scale=-1.0), mb.MEMO_ERR_INVALID_ARG),
    (dict(causal=0), mb.MEMO_ERR_UNSUPPORTED),
    (dict(flags=2), mb.MEMO_ERR_UNSUPPORTED),           # only bit 0 (deterministic dQ) is defined
    (dict(d=64), mb.MEMO_ERR_UNSUPPORTED),            # bf16 path is built for d = 128
    (dict(d=96, dtype=mb.MEMO_F32), mb.MEMO_ERR_UNSUPPORTED),
    (dict(dtype=7), mb.MEMO_ERR_UNSUPPORTED),
    (dict(stride_s=132), mb.MEMO_ERR_UNSUPPORTED),    # rows not 16-byte aligned
    (dict(stride_s=64), mb.MEMO_ERR_INVALID_ARG),     # rows overlap
    (dict(stride_s=(1 << 24) + 8, stride_b=1 << 40), mb.MEMO_ERR_UNSUPPORTED),   # 64 rows span over 4 GiB
    # one workgroup per pair of 256-row tiles: 2^21 pairs x 1024 heads does not fit a grid
    (dict(S=1 << 30, H=1024, stride_s=1024 * 128, stride_b=1 << 50), mb.MEMO_ERR_UNSUPPORTED),
])
def test_attention_rejects_bad_descriptors_before_any_launch(kw, status):
    d = _desc(**kw)
    fake = ctypes.c_void_p(4096)
    assert mb.lib().memo_attn_fwd(ctypes.byref(d), fake, fake, fake, fake, fake, None) == status
    assert mb.lib().memo_attn_bwd_workspace_bytes(ctypes.byref(d)) == 0


def test_deterministic_flag_is_accepted():
    # bit 0 asks for bit-reproducible dQ; the backward has no atomics, so the bit is accepted as a no-op
    assert mb.lib().memo_attn_bwd_workspace_bytes(ctypes.byref(_desc(flags=1))) == \
        mb.lib().memo_attn_bwd_workspace_bytes(ctypes.byref(_desc(flags=0))) > 0


def test_attention_rejects_null_and_misaligned_pointers():
    d = _desc()
    ok = ctypes.c_void_p(4096)
    L = mb.lib()
    assert L.memo_attn_fwd(ctypes.byref(d), None, ok, ok, ok, ok, None) == mb.MEMO_ERR_INVALID_ARG
    assert L.memo_attn_fwd(None, ok, ok, ok, ok, ok, None) == mb.MEMO_ERR_INVALID_ARG
    assert L.memo_attn_fwd(ctypes.byref(d), ctypes.c_void_p(4100), ok, ok, ok, ok, None) == mb.MEMO_ERR_UNSUPPORTED
    need = L.memo_attn_bwd_workspace_bytes(ctypes.byref(d))
    assert need >= 256 * 4 and need % 256 == 0
    args = [ok] * 9
    assert L.memo_attn_bwd(ctypes.byref(d), *args, None, 0, None) == mb.MEMO_ERR_WORKSPACE
    assert L.memo_attn_bwd(ctypes.byref(d), *args, ok, need - 1, None) == mb.MEMO_ERR_WORKSPACE
    assert L.memo_attn_bwd(ctypes.byref(d), *args, ctypes.c_void_p(4100), need, None) == mb.MEMO_ERR_WORKSPACE


def test_swap_rejects_before_any_copy():
    L = mb.lib()
    ok = ctypes.c_void_p(4096)
    # host store one byte too small: the paper's host out-of-memory case
    assert L.memo_swap_out(ok, 64, 16, 0.5, ok, 64 * 16 // 2 - 1, None, None, None) == mb.MEMO_ERR_HOST_CAPACITY
    assert L.memo_swap_in(ok, 64, 16, 0.5, ok, 64 * 16 // 2 - 1, None, None, None) == mb.MEMO_ERR_HOST_CAPACITY
    assert L.memo_swap_out(None, 64, 16, 0.5, ok, 4096, None, None, None) == mb.MEMO_ERR_INVALID_ARG
    assert L.memo_swap_out(ok, 64, 16, 0.5, None, 4096, None, None, None) == mb.MEMO_ERR_INVALID_ARG
    assert L.memo_swap_out(ok, 64, 16, 1.5, ok, 4096, None, None, None) == mb.MEMO_ERR_INVALID_ARG
    assert L.memo_swap_out(ok, 64, 0, 0.5, ok, 4096, None, None, None) == mb.MEMO_ERR_INVALID_ARG


# ------------------------------------------------------------- alpha (Section 4.1)
@pytest.mark.parametrize("case", [
    dict(s_in=1, s_attn=1, s_oth=14, bandwidth=32, t_layer=1.0, n_layers=32, m_cpu=1e9),
    dict(s_in=1, s_attn=1, s_oth=14, bandwidth=1, t_layer=9.0, n_layers=32, m_cpu=1e9),
    dict(s_in=1, s_attn=1, s_oth=14, bandwidth=1e9, t_layer=1.0, n_layers=32, m_cpu=165),
    dict(s_in=8.0, s_attn=8.0, s_oth=112.0, bandwidth=57.0, t_layer=1.3, n_layers=32, m_cpu=2048.0),
    dict(s_in=1, s_attn=1, s_oth=14, bandwidth=1e9, t_layer=1.0, n_layers=2, m_cpu=0.0),
])
def test_alpha_closed_form_brackets_the_oracle_grid(oracle, case):
    steps = 4096
    got = mb.memo_solve_alpha(**case)
    grid = oracle.alpha_grid(steps=steps, **case)
    assert 0.0 <= got <= 1.0
    # the grid scan returns the largest feasible grid point: the exact optimum lies in
    # [grid, grid + 1/steps)
    assert grid <= got + 1e-12 and got < grid + 1.0 / steps + 1e-12


def test_alpha_infeasible_cases(oracle):
    with pytest.raises(mb.MemoError) as e:
        mb.memo_solve_alpha(1, 1, 14, 1, 1.0, 32, 1e9)      # copy of the whole tensors too slow
    assert e.value.status == mb.MEMO_ERR_UNSUPPORTED
    assert oracle.alpha_grid(1, 1, 14, 1, 1.0, 32, 1e9, 8) == -1.0
    with pytest.raises(mb.MemoError) as e:
        mb.memo_solve_alpha(1, 1, 14, 1e9, 1.0, 32, 10.0)   # host memory too small
    assert e.value.status == mb.MEMO_ERR_HOST_CAPACITY
    assert oracle.alpha_grid(1, 1, 14, 1e9, 1.0, 32, 10.0, 8) == -1.0
    with pytest.raises(mb.MemoError):
        mb.memo_solve_alpha(1, 1, 0, 1, 1.0, 32, 10.0)


# ------------------------------------------- rounding buffers (Section 4.1, Figure 5)
@pytest.mark.parametrize("seed", range(6))
def test_buffer_plan_matches_oracle(seed):
    import numpy as np
    from oracle import memo_sched_oracle as so
    rng = np.random.default_rng(seed)
    S = int(rng.integers(1, 5000))
    tensors = [(int(rng.integers(1, 3000)), float(rng.choice(ALPHAS))) for _ in range(int(rng.integers(1, 20)))]
    slots, dev, host = mb.memo_buffer_plan_make(S, tensors)
    oslots, odev, ohost = so.buffer_plan(S, tensors)
    assert (dev, host) == (odev, ohost)
    assert slots == oslots


def test_buffer_plan_full_size_layer():
    # one GPU's share of a 7B layer at S = 2^20 (16 tensors of S x 1 KiB)
    from oracle import memo_sched_oracle as so
    tensors = [(1024, 1.0), (1024, 1.0)] + [(1024, 0.375)] * 14
    slots, dev, host = mb.memo_buffer_plan_make(1 << 20, tensors)
    assert (slots, dev, host) == so.buffer_plan(1 << 20, tensors)
    assert dev == 16 << 30


def test_buffer_plan_and_sched_reject_bad_arguments():
    L = mb.lib()
    ok = ctypes.c_void_p(4096)
    descs = (mb.MemoTensorDesc * 2)()
    descs[0].row_bytes, descs[0].alpha = 64, 1.0
    descs[1].row_bytes, descs[1].alpha = 32, 0.5
    slots = (mb.MemoTensorSlot * 2)()
    dev, host = ctypes.c_size_t(0), ctypes.c_size_t(0)
    args = (slots, ctypes.byref(dev), ctypes.byref(host))
    assert L.memo_buffer_plan_make(16, 2, descs, *args) == mb.MEMO_OK
    assert L.memo_buffer_plan_make(0, 2, descs, *args) == mb.MEMO_ERR_INVALID_ARG
    assert L.memo_buffer_plan_make(16, 0, descs, *args) == mb.MEMO_ERR_INVALID_ARG
    assert L.memo_buffer_plan_make(16, 2, None, *args) == mb.MEMO_ERR_INVALID_ARG
    descs[1].alpha = 1.25
    assert L.memo_buffer_plan_make(16, 2, descs, *args) == mb.MEMO_ERR_INVALID_ARG
    descs[1].alpha = 0.5
    descs[0].row_bytes = 0
    assert L.memo_buffer_plan_make(16, 2, descs, *args) == mb.MEMO_ERR_INVALID_ARG
    descs[0].row_bytes = 64

    h = ctypes.c_void_p(None)
    create = lambda n, cap, b0=ok, b1=ok, hs=ok: L.memo_sched_create(
        ctypes.byref(h), n, 16, 2, descs, b0, b1, hs, cap, None, None, None)
    per_layer = host.value
    # five layers hold three slots on the host: one byte short is the host out-of-memory case
    assert create(5, 3 * per_layer - 1) == mb.MEMO_ERR_HOST_CAPACITY and not h.value
    assert create(0, 1 << 20) == mb.MEMO_ERR_INVALID_ARG
    assert create(5, 1 << 20, b0=None) == mb.MEMO_ERR_INVALID_ARG
    assert create(5, 1 << 20, hs=None) == mb.MEMO_ERR_INVALID_ARG
    assert L.memo_sched_forward_begin(None, 0) == mb.MEMO_ERR_INVALID_ARG
    assert L.memo_sched_backward_end(None, 0) == mb.MEMO_ERR_INVALID_ARG
    assert L.memo_sched_buffer(None, 0) is None
    assert L.memo_sched_destroy(None) == mb.MEMO_OK


# ------------------------------------------- token-wise recomputation (Section 4.1)
def test_recompute_entry_points_reject_bad_arguments():
    L = mb.lib()
    ok = ctypes.c_void_p(4096)
    odd = ctypes.c_void_p(4100)
    ln = lambda x=ok, g=ok, b=ok, y=ok, S=64, h=4096, eps=1e-5, r0=0, r1=64: \
        L.memo_layernorm_rows(x, g, b, y, S, h, eps, r0, r1, None)
    assert ln(x=None) == mb.MEMO_ERR_INVALID_ARG
    assert ln(r0=-1) == mb.MEMO_ERR_INVALID_ARG
    assert ln(r0=10, r1=9) == mb.MEMO_ERR_INVALID_ARG
    assert ln(r1=65) == mb.MEMO_ERR_INVALID_ARG
    assert ln(eps=-1.0) == mb.MEMO_ERR_INVALID_ARG
    assert ln(eps=float("nan")) == mb.MEMO_ERR_INVALID_ARG
    assert ln(h=4000) == mb.MEMO_ERR_UNSUPPORTED
    assert ln(h=16384) == mb.MEMO_ERR_UNSUPPORTED
    assert ln(y=odd) == mb.MEMO_ERR_UNSUPPORTED
    assert ln(r0=7, r1=7) == mb.MEMO_OK                      # empty range: nothing queued
    lin = lambda a=ok, w=ok, bias=None, out=ok, S=64, K=4096, N=1536, r0=0, r1=64: \
        L.memo_linear_rows(a, w, bias, out, S, K, N, r0, r1, None)
    assert lin(w=None) == mb.MEMO_ERR_INVALID_ARG
    assert lin(r1=100) == mb.MEMO_ERR_INVALID_ARG
    assert lin(K=100) == mb.MEMO_ERR_UNSUPPORTED
    assert lin(N=1500) == mb.MEMO_ERR_UNSUPPORTED
    assert lin(bias=odd) == mb.MEMO_ERR_UNSUPPORTED
    assert lin(r0=64, r1=64) == mb.MEMO_OK
