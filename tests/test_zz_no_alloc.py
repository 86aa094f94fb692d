"""The backward entry point that allocates nothing (memo_attn_bwd_static) against memo_attn_bwd:
same kernels, the D_i buffer in the library's static device array instead of a caller workspace.
Two calls in a row on the same GPU, the second on a smaller problem, must both reproduce the
workspace entry point bit for bit (the array keeps the first call's contents)."""
import ctypes

import pytest
import torch

from paper_2407_12117_amd import binding as mb
from paper_2407_12117_amd import synth

gpu = pytest.mark.gpu


def test_static_backward_refuses_on_the_host_before_touching_a_device():
    """No GPU needed: a problem beyond the array, a bad descriptor and a null pointer are all
    refused before the first HIP call."""
    L = mb.lib()
    ok = ctypes.c_void_p(4096)
    mk = lambda **kw: mb.MemoAttnDesc(**{**dict(B=1, H=1, d=128, S=256, dtype=mb.MEMO_BF16, scale=0.1,
                                                  stride_b=1 << 40, stride_s=128, stride_h=128, causal=1,
                                                  flags=0), **kw})
    args = [ok] * 9
    big = mk(S=(4 << 20) + 1)
    assert L.memo_attn_bwd_static(ctypes.byref(big), *args, None) == mb.MEMO_ERR_WORKSPACE
    assert L.memo_attn_bwd_static(ctypes.byref(mk(S=1 << 20, H=5, stride_s=640)), *args, None) == mb.MEMO_ERR_WORKSPACE
    assert L.memo_attn_bwd_static(ctypes.byref(mk(S=0)), *args, None) == mb.MEMO_ERR_INVALID_ARG
    assert L.memo_attn_bwd_static(ctypes.byref(mk(causal=0)), *args, None) == mb.MEMO_ERR_UNSUPPORTED
    assert L.memo_attn_bwd_static(None, *args, None) == mb.MEMO_ERR_INVALID_ARG
    assert L.memo_attn_bwd_static(ctypes.byref(mk()), None, *args[1:], None) == mb.MEMO_ERR_INVALID_ARG


def _both(B, S, H, d, dtype, seed):
    print(f"[case] static backward B={B} S={S} H={H} d={d} {dtype} seed={seed}", flush=True)
    scale = synth.default_scale(d)
    q, k, v, g = (t.cuda() for t in synth.attn_inputs(B, S, H, d, dtype, seed))
    o, lse = mb.memo_attn_fwd(q, k, v, scale)
    want = mb.memo_attn_bwd(q, k, v, o, lse, g, scale)
    got = tuple(torch.full_like(q, float("nan")) for _ in range(3))
    torch.cuda.synchronize()
    # cumulative number of allocations torch's caching allocator has served: unlike the bytes in
    # use, it cannot fall when the collector frees an unrelated tensor meanwhile
    count = lambda: torch.cuda.memory_stats()["allocation.all.allocated"]
    before = count()
    mb.memo_attn_bwd_static(q, k, v, o, lse, g, scale, *got)
    torch.cuda.synchronize()
    assert count() == before, "memo_attn_bwd_static made torch allocate device memory"
    for name, a, b in zip(("dQ", "dK", "dV"), got, want):
        assert torch.equal(a, b), f"{name} differs from memo_attn_bwd"


@gpu
def test_static_backward_two_calls_second_smaller():
    _both(1, 3000, 2, 128, "bf16", 501)
    _both(2, 700, 1, 128, "bf16", 502)      # smaller: the array still holds the first call's D_i


@gpu
def test_static_backward_fp32_then_ragged_bf16():
    _both(1, 1024, 1, 64, "f32", 503)
    _both(1, 333, 3, 128, "bf16", 504)


@gpu
def test_static_backward_rejects_more_rows_than_the_array_holds():
    S = (4 << 20) + 128
    q = torch.empty((1, S, 1, 128), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((1, 1, S), dtype=torch.float32, device="cuda")
    with pytest.raises(mb.MemoError) as err:
        mb.memo_attn_bwd_static(q, q, q, q, lse, q, 0.1, q, q, q)
    assert err.value.status == mb.MEMO_ERR_WORKSPACE
