"""GPU parity of the token-wise recomputation (Section 4.1): LayerNorm and the projection that
rebuild "input_norm" and "q, k, v" from the stored layer input.

* each kernel against the fp64 oracle on identical (once-rounded) bf16 inputs;
* a row recomputed in any range is bit-identical to the same row of a pass over all rows, and
  rows outside the range are not touched;
* swap-out of the first k rows + recomputation of rows [k,S) rebuilds the tensors bit for bit;
* full-size cases (S = 2^18 and S = 2^20, h = 4096 -> 1536) on sampled rows.
"""
import numpy as np
import pytest
import torch

from oracle import memo_recompute_oracle as ro
from paper_2407_12117_amd import binding as mb

import gpu_util as gu

pytestmark = pytest.mark.gpu

EPS = 1e-5


def _params(h, N, K, seed):
    g = torch.Generator().manual_seed(seed)
    gamma = (1.0 + 0.1 * torch.randn(h, generator=g)).to(torch.bfloat16)
    beta = (0.1 * torch.randn(h, generator=g)).to(torch.bfloat16)
    w = (torch.randn((N, K), generator=g) / K ** 0.5).to(torch.bfloat16)
    bias = (0.1 * torch.randn(N, generator=g)).to(torch.bfloat16)
    return gamma, beta, w, bias


@pytest.mark.parametrize("S,h", [(1, 512), (37, 512), (300, 4096), (129, 5120), (64, 8192)])
def test_layernorm_matches_oracle(S, h):
    print(f"[case] layernorm S={S} h={h}", flush=True)
    g = torch.Generator().manual_seed(S + h)
    x = (2.0 * torch.randn((S, h), generator=g) + 0.5).to(torch.bfloat16)
    gamma, beta, _, _ = _params(h, 128, 128, 3)
    y = mb.memo_layernorm_rows(x.cuda(), gamma.cuda(), beta.cuda(), EPS)
    torch.cuda.synchronize()
    ref = ro.layernorm(gu.to_f64(x), gu.to_f64(gamma), gu.to_f64(beta), EPS)
    gu.assert_close("layernorm", gu.to_f64(y), ref, "bf16")


def test_layernorm_constant_rows_give_beta():
    h = 1024
    x = torch.full((5, h), 3.25, dtype=torch.bfloat16)
    gamma, beta, _, _ = _params(h, 128, 128, 4)
    y = mb.memo_layernorm_rows(x.cuda(), gamma.cuda(), beta.cuda(), EPS)
    assert torch.equal(y.cpu(), beta.expand(5, h))


@pytest.mark.parametrize("S,K,N,with_bias", [(1, 128, 128, True), (77, 128, 128, False), (200, 512, 256, True),
                                              (128, 4096, 1536, True), (333, 1024, 384, False)])
def test_linear_matches_oracle(S, K, N, with_bias):
    print(f"[case] linear S={S} K={K} N={N} bias={with_bias}", flush=True)
    g = torch.Generator().manual_seed(S + K + N)
    a = torch.randn((S, K), generator=g).to(torch.bfloat16)
    _, _, w, bias = _params(512, N, K, 5)
    out = mb.memo_linear_rows(a.cuda(), w.cuda(), bias.cuda() if with_bias else None)
    torch.cuda.synchronize()
    ref = ro.linear(gu.to_f64(a), gu.to_f64(w), gu.to_f64(bias) if with_bias else None)
    gu.assert_close("linear", gu.to_f64(out), ref, "bf16")


def test_linear_identity_weight_is_exact():
    S, K = 70, 256
    a = torch.randn((S, K), generator=torch.Generator().manual_seed(9)).to(torch.bfloat16)
    w = torch.eye(K).to(torch.bfloat16)
    out = mb.memo_linear_rows(a.cuda(), w.cuda())
    assert torch.equal(out.cpu(), a)


@pytest.mark.parametrize("k", [0, 1, 77, 128, 255, 299, 300])
def test_rows_recomputed_in_a_range_are_bit_identical(k):
    S, h, N = 300, 1024, 384
    print(f"[case] recompute range k={k}", flush=True)
    g = torch.Generator().manual_seed(11)
    x = torch.randn((S, h), generator=g).to(torch.bfloat16).cuda()
    gamma, beta, w, bias = (t.cuda() for t in _params(h, N, h, 6))
    norm = mb.memo_layernorm_rows(x, gamma, beta, EPS)
    qkv = mb.memo_linear_rows(norm, w, bias)
    poison = -7.0
    norm2 = torch.full_like(norm, poison)
    qkv2 = torch.full_like(qkv, poison)
    mb.memo_layernorm_rows(x, gamma, beta, EPS, y=norm2, rows=(k, S))
    norm2[:k] = norm[:k]                      # stands for the rows that came back from the host
    mb.memo_linear_rows(norm2, w, bias, out=qkv2, rows=(k, S))
    torch.cuda.synchronize()
    assert torch.equal(norm2, norm)
    assert torch.equal(qkv2[k:], qkv[k:])
    assert bool((qkv2[:k] == poison).all())


@pytest.mark.parametrize("alpha", [0.0, 0.3, 0.625, 1.0])
def test_swap_plus_recompute_rebuilds_the_saved_tensors(alpha):
    S, h, N = 1000, 2048, 768
    print(f"[case] swap+recompute alpha={alpha}", flush=True)
    g = torch.Generator().manual_seed(12)
    x = torch.randn((S, h), generator=g).to(torch.bfloat16).cuda()
    gamma, beta, w, bias = (t.cuda() for t in _params(h, N, h, 7))
    norm = mb.memo_layernorm_rows(x, gamma, beta, EPS)
    qkv = mb.memo_linear_rows(norm, w, bias)
    torch.cuda.synchronize()
    keep_norm, keep_qkv = norm.clone(), qkv.clone()
    k = mb.memo_split_tokens(S, alpha)
    side = torch.cuda.Stream()
    hosts = [torch.empty(max(1, k * t.shape[1] * 2), dtype=torch.uint8, pin_memory=True) for t in (norm, qkv)]
    ready, out_done = torch.cuda.Event(), [torch.cuda.Event(), torch.cuda.Event()]
    ready.record()
    for t, hst, ev in zip((norm, qkv), hosts, out_done):
        mb.memo_swap_out(t, alpha, hst, side, wait_event=ready, done_event=ev)
    for ev in out_done:
        torch.cuda.current_stream().wait_event(ev)
    norm.fill_(-3.0)                           # the buffers are reused by later layers
    qkv.fill_(-3.0)
    poisoned, in_done = torch.cuda.Event(), [torch.cuda.Event(), torch.cuda.Event()]
    poisoned.record()
    for t, hst, ev in zip((norm, qkv), hosts, in_done):
        mb.memo_swap_in(t, alpha, hst, side, wait_event=poisoned, done_event=ev)
    for ev in in_done:
        torch.cuda.current_stream().wait_event(ev)
    mb.memo_layernorm_rows(x, gamma, beta, EPS, y=norm, rows=(k, S))
    mb.memo_linear_rows(norm, w, bias, out=qkv, rows=(k, S))
    torch.cuda.synchronize()
    assert torch.equal(norm, keep_norm)
    assert torch.equal(qkv, keep_qkv)
    # and against the oracle run on the layer input x alone (nothing of the HIP path enters the
    # reference): what the backward finds after swap-in + recomputation is LayerNorm(x) and its
    # projection on every row, swapped or recomputed.  The oracle keeps input_norm in fp64 where the
    # kernels store it as bf16 between the two steps; q, k, v reach |x| > 4, hence the scaled bar.
    ref_norm = ro.layernorm(gu.to_f64(x), gu.to_f64(gamma), gu.to_f64(beta), EPS)
    ref_qkv = ro.linear(ref_norm, gu.to_f64(w), gu.to_f64(bias))
    gu.assert_close("stitched qkv", gu.to_f64(qkv), ref_qkv, "bf16", scaled=True)
    gu.assert_close("norm", gu.to_f64(norm), ref_norm, "bf16", scaled=True)


@pytest.mark.parametrize("S,alpha", [(1 << 18, 0.9), (1 << 20, 0.47)])
def test_full_size_layer_sampled_rows(S, alpha):
    """One GPU's share of a 7B layer at S = 2^18 and at S = 2^20 (where S*h = 2^32 elements: every
    row offset must be 64-bit): h = 4096 -> q, k, v of 4 heads (N = 1536); rows [k,S) are
    recomputed, sampled rows are checked against the oracle run on the same rows of x."""
    h, N = 4096, 1536
    print(f"[case] recompute full size S={S} alpha={alpha}", flush=True)
    g = torch.Generator(device="cuda").manual_seed(13)
    x = torch.randn((S, h), generator=g, device="cuda").to(torch.bfloat16)
    gamma, beta, w, bias = (t.cuda() for t in _params(h, N, h, 8))
    k = mb.memo_split_tokens(S, alpha)
    norm = torch.full((S, h), -5.0, dtype=torch.bfloat16, device="cuda")
    qkv = torch.full((S, N), -5.0, dtype=torch.bfloat16, device="cuda")
    mb.memo_layernorm_rows(x, gamma, beta, EPS, y=norm, rows=(k, S))
    mb.memo_linear_rows(norm, w, bias, out=qkv, rows=(k, S))
    torch.cuda.synchronize()
    assert bool((qkv[k - 64:k] == -5.0).all()) and bool((norm[k - 64:k] == -5.0).all())
    assert bool((qkv[0] == -5.0).all())
    # rows on both sides of the 2^31- and 2^32-byte offsets of x (8 KiB rows) and of 2^31 bytes of qkv
    marks = [m for m in ((1 << 31) // (2 * h), (1 << 32) // (2 * h), (1 << 31) // (2 * N)) if k < m < S - 1]
    rows = torch.tensor(sorted({k, k + 1, k + 127, k + 128, (k + S) // 2, S - 129, S - 2, S - 1} |
                               {m + dlt for m in marks for dlt in (-1, 0, 1)}), device="cuda")
    xs, ns, qs = gu.to_f64(x[rows]), gu.to_f64(norm[rows]), gu.to_f64(qkv[rows])
    ref_n = ro.layernorm(xs, gu.to_f64(gamma), gu.to_f64(beta), EPS)
    gu.assert_close("norm rows", ns, ref_n, "bf16", scaled=True)
    gu.assert_close("qkv rows", qs, ro.linear(ref_n, gu.to_f64(w), gu.to_f64(bias)), "bf16", scaled=True)
    assert torch.isfinite(qkv[k:].float()).all()
