"""GPU parity of the two-rounding-buffer schedule (Section 4.1, Figure 5; Section 4.3.4).

1. Bytes: every backward pass finds in its buffer exactly what the schedule oracle's byte
   replay gives (swapped prefixes of its own layer; the last two layers untouched), over
   two iterations, with copies that take far longer than the "compute" so that a missing
   wait would show.
2. A stack of stand-in layers with real attention gives bit-identical activations and
   gradients with swap + regeneration as with every layer resident; one layer's attention
   is checked against the fp64 oracle on the inputs the stack fed it.
3. Calls out of order are refused without queueing anything.
"""
import numpy as np
import pytest
import torch

from oracle import memo_sched_oracle as so
from paper_2407_12117_amd import binding as mb
from paper_2407_12117_amd import synth

import gpu_util as gu
import layer_stack as ls

pytestmark = pytest.mark.gpu

POISON = 0xEE


def _payload(dev_bytes, layer, it):
    rng = np.random.default_rng(100 * it + layer)
    a = rng.integers(0, 255, dev_bytes, dtype=np.uint8)
    a[a == POISON] = 0x11
    return a


@pytest.mark.parametrize("n_layers,S,tensors", [
    (1, 64, [(256, 1.0)]),
    (2, 64, [(256, 1.0), (100, 0.5)]),
    (3, 300, [(512, 1.0), (1024, 0.5), (96, 0.0), (2048, 0.9)]),
    (6, 8192, [(2048, 1.0), (2048, 1.0), (2048, 0.625), (1000, 0.3), (24, 1.0)]),
    (7, 4096, [(4096, 1.0), (4096, 0.75), (4096, 0.75), (4096, 0.125)]),
])
def test_backward_finds_what_the_oracle_replay_gives(n_layers, S, tensors):
    print(f"[case] sched bytes n={n_layers} S={S} tensors={tensors}", flush=True)
    slots, dev_bytes, host_bytes = mb.memo_buffer_plan_make(S, tensors)
    assert (slots, dev_bytes, host_bytes) == so.buffer_plan(S, tensors)
    bufs = [torch.full((dev_bytes,), POISON, dtype=torch.uint8, device="cuda") for _ in range(2)]
    held = so.host_store_bytes(n_layers, host_bytes)
    host = torch.full((max(held, 256),), POISON, dtype=torch.uint8, pin_memory=True)
    compute, off, pre = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    sched = mb.MemoSched(n_layers, S, tensors, bufs, host, compute, off, pre)
    for it in range(2):
        src = [torch.from_numpy(_payload(dev_bytes, l, it)).cuda() for l in range(n_layers)]
        seen = [None] * n_layers
        torch.cuda.synchronize()
        with torch.cuda.stream(compute):
            for i in range(n_layers):
                sched.forward_begin(i)
                sched.buffer(i).copy_(src[i])
                sched.forward_end(i)
            for i in range(n_layers - 1, -1, -1):
                sched.backward_begin(i)
                seen[i] = sched.buffer(i).clone()
                sched.buffer(i).fill_(POISON)       # the content is dead after its backward
                sched.backward_end(i)
        torch.cuda.synchronize()
        want = so.replay_bytes(n_layers, S, tensors, lambda l: _payload(dev_bytes, l, it),
                               poison=POISON)
        for i in range(n_layers):
            assert np.array_equal(seen[i].cpu().numpy(), want[i]), f"iteration {it} layer {i}"
    sched.destroy()


@pytest.mark.parametrize("n_layers,S,H,alpha", [(4, 640, 4, 0.5), (5, 1100, 4, 0.3), (3, 384, 8, 0.0),
                                                 (4, 512, 4, 1.0)])
def test_swapped_stack_equals_resident_stack(oracle, n_layers, S, H, alpha):
    print(f"[case] sched stack n={n_layers} S={S} H={H} alpha={alpha}", flush=True)
    d, scale = 128, synth.default_scale(128)
    g = torch.Generator().manual_seed(77)
    x0 = torch.randn((S, H * d), generator=g).to(torch.bfloat16).cuda()
    d_out = torch.randn((S, H * d), generator=g).to(torch.bfloat16).cuda()
    results = {}
    captured = {}
    for swap in (False, True):
        st = ls.LayerStack(n_layers, S, H, d, alpha, scale, swap=swap, n_saved=6)
        if swap:
            for b in st.buffers:
                b.fill_(POISON)

        def grab(i, st=st, swap=swap):
            if swap and i == 0:
                # what the first layer's backward is about to read, dropped rows regenerated
                captured["qkvo"] = [st.view(0, t).clone() for t in (3, 4, 5, 1)]
                captured["x_norm"] = [st.view(0, t).clone() for t in (0, 2)]
                captured["lse"] = st.lse[0].clone()
                captured["d_o"] = st.dx.clone()
        torch.cuda.synchronize()
        y = st.forward(x0)
        dx = st.backward(d_out, on_layer=grab)
        torch.cuda.synchronize()                      # both ran on the stack's compute stream
        y, dx = y.clone(), dx.clone()
        if swap:
            captured["dq"] = st.grads[0].clone()      # layer 0 ran last
        st.close()
        results[swap] = (y.cpu(), dx.cpu())
    assert torch.equal(results[True][0], results[False][0])
    assert torch.equal(results[True][1], results[False][1])
    assert torch.isfinite(results[True][1].float()).all()

    # what layer 0's backward found in its buffer after prefetch + token-wise recomputation, against
    # the recomputation oracle run on the stored layer input alone (rows [0,k) came from the host,
    # rows [k,S) from the LayerNorm and projection kernels)
    from oracle import memo_recompute_oracle as ro
    x_in, norm = (gu.to_f64(t) for t in captured["x_norm"])
    assert np.array_equal(x_in, gu.to_f64(x0))
    gamma, beta, proj = ls.layer_params(0, H * d, "cpu")
    ref_norm = ro.layernorm(x_in, gu.to_f64(gamma), gu.to_f64(beta), ls.EPS)
    gu.assert_close("norm", norm, ref_norm, "bf16", scaled=True)
    for name, got, (w, b) in zip("qkv", captured["qkvo"][:3], proj):
        gu.assert_close(name, gu.to_f64(got), ro.linear(ref_norm, gu.to_f64(w), gu.to_f64(b)), "bf16", scaled=True)

    # layer 0 of the swapped run against the fp64 oracle, on the very tensors it was fed
    q, k, v, o = [gu.to_f64(t).reshape(1, S, H, d) for t in captured["qkvo"]]
    d_o = gu.to_f64(captured["d_o"]).reshape(1, S, H, d)
    ref_o, ref_lse = oracle.attn_fwd(q, k, v, scale)
    ref_dq, _, _ = oracle.attn_bwd(q, k, v, d_o, scale)
    gu.assert_close("o", o, ref_o, "bf16")
    assert np.abs(gu.to_f64(captured["lse"]) - ref_lse).max() <= gu.LSE_MAX_ABS_BF16
    # The bars are stated for unit-scale N(0,1) inputs; here dO has grown through the
    # layers above and q, k carry the layer scalars, so the max-abs bar is taken relative
    # to the largest reference magnitude (the relative-L2 bar needs no such care).
    max_abs, rel = gu.errors(gu.to_f64(captured["dq"]), ref_dq)
    assert rel <= gu.BF16_REL_L2, rel
    assert max_abs <= gu.BF16_MAX_ABS * max(1.0, float(np.abs(ref_dq).max())), max_abs


def test_calls_out_of_order_are_refused():
    tensors = [(256, 1.0), (256, 0.5)]
    _, dev_bytes, host_bytes = mb.memo_buffer_plan_make(128, tensors)
    bufs = [torch.zeros(dev_bytes, dtype=torch.uint8, device="cuda") for _ in range(2)]
    host = torch.zeros(2 * host_bytes, dtype=torch.uint8, pin_memory=True)
    s = torch.cuda.Stream()
    sched = mb.MemoSched(4, 128, tensors, bufs, host, s, s, s)
    L = mb.lib()
    for bad in (lambda: sched.forward_end(0), lambda: sched.forward_begin(1),
                lambda: sched.backward_begin(3), lambda: sched.forward_begin(4)):
        with pytest.raises(mb.MemoError) as e:
            bad()
        assert e.value.status == mb.MEMO_ERR_INVALID_ARG
    for i in range(4):
        sched.forward_begin(i)
        sched.forward_end(i)
    with pytest.raises(mb.MemoError):
        sched.forward_begin(0)                     # the backward passes come first
    with pytest.raises(mb.MemoError):
        sched.backward_begin(2)
    for i in range(3, -1, -1):
        sched.backward_begin(i)
        sched.backward_end(i)
    sched.forward_begin(0)                         # next iteration
    assert L.memo_sched_buffer(sched._h, 1) == bufs[1].data_ptr()
    assert L.memo_sched_buffer(sched._h, 2) == bufs[0].data_ptr()
    torch.cuda.synchronize()
    sched.destroy()

    # host store one slot short: the host out-of-memory case, before anything is created
    small = torch.zeros(2 * host_bytes - 1, dtype=torch.uint8, pin_memory=True)
    with pytest.raises(mb.MemoError) as e:
        mb.MemoSched(4, 128, tensors, bufs, small, s, s, s)
    assert e.value.status == mb.MEMO_ERR_HOST_CAPACITY
