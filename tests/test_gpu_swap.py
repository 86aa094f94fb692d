"""GPU parity of the token-wise swap (Section 4.1): bytes on the host store and bytes
restored on the device are identical to what the oracle's memcpy bookkeeping gives;
rows marked for recomputation are never read or written; stream/event ordering holds."""
import numpy as np
import pytest
import torch

from paper_2407_12117_amd import binding as mb
from paper_2407_12117_amd import synth

pytestmark = pytest.mark.gpu

ALPHAS = [t / 8 for t in range(9)] + [0.9]


def _pinned(nbytes, fill):
    t = torch.empty(max(nbytes, 1), dtype=torch.uint8, pin_memory=True)
    t.fill_(fill)
    return t


@pytest.mark.parametrize("alpha", ALPHAS)
@pytest.mark.parametrize("S,row_bytes", [(1024, 1024), (203, 40), (4096, 8192)])
def test_round_trip_matches_oracle(oracle, alpha, S, row_bytes):
    print(f"[case] swap S={S} row_bytes={row_bytes} alpha={alpha}", flush=True)
    act_cpu = synth.activation(S, row_bytes, seed=5)
    act = act_cpu.cuda()
    host = _pinned(S * row_bytes + 64, 0xEE)
    side = torch.cuda.Stream()
    done = torch.cuda.Event()
    ready = torch.cuda.Event()
    ready.record()
    mb.memo_swap_out(act, alpha, host, side, wait_event=ready, done_event=done)
    done.synchronize()
    # oracle: same bytes through memcpy bookkeeping
    ref_host = np.full(S * row_bytes + 64, 0xEE, dtype=np.uint8)
    n = oracle.swap_out(act_cpu.numpy().reshape(-1), row_bytes, alpha, ref_host)
    assert n == mb.memo_swap_plan_make(S, row_bytes, alpha)["bytes_swapped"]
    assert np.array_equal(host.numpy(), ref_host)

    # forward is over: the device buffer is reused (poisoned), then the swapped rows return
    restored = torch.full_like(act, 0x5A)
    poisoned, done2 = torch.cuda.Event(), torch.cuda.Event()
    poisoned.record()                      # the copy stream must not overtake the fill
    mb.memo_swap_in(restored, alpha, host, side, wait_event=poisoned, done_event=done2)
    done2.synchronize()
    ref_restored = np.full(S * row_bytes, 0x5A, dtype=np.uint8)
    oracle.swap_in(ref_restored, row_bytes, alpha, ref_host)
    assert np.array_equal(restored.cpu().numpy().reshape(-1), ref_restored)


def test_c1_activation_fp32(oracle):
    c = synth.CONFIGS["C1"]
    S, row_bytes = c["S"], c["act_cols"] * c["act_elem"]
    act = torch.randn((S, c["act_cols"]), generator=torch.Generator().manual_seed(1001)).cuda()
    host = torch.zeros((S, c["act_cols"]), dtype=torch.float32, pin_memory=True)
    side = torch.cuda.Stream()
    ev = torch.cuda.Event()
    ready = torch.cuda.Event()
    ready.record()
    mb.memo_swap_out(act, c["alpha"], host, side, wait_event=ready, done_event=ev)
    ev.synchronize()
    k = oracle.split_tokens(S, c["alpha"])
    assert k == 512
    assert torch.equal(host[:k], act[:k].cpu()) and host[k:].abs().max().item() == 0.0
    back = torch.full_like(act, float("nan"))
    filled = torch.cuda.Event()
    filled.record()
    mb.memo_swap_in(back, c["alpha"], host, side, wait_event=filled, done_event=ev)
    ev.synchronize()
    assert torch.equal(back[:k], act[:k]) and torch.isnan(back[k:]).all()


def test_swap_out_waits_for_the_producer_event():
    # The activation is produced on the compute stream by a long chain of kernels; the copy on
    # the side stream must see the final bytes, which it only can if it waits for the event.
    S, cols = 8192, 2048
    act = torch.zeros((S, cols), dtype=torch.float32, device="cuda")
    host = torch.zeros((S, cols), dtype=torch.float32, pin_memory=True)
    side = torch.cuda.Stream()
    produced, done = torch.cuda.Event(), torch.cuda.Event()
    torch.cuda.synchronize()
    for _ in range(200):
        act.add_(1.0)
    produced.record()
    mb.memo_swap_out(act, 1.0, host, side, wait_event=produced, done_event=done)
    done.synchronize()
    assert host.min().item() == 200.0 and host.max().item() == 200.0


def test_done_event_gates_reuse_of_the_device_buffer():
    # Section 4.1: an event tells when the buffer has been fully offloaded and may be rewritten.
    S, cols = 16384, 4096
    act = torch.full((S, cols), 3.0, dtype=torch.float32, device="cuda")
    host = torch.zeros((S, cols), dtype=torch.float32, pin_memory=True)
    side = torch.cuda.Stream()
    produced, done = torch.cuda.Event(), torch.cuda.Event()
    produced.record()
    mb.memo_swap_out(act, 1.0, host, side, wait_event=produced, done_event=done)
    torch.cuda.current_stream().wait_event(done)     # the next layer waits, then overwrites
    act.fill_(-1.0)
    torch.cuda.synchronize()
    assert host.min().item() == 3.0 and host.max().item() == 3.0


def test_alpha_zero_queues_no_copy_but_honours_events():
    act = torch.ones((64, 64), dtype=torch.float32, device="cuda")
    host = torch.zeros((64, 64), dtype=torch.float32, pin_memory=True)
    side = torch.cuda.Stream()
    done = torch.cuda.Event()
    mb.memo_swap_out(act, 0.0, host, side, done_event=done)
    done.synchronize()
    assert host.abs().max().item() == 0.0


def test_host_capacity_error_leaves_host_untouched():
    act = torch.ones((64, 64), dtype=torch.float32, device="cuda")
    host = torch.zeros((31, 64), dtype=torch.float32, pin_memory=True)
    side = torch.cuda.Stream()
    with pytest.raises(mb.MemoError) as e:
        mb.memo_swap_out(act, 0.5, host, side)
    assert e.value.status == mb.MEMO_ERR_HOST_CAPACITY
    torch.cuda.synchronize()
    assert host.abs().max().item() == 0.0


def test_pinned_helpers():
    import ctypes
    p = ctypes.c_void_p()
    assert mb.lib().memo_host_alloc(ctypes.byref(p), 1 << 20) == mb.MEMO_OK and p.value
    assert mb.lib().memo_host_free(p) == mb.MEMO_OK
