"""GPU parity: the HIP attention path vs the fp64 oracle, element by element, through the
C-ABI.  Sizes here are ones the dense oracle finishes in seconds; they span several tiles
(256-row query tiles and 64-row key tiles in the forward and dQ kernels, 256-row key tiles and 32-row
query tiles in the dK/dV kernel) and ragged tails."""
import math

import numpy as np
import pytest
import torch

from paper_2407_12117_amd import binding as mb
from paper_2407_12117_amd import synth
from gpu_util import LSE_MAX_ABS_BF16, assert_close, gpu_fwd_bwd, to_f64

pytestmark = pytest.mark.gpu


def _dense_case(oracle, B, S, H, d, dtype, seed, scale=None, scaled=False):
    print(f"[case] dense B={B} S={S} H={H} d={d} {dtype} seed={seed}", flush=True)
    scale = synth.default_scale(d) if scale is None else scale
    q, k, v, g = synth.attn_inputs(B, S, H, d, dtype, seed)
    o, lse, dq, dk, dv = gpu_fwd_bwd(*(t.cuda() for t in (q, k, v, g)), scale)
    qf, kf, vf, gf = (to_f64(t) for t in (q, k, v, g))
    ro, rlse = oracle.attn_fwd(qf, kf, vf, scale)
    rdq, rdk, rdv = oracle.attn_bwd(qf, kf, vf, gf, scale)
    assert_close("O", to_f64(o), ro, dtype)
    lse_err = np.abs(to_f64(lse) - rlse).max()
    assert lse_err <= (LSE_MAX_ABS_BF16 if dtype == "bf16" else 1e-4), f"LSE max_abs={lse_err:.3e}"
    assert_close("dQ", to_f64(dq), rdq, dtype, scaled)
    assert_close("dK", to_f64(dk), rdk, dtype, scaled)
    assert_close("dV", to_f64(dv), rdv, dtype, scaled)


def test_c1_fp32_dense(oracle):
    c = synth.CONFIGS["C1"]
    _dense_case(oracle, c["B"], c["S"], c["H"], c["d"], "f32", synth.config_seed("C1"))


@pytest.mark.parametrize("B,S,H,d", [(2, 333, 3, 64), (1, 257, 2, 128), (1, 1, 1, 64), (2, 31, 1, 128)])
def test_fp32_ragged_and_small(oracle, B, S, H, d):
    _dense_case(oracle, B, S, H, d, "f32", 7 + S)


@pytest.mark.parametrize("S", [1, 2, 31, 32, 33, 63, 64, 65, 97, 127, 128, 129, 200, 255, 256, 257, 287, 289, 383, 385, 511, 513, 777])
def test_bf16_small_and_ragged(oracle, S):
    _dense_case(oracle, 2, S, 2, 128, "bf16", 100 + S)


@pytest.mark.parametrize("B,S,H", [(1, 2048, 2), (2, 1024, 3), (1, 3000, 1)])
def test_bf16_multi_tile(oracle, B, S, H):
    _dense_case(oracle, B, S, H, 128, "bf16", 300 + S)


def test_bf16_many_query_tiles_dense(oracle):
    # every element of dK, dV compared where the dK/dV kernel's query loop runs up to 515 times
    # (key tile 0) and the forward / dQ kernels walk up to 258 key tiles; ragged tail
    _dense_case(oracle, 1, 16461, 1, 128, "bf16", 333)


def test_bf16_scale_below_the_usual_one(oracle):
    _dense_case(oracle, 1, 500, 2, 128, "bf16", 41, scale=0.06)


def test_bf16_scale_above_the_usual_one(oracle):
    # scale 0.2 > 1/sqrt(128): peaked softmax, gradients of magnitude > 4, where half a bf16 ulp
    # alone exceeds 2e-2: the absolute bar scales with max|ref| (gpu_util), the relative one stays
    _dense_case(oracle, 1, 500, 2, 128, "bf16", 41, scale=0.2, scaled=True)


@pytest.mark.parametrize("log2_per_tile", [3.0, 12.0, 500.0])
def test_bf16_forward_with_scores_climbing_along_the_keys(oracle, log2_per_tile):
    # The forward keeps a running maximum that it brings up to date only when a row sum shows a score
    # far above it (2^40).  Here every score grows with the key index by `log2_per_tile` binary orders
    # of magnitude per 64-key tile: 3 and 12 let the exponentials run up to 2^40 between updates, 500
    # forces an update (and the rescaling of everything accumulated so far) on every tile.
    # Forward only: with a common offset this large in K, dQ and dK are differences of nearly equal
    # sums, which the bf16 rounding of dS alone moves by several per cent in any implementation.
    B, S, H, d = 1, 1100, 2, 128
    scale = synth.default_scale(d)
    q, k, v, _ = synth.attn_inputs(B, S, H, d, "bf16", 77)
    slope = log2_per_tile / 64.0 / (scale * math.log2(math.e))        # growth of q.k per key
    q = (0.05 * q.float() + 1.0).to(torch.bfloat16)                     # q.k = sum_c k_c, nearly
    k = (0.05 * k.float() + (slope / d) * torch.arange(S, dtype=torch.float32).view(1, S, 1, 1)).to(torch.bfloat16)
    print(f"[case] climbing scores, {log2_per_tile} binary orders per tile", flush=True)
    o, lse = mb.memo_attn_fwd(q.cuda(), k.cuda(), v.cuda(), scale)
    ro, rlse = oracle.attn_fwd(to_f64(q), to_f64(k), to_f64(v), scale)
    assert_close("O", to_f64(o), ro, "bf16")
    # the logsumexp itself grows to thousands here: fp32 holds it to a relative 2^-24 or so
    assert np.abs(to_f64(lse) - rlse).max() <= LSE_MAX_ABS_BF16 * max(1.0, np.abs(rlse).max())


def test_bf16_nan_in_one_key_row_reaches_what_depends_on_it():
    # a NaN in key row j of head 0: o, lse, dq of query rows i >= j are non-finite (they see the key),
    # rows before the 256-row block of j are bit-identical to the clean run (inside the block a masked
    # zero probability may still meet the NaN in a contraction); every dk, dv row of that head is
    # reached through some query row i >= j; head 1 is untouched
    B, S, H, d, j = 1, 700, 2, 128, 389
    q, k, v, g = (t.cuda() for t in synth.attn_inputs(B, S, H, d, "bf16", 123))
    scale = synth.default_scale(d)
    clean = gpu_fwd_bwd(q, k, v, g, scale)
    k2 = k.clone()
    k2[0, j, 0, 5] = float("nan")
    o, lse, dq, dk, dv = gpu_fwd_bwd(q, k2, v, g, scale)
    for name, t, c, tok in (("o", o, clean[0], 1), ("lse", lse, clean[1], 2), ("dq", dq, clean[2], 1)):
        sl = lambda x, a, b, h: x[0, a:b, h] if tok == 1 else x[0, h, a:b]
        assert torch.isnan(sl(t, j, S, 0).float()).all(), f"{name}: rows that see the NaN key must be NaN"
        assert torch.equal(sl(t, 0, j // 256 * 256, 0), sl(c, 0, j // 256 * 256, 0)), f"{name}: rows before the NaN key's block changed"
        assert torch.equal(sl(t, 0, S, 1), sl(c, 0, S, 1)), f"{name}: the other head changed"
    for name, t, c in (("dk", dk, clean[3]), ("dv", dv, clean[4])):
        assert torch.isnan(t[0, :, 0].float()).all(), f"{name}: every key row of the head is reached"
        assert torch.equal(t[0, :, 1], c[0, :, 1]), f"{name}: the other head changed"


def test_bf16_strided_views_of_a_packed_qkv(oracle):
    # q, k, v as slices of one [B,S,3,H,d] buffer: stride_s = 3*H*d
    B, S, H, d = 1, 640, 2, 128
    print(f"[case] packed qkv S={S}", flush=True)
    scale = synth.default_scale(d)
    q, k, v, g = synth.attn_inputs(B, S, H, d, "bf16", 55)
    packed = torch.stack((q, k, v), dim=2).cuda()
    pg = torch.zeros_like(packed)
    pg[:, :, 0] = g.cuda()
    qd, kd, vd, gd = packed[:, :, 0], packed[:, :, 1], packed[:, :, 2], pg[:, :, 0]
    out = torch.zeros_like(packed)
    o, lse = mb.memo_attn_fwd(qd, kd, vd, scale, o=out[:, :, 0])
    grads = torch.zeros_like(packed)
    dq, dk, dv = mb.memo_attn_bwd(qd, kd, vd, o, lse, gd, scale, dq=grads[:, :, 0], dk=grads[:, :, 1],
                                  dv=grads[:, :, 2])
    torch.cuda.synchronize()
    qf, kf, vf, gf = (to_f64(t) for t in (q, k, v, g))
    ro, _ = oracle.attn_fwd(qf, kf, vf, scale)
    rdq, rdk, rdv = oracle.attn_bwd(qf, kf, vf, gf, scale)
    assert_close("O", to_f64(o), ro, "bf16")
    assert_close("dQ", to_f64(dq), rdq, "bf16")
    assert_close("dK", to_f64(dk), rdk, "bf16")
    assert_close("dV", to_f64(dv), rdv, "bf16")
    # the untouched slots of the packed output buffers stay zero
    assert out[:, :, 1:].abs().max().item() == 0.0


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_bf16_random_shapes_and_row_padding(oracle, seed):
    # shapes drawn at random (batch 1..2, heads 1..3, lengths on no tile edge in particular), rows
    # of 128 values inside rows of 128, 136 or 192: all eight tensors share the padded layout
    rng = np.random.default_rng(seed)
    scale = synth.default_scale(128)
    for case in range(5):
        B, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
        S = int(rng.choice([rng.integers(1, 70), rng.integers(70, 600), rng.integers(600, 2200)]))
        pad = int(rng.choice([0, 8, 64]))
        print(f"[case] random shape seed={seed} B={B} S={S} H={H} pad={pad}", flush=True)

        def padded(values=None):
            buf = torch.zeros(B, S, H, 128 + pad, dtype=torch.bfloat16, device="cuda")[..., :128]
            if values is not None:
                buf.copy_(values)
            return buf

        q, k, v, g = synth.attn_inputs(B, S, H, 128, "bf16", 5000 + 10 * seed + case)
        qd, kd, vd, gd = (padded(x) for x in (q, k, v, g))
        o, lse = mb.memo_attn_fwd(qd, kd, vd, scale, o=padded())
        dq, dk, dv = mb.memo_attn_bwd(qd, kd, vd, o, lse, gd, scale, dq=padded(), dk=padded(), dv=padded())
        torch.cuda.synchronize()
        qf, kf, vf, gf = (to_f64(x) for x in (q, k, v, g))
        ro, rlse = oracle.attn_fwd(qf, kf, vf, scale)
        rdq, rdk, rdv = oracle.attn_bwd(qf, kf, vf, gf, scale)
        assert_close("O", to_f64(o), ro, "bf16")
        assert np.abs(to_f64(lse) - rlse).max() <= LSE_MAX_ABS_BF16
        assert_close("dQ", to_f64(dq), rdq, "bf16")
        assert_close("dK", to_f64(dk), rdk, "bf16")
        assert_close("dV", to_f64(dv), rdv, "bf16")


def test_bf16_constant_values_give_constant_output():
    # rows of the softmax sum to one: V = 1 -> O = 1 (bf16 rounding of P allows 2^-8)
    B, S, H, d = 1, 1500, 2, 128
    q, k, _, _ = synth.attn_inputs(B, S, H, d, "bf16", 77)
    v = torch.ones_like(q)
    o, _ = mb.memo_attn_fwd(q.cuda(), k.cuda(), v.cuda(), synth.default_scale(d))
    torch.cuda.synchronize()
    assert (o.float() - 1.0).abs().max().item() <= 2 ** -7


def test_bf16_causality():
    # changing keys / values after position p leaves O[:p], LSE[:p] bit-identical
    B, S, H, d, p = 1, 700, 1, 128, 300
    q, k, v, _ = (t.cuda() for t in synth.attn_inputs(B, S, H, d, "bf16", 88))
    scale = synth.default_scale(d)
    o1, l1 = mb.memo_attn_fwd(q, k, v, scale)
    k2, v2 = k.clone(), v.clone()
    k2[:, p:] += 3.0
    v2[:, p:] -= 2.0
    o2, l2 = mb.memo_attn_fwd(q, k2, v2, scale)
    torch.cuda.synchronize()
    assert torch.equal(o1[:, :p], o2[:, :p]) and torch.equal(l1[:, :, :p], l2[:, :, :p])
    assert not torch.equal(o1[:, p:], o2[:, p:])


def test_bf16_is_deterministic():
    B, S, H, d = 1, 900, 2, 128
    q, k, v, g = (t.cuda() for t in synth.attn_inputs(B, S, H, d, "bf16", 99))
    a = gpu_fwd_bwd(q, k, v, g, synth.default_scale(d))
    b = gpu_fwd_bwd(q, k, v, g, synth.default_scale(d))
    for x, y in zip(a, b):
        assert torch.equal(x, y)
