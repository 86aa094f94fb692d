"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds none of the method's arithmetic: it only draws the random
tensors and byte patterns that both the HIP path and the CPU oracle are fed.
Values are rounded to the test dtype once, here, so both sides see identical
numbers.

Recipe (the paper trains on unnamed text; these stand in for it): Q, K, V, dO
are i.i.d. N(0,1) in layout [B, S, H, d]; with scale 1/sqrt(d) the scores are
about N(0,1), an early-training regime.  Saved activations are a byte pattern
that is a function of (row, column, seed), so a misplaced row is detected.
"""
import math

import torch

# The five workloads: attention shape + the activation that is swapped beside it.
CONFIGS = {
    "C1": dict(B=1, H=1, S=1024, d=64, dtype="f32", act_cols=256, act_elem=4, alpha=0.5),
    "C2": dict(B=1, H=4, S=32768, d=128, dtype="bf16", act_cols=4096, act_elem=2, alpha=0.75),
    "C3": dict(B=1, H=4, S=131072, d=128, dtype="bf16", act_cols=4096, act_elem=2, alpha=1.0),
    "C4": dict(B=1, H=5, S=262144, d=128, dtype="bf16", act_cols=5120, act_elem=2, alpha=0.9),
    "C5": dict(B=1, H=4, S=1048576, d=128, dtype="bf16", act_cols=4096, act_elem=2, alpha=1.0),
}


def config_seed(name):
    return 1000 + int(name[1:])


def torch_dtype(name):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def attn_inputs(B, S, H, d, dtype, seed, device="cpu"):
    """q, k, v, d_o: [B,S,H,d] tensors of `dtype` ("f32" | "bf16"), N(0,1) rounded once."""
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    out = []
    for _ in range(4):
        t = torch.randn((B, S, H, d), generator=g, dtype=torch.float32, device=device)
        out.append(t.to(torch_dtype(dtype)))
    return tuple(out)


def default_scale(d):
    return 1.0 / math.sqrt(d)


def activation(S, row_bytes, seed, device="cpu", chunk_rows=None):
    """uint8 tensor [S, row_bytes]; byte (r, c) = hash of (r, c, seed)."""
    act = torch.empty((S, row_bytes), dtype=torch.uint8, device=device)
    if chunk_rows is None:
        chunk_rows = max(1, (1 << 25) // max(1, row_bytes))
    cols = torch.arange(row_bytes, dtype=torch.int64, device=device)
    for r0 in range(0, S, chunk_rows):
        r1 = min(S, r0 + chunk_rows)
        rows = torch.arange(r0, r1, dtype=torch.int64, device=device)
        act[r0:r1] = activation_bytes(rows[:, None], cols[None, :], seed)
    return act


def activation_bytes(rows, cols, seed):
    """The byte pattern itself, for int64 tensors `rows`, `cols` (broadcastable)."""
    x = rows * 2654435761 + cols * 40503 + int(seed) * 97
    x = x ^ (x >> 13)
    return ((x >> 3) & 0xFF).to(torch.uint8)
