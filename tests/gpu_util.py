"""Helpers shared by the GPU parity tests (not collected by pytest)."""
import numpy as np
import torch

from paper_2407_12117_amd import binding as mb

# Parity bars.  bf16: outputs and gradients within max-abs 2e-2 and relative-L2 1e-2 of the
# fp64 oracle; fp32 path within 1e-4.  The logsumexp is an fp32 output on both paths (bf16
# inputs are exact in fp32, products accumulate in fp32), so it gets a much tighter bar.
# The absolute bar belongs to unit-scale outputs (|x| up to about 4, where half a bf16 ulp is at most
# 1.6e-2): a correctly rounded bf16 result of magnitude m is off by up to m * 2^-9, so a case whose
# outputs are larger (a scale above 1/sqrt(d), unnormalised activations) uses the same bar times
# max(1, max|ref|) (`scaled=True`); the relative-L2 bar is scale-free and never changes.
BF16_MAX_ABS, BF16_REL_L2 = 2e-2, 1e-2
F32_MAX_ABS = 1e-4
LSE_MAX_ABS_BF16 = 1e-4


def to_f64(t):
    return t.detach().to("cpu").to(torch.float64).numpy()


def gpu_fwd_bwd(q, k, v, d_o, scale):
    """Runs the library on cuda tensors; returns (o, lse, dq, dk, dv) as cuda tensors."""
    o, lse = mb.memo_attn_fwd(q, k, v, scale)
    dq, dk, dv = mb.memo_attn_bwd(q, k, v, o, lse, d_o, scale)
    torch.cuda.synchronize()
    return o, lse, dq, dk, dv


def errors(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    diff = got - ref
    max_abs = float(np.abs(diff).max()) if diff.size else 0.0
    den = float(np.linalg.norm(ref.ravel()))
    rel = float(np.linalg.norm(diff.ravel())) / den if den > 0 else float(np.linalg.norm(diff.ravel()))
    return max_abs, rel


def assert_close(name, got, ref, dtype, scaled=False):
    assert np.isfinite(np.asarray(got, dtype=np.float64)).all(), f"{name}: non-finite values"
    max_abs, rel = errors(got, ref)
    if dtype == "bf16":
        bar = BF16_MAX_ABS * (max(1.0, float(np.abs(ref).max())) if scaled else 1.0)
        assert max_abs <= bar and rel <= BF16_REL_L2, f"{name}: max_abs={max_abs:.3e} (bar {bar:.3e}) rel_l2={rel:.3e}"
    else:
        assert max_abs <= F32_MAX_ABS, f"{name}: max_abs={max_abs:.3e} rel_l2={rel:.3e}"
    return max_abs, rel
