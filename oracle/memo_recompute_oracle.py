"""Oracle of the token-wise recomputation of a layer's first saved tensors (Section 4.1:
the stored layer input is what "input_norm", "q", "k", "v" are rebuilt from; the rows
that were swapped come back from the host, the dropped rows [k, S) are recomputed).

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Plain numpy in float64, no blocking:
  input_norm = LayerNorm(x) over the hidden dimension (biased variance, eps inside the root)
  qkv        = input_norm @ W^T + bias          (W is [out_features, in_features])
Both are functions of one token row at a time, which is what makes the split by token legal.
"""
import numpy as np


def layernorm(x, gamma, beta, eps):
    """x: [rows, h]; gamma, beta: [h].  float64 in and out."""
    x = np.asarray(x, dtype=np.float64)
    mean = x.mean(axis=1, keepdims=True)
    var = ((x - mean) ** 2).mean(axis=1, keepdims=True)
    return (x - mean) / np.sqrt(var + eps) * np.asarray(gamma, np.float64) + np.asarray(beta, np.float64)


def linear(a, w, bias=None):
    """a: [rows, K]; w: [N, K]; bias: [N] or None -> [rows, N]."""
    out = np.asarray(a, np.float64) @ np.asarray(w, np.float64).T
    if bias is not None:
        out = out + np.asarray(bias, np.float64)
    return out


def stitch(swapped_rows, recomputed_rows, k):
    """The tensor the backward sees: rows [0,k) as they came back from the host, rows [k,S)
    recomputed.  swapped_rows holds at least k rows, recomputed_rows is indexed by token."""
    return np.concatenate([np.asarray(swapped_rows)[:k], np.asarray(recomputed_rows)[k:]], axis=0)
