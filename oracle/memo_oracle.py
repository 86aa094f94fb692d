"""ctypes front end of the fp64 CPU oracle (oracle/memo_oracle.c).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only tests, the smoke check and the
benchmark's cpu_baseline leg import this.  It imports nothing from the HIP
package.  Arrays in and out are numpy float64 (attention) or uint8 (swap).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "memo_oracle.c")
_LIB = os.path.join(_HERE, "libmemo_oracle.so")

_c_d = ctypes.POINTER(ctypes.c_double)
_c_i64 = ctypes.POINTER(ctypes.c_int64)
_c_u8 = ctypes.POINTER(ctypes.c_ubyte)


def build(force=False):
    """Compile the C oracle with gcc (fp64, -O2, OpenMP over rows/columns)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra",
           "-fno-fast-math", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.memo_oracle_attn_fwd.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_double, _c_d, _c_d, _c_d, _c_d, _c_d]
        L.memo_oracle_attn_fwd.restype = None
        L.memo_oracle_attn_bwd.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_double, _c_d, _c_d, _c_d, _c_d, _c_d, _c_d, _c_d]
        L.memo_oracle_attn_bwd.restype = None
        L.memo_oracle_head_rows.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_double,
                                            _c_d, _c_d, _c_d, _c_d, ctypes.c_int64, _c_i64,
                                            _c_d, _c_d, _c_d, _c_d]
        L.memo_oracle_head_rows.restype = None
        L.memo_oracle_head_dkdv_tail.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_double,
                                                 _c_d, _c_d, _c_d, _c_d, ctypes.c_int64, _c_d, _c_d]
        L.memo_oracle_head_dkdv_tail.restype = None
        L.memo_oracle_split_tokens.argtypes = [ctypes.c_int64, ctypes.c_double]
        L.memo_oracle_split_tokens.restype = ctypes.c_int64
        L.memo_oracle_swap_plan.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_double, _c_i64]
        L.memo_oracle_swap_plan.restype = ctypes.c_int
        L.memo_oracle_swap_out.argtypes = [_c_u8, ctypes.c_int64, ctypes.c_int64, ctypes.c_double,
                                           _c_u8, ctypes.c_int64]
        L.memo_oracle_swap_out.restype = ctypes.c_int64
        L.memo_oracle_swap_in.argtypes = [_c_u8, ctypes.c_int64, ctypes.c_int64, ctypes.c_double,
                                          _c_u8, ctypes.c_int64]
        L.memo_oracle_swap_in.restype = ctypes.c_int64
        L.memo_oracle_alpha_grid.argtypes = [ctypes.c_double] * 5 + [ctypes.c_int, ctypes.c_double,
                                                                     ctypes.c_int]
        L.memo_oracle_alpha_grid.restype = ctypes.c_double
        L.memo_oracle_num_threads.argtypes = []
        L.memo_oracle_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a


def _p(a):
    return a.ctypes.data_as(_c_d)


def num_threads():
    return int(lib().memo_oracle_num_threads())


def attn_fwd(q, k, v, scale):
    """q,k,v: [B,S,H,d] -> (o [B,S,H,d], lse [B,H,S]), all float64."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, S, H, d = q.shape
    assert k.shape == q.shape and v.shape == q.shape
    o = np.empty_like(q)
    lse = np.empty((B, H, S), dtype=np.float64)
    lib().memo_oracle_attn_fwd(B, S, H, d, float(scale), _p(q), _p(k), _p(v), _p(o), _p(lse))
    return o, lse


def attn_bwd(q, k, v, d_o, scale):
    """Gradients of L = sum(O*dO): returns (dq, dk, dv), [B,S,H,d] float64."""
    q, k, v, d_o = _f64(q), _f64(k), _f64(v), _f64(d_o)
    B, S, H, d = q.shape
    dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
    lib().memo_oracle_attn_bwd(B, S, H, d, float(scale), _p(q), _p(k), _p(v), _p(d_o),
                               _p(dq), _p(dk), _p(dv))
    return dq, dk, dv


def head_rows(q, k, v, d_o, rows, scale):
    """One head, q,k,v,d_o: [S,d].  For the listed query rows returns
    (o [n,d], lse [n], delta [n], dq [n,d]); delta and dq are None if d_o is None."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    S, d = q.shape
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    assert rows.ndim == 1 and (rows >= 0).all() and (rows < S).all()
    n = rows.shape[0]
    o = np.empty((n, d), dtype=np.float64)
    lse = np.empty((n,), dtype=np.float64)
    if d_o is None:
        lib().memo_oracle_head_rows(S, d, float(scale), _p(q), _p(k), _p(v), None, n,
                                    rows.ctypes.data_as(_c_i64), _p(o), _p(lse), None, None)
        return o, lse, None, None
    d_o = _f64(d_o)
    delta = np.empty((n,), dtype=np.float64)
    dq = np.empty((n, d), dtype=np.float64)
    lib().memo_oracle_head_rows(S, d, float(scale), _p(q), _p(k), _p(v), _p(d_o), n,
                                rows.ctypes.data_as(_c_i64), _p(o), _p(lse), _p(delta), _p(dq))
    return o, lse, delta, dq


def head_dkdv_tail(q, k, v, d_o, j0, scale):
    """One head: (dk, dv) for key columns [j0, S), each [S-j0, d]."""
    q, k, v, d_o = _f64(q), _f64(k), _f64(v), _f64(d_o)
    S, d = q.shape
    assert 0 <= j0 < S
    dk = np.empty((S - j0, d), dtype=np.float64)
    dv = np.empty((S - j0, d), dtype=np.float64)
    lib().memo_oracle_head_dkdv_tail(S, d, float(scale), _p(q), _p(k), _p(v), _p(d_o), int(j0),
                                     _p(dk), _p(dv))
    return dk, dv


def split_tokens(S, alpha):
    return int(lib().memo_oracle_split_tokens(int(S), float(alpha)))


def swap_plan(S, row_bytes, alpha):
    """dict(k_swapped, n_recompute, bytes_swapped, bytes_dropped, recompute_byte_offset) or None."""
    out = (ctypes.c_int64 * 5)()
    rc = lib().memo_oracle_swap_plan(int(S), int(row_bytes), float(alpha), out)
    if rc != 0:
        return None
    return dict(k_swapped=out[0], n_recompute=out[1], bytes_swapped=out[2], bytes_dropped=out[3],
                recompute_byte_offset=out[4])


def swap_out(act, row_bytes, alpha, host):
    """act: uint8 [S*row_bytes]; host: uint8 buffer (written in place). Returns bytes or <0."""
    assert act.dtype == np.uint8 and host.dtype == np.uint8
    S = act.size // row_bytes
    return int(lib().memo_oracle_swap_out(act.ctypes.data_as(_c_u8), S, int(row_bytes), float(alpha),
                                          host.ctypes.data_as(_c_u8), host.size))


def swap_in(act, row_bytes, alpha, host):
    assert act.dtype == np.uint8 and host.dtype == np.uint8
    S = act.size // row_bytes
    return int(lib().memo_oracle_swap_in(act.ctypes.data_as(_c_u8), S, int(row_bytes), float(alpha),
                                         host.ctypes.data_as(_c_u8), host.size))


def alpha_grid(s_in, s_attn, s_oth, bandwidth, t_layer, n_layers, m_cpu, steps):
    return float(lib().memo_oracle_alpha_grid(float(s_in), float(s_attn), float(s_oth),
                                              float(bandwidth), float(t_layer), int(n_layers),
                                              float(m_cpu), int(steps)))
