"""Thin ctypes binding of libmemo.so (contract: include/memo.h).

Argument marshalling only: every step of the path runs inside the library's kernels
and copies.  PyTorch appears only as the owner of device memory, pinned host memory
and streams.  There is no fallback: if the library is not built, loading raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmemo.so")

MEMO_OK = 0
MEMO_ERR_INVALID_ARG = 1
MEMO_ERR_UNSUPPORTED = 2
MEMO_ERR_HOST_CAPACITY = 3
MEMO_ERR_WORKSPACE = 4
MEMO_ERR_DEVICE = 5
MEMO_F32 = 0
MEMO_BF16 = 1

EXPORTS = [
    "memo_attn_fwd", "memo_attn_bwd_workspace_bytes", "memo_attn_bwd", "memo_attn_bwd_staged",
    "memo_attn_bwd_static",
    "memo_split_tokens",
    "memo_swap_plan_make", "memo_swap_out", "memo_swap_in", "memo_solve_alpha",
    "memo_host_alloc", "memo_host_free", "memo_status_str",
    "memo_buffer_plan_make", "memo_sched_create", "memo_sched_forward_begin",
    "memo_sched_forward_end", "memo_sched_backward_begin", "memo_sched_backward_end",
    "memo_sched_buffer", "memo_sched_destroy",
    "memo_layernorm_rows", "memo_linear_rows",
    "memo_trace_to_requests", "memo_dsa_plan", "memo_dsa_plan_bilevel",
]


class MemoAttnDesc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("d", ctypes.c_int32),
                ("S", ctypes.c_int64), ("dtype", ctypes.c_int32), ("scale", ctypes.c_float),
                ("stride_b", ctypes.c_int64), ("stride_s", ctypes.c_int64),
                ("stride_h", ctypes.c_int64), ("causal", ctypes.c_int32),
                ("flags", ctypes.c_uint32)]


class MemoSwapPlan(ctypes.Structure):
    _fields_ = [("S", ctypes.c_int64), ("row_bytes", ctypes.c_int64),
                ("k_swapped", ctypes.c_int64), ("n_recompute", ctypes.c_int64),
                ("bytes_swapped", ctypes.c_int64), ("bytes_dropped", ctypes.c_int64),
                ("recompute_byte_offset", ctypes.c_int64)]


class MemoTensorDesc(ctypes.Structure):
    _fields_ = [("row_bytes", ctypes.c_int64), ("alpha", ctypes.c_double)]


class MemoTensorSlot(ctypes.Structure):
    _fields_ = [("dev_offset", ctypes.c_int64), ("host_offset", ctypes.c_int64),
                ("k_swapped", ctypes.c_int64), ("bytes_swapped", ctypes.c_size_t)]


class MemoDsaRequest(ctypes.Structure):
    _fields_ = [("size", ctypes.c_int64), ("start", ctypes.c_int32), ("end", ctypes.c_int32)]


class MemoBilevelPlan(ctypes.Structure):
    _fields_ = [("peak", ctypes.c_int64), ("fwd_peak", ctypes.c_int64), ("bwd_peak", ctypes.c_int64),
                ("fwd_offsets", ctypes.POINTER(ctypes.c_int64)), ("bwd_offsets", ctypes.POINTER(ctypes.c_int64)),
                ("fwd_base", ctypes.POINTER(ctypes.c_int64)), ("bwd_base", ctypes.POINTER(ctypes.c_int64)),
                ("outer_addr", ctypes.POINTER(ctypes.c_int64)), ("optimal", ctypes.c_int32)]


class MemoError(RuntimeError):
    def __init__(self, status, what):
        self.status = int(status)
        super().__init__(f"{what}: {status_str(status)} (status {int(status)})")


_lib = None


def lib():
    """Loads libmemo.so; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                           "`python -c 'import __graft_entry__ as g; g.build()'`")
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, f64, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_double, ctypes.c_size_t
    dp = ctypes.POINTER(MemoAttnDesc)
    L.memo_attn_fwd.argtypes = [dp, vp, vp, vp, vp, vp, vp]
    L.memo_attn_fwd.restype = ctypes.c_int
    L.memo_attn_bwd_workspace_bytes.argtypes = [dp]
    L.memo_attn_bwd_workspace_bytes.restype = sz
    L.memo_attn_bwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.memo_attn_bwd.restype = ctypes.c_int
    L.memo_attn_bwd_staged.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp,
                                       ctypes.POINTER(ctypes.c_void_p)]
    L.memo_attn_bwd_staged.restype = ctypes.c_int
    L.memo_attn_bwd_static.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.memo_attn_bwd_static.restype = ctypes.c_int
    L.memo_split_tokens.argtypes = [i64, f64]
    L.memo_split_tokens.restype = i64
    L.memo_swap_plan_make.argtypes = [i64, i64, f64, ctypes.POINTER(MemoSwapPlan)]
    L.memo_swap_plan_make.restype = ctypes.c_int
    L.memo_swap_out.argtypes = [vp, i64, i64, f64, vp, sz, vp, vp, vp]
    L.memo_swap_out.restype = ctypes.c_int
    L.memo_swap_in.argtypes = [vp, i64, i64, f64, vp, sz, vp, vp, vp]
    L.memo_swap_in.restype = ctypes.c_int
    L.memo_solve_alpha.argtypes = [f64, f64, f64, f64, f64, ctypes.c_int32, f64,
                                   ctypes.POINTER(ctypes.c_double)]
    L.memo_solve_alpha.restype = ctypes.c_int
    L.memo_host_alloc.argtypes = [ctypes.POINTER(ctypes.c_void_p), sz]
    L.memo_host_alloc.restype = ctypes.c_int
    L.memo_host_free.argtypes = [vp]
    L.memo_host_free.restype = ctypes.c_int
    L.memo_status_str.argtypes = [ctypes.c_int]
    L.memo_status_str.restype = ctypes.c_char_p
    tdp = ctypes.POINTER(MemoTensorDesc)
    L.memo_buffer_plan_make.argtypes = [i64, ctypes.c_int32, tdp, ctypes.POINTER(MemoTensorSlot),
                                        ctypes.POINTER(sz), ctypes.POINTER(sz)]
    L.memo_buffer_plan_make.restype = ctypes.c_int
    L.memo_sched_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int32, i64, ctypes.c_int32, tdp,
                                    vp, vp, vp, sz, vp, vp, vp]
    L.memo_sched_create.restype = ctypes.c_int
    for name in ("memo_sched_forward_begin", "memo_sched_forward_end",
                 "memo_sched_backward_begin", "memo_sched_backward_end"):
        getattr(L, name).argtypes = [vp, ctypes.c_int32]
        getattr(L, name).restype = ctypes.c_int
    L.memo_sched_buffer.argtypes = [vp, ctypes.c_int32]
    L.memo_sched_buffer.restype = vp
    L.memo_sched_destroy.argtypes = [vp]
    L.memo_sched_destroy.restype = ctypes.c_int
    rp, i64p, i32p = ctypes.POINTER(MemoDsaRequest), ctypes.POINTER(i64), ctypes.POINTER(ctypes.c_int32)
    L.memo_trace_to_requests.argtypes = [ctypes.c_int32, i32p, i64p, i64p, rp, i64p, i32p]
    L.memo_trace_to_requests.restype = ctypes.c_int
    L.memo_dsa_plan.argtypes = [ctypes.c_int32, rp, i64, i64, i64p, i64p, i32p]
    L.memo_dsa_plan.restype = ctypes.c_int
    L.memo_dsa_plan_bilevel.argtypes = [ctypes.c_int32, rp, ctypes.c_int32, rp, ctypes.c_int32, i32p, i32p,
                                        ctypes.c_int32, rp, i64, i64, ctypes.POINTER(MemoBilevelPlan)]
    L.memo_dsa_plan_bilevel.restype = ctypes.c_int
    L.memo_layernorm_rows.argtypes = [vp, vp, vp, vp, i64, ctypes.c_int32, ctypes.c_float, i64, i64, vp]
    L.memo_layernorm_rows.restype = ctypes.c_int
    L.memo_linear_rows.argtypes = [vp, vp, vp, vp, i64, ctypes.c_int32, ctypes.c_int32, i64, i64, vp]
    L.memo_linear_rows.restype = ctypes.c_int
    _lib = L
    return L


def status_str(status):
    return lib().memo_status_str(int(status)).decode()


def _check(status, what):
    if status != MEMO_OK:
        raise MemoError(status, what)


def _stream_ptr(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _event_ptr(event, create_on=None):
    """hipEvent_t of a torch event.  torch creates the handle lazily at the first record():
    an event the library is to record (create_on = that stream) is recorded once here to
    bring the handle into being (the library's later record supersedes it); an event the
    library is to WAIT for must already have been recorded by its producer."""
    if event is None:
        return None
    if isinstance(event, int):
        return event
    if not event.cuda_event:
        if create_on is None:
            raise ValueError("wait_event has never been recorded: there is nothing to wait for")
        event.record(create_on if not isinstance(create_on, int) else None)
    return event.cuda_event


def _stream_obj(stream):
    return torch.cuda.current_stream() if stream is None else stream


def make_desc(q, scale, causal=1, flags=0):
    """Descriptor for a [B,S,H,d] tensor (any strides with contiguous last dim)."""
    if q.dim() != 4 or q.stride(3) != 1:
        raise ValueError("attention tensors must be [B,S,H,d] with contiguous d")
    dt = {torch.float32: MEMO_F32, torch.bfloat16: MEMO_BF16}.get(q.dtype)
    if dt is None:
        raise ValueError(f"unsupported dtype {q.dtype}")
    B, S, H, d = q.shape
    return MemoAttnDesc(B=B, H=H, d=d, S=S, dtype=dt, scale=float(scale),
                        stride_b=q.stride(0), stride_s=q.stride(1), stride_h=q.stride(2),
                        causal=causal, flags=flags)


def _same_layout(ref, *others):
    for t in others:
        if t.shape != ref.shape or t.stride() != ref.stride() or t.dtype != ref.dtype:
            raise ValueError("q, k, v, o, d_o, dq, dk, dv must share shape, strides and dtype")
        if t.device != ref.device:
            raise ValueError("tensors must live on one device")


def memo_attn_fwd(q, k, v, scale, o=None, lse=None, stream=None):
    """o, lse = causal softmax attention of q,k,v [B,S,H,d]; lse is [B,H,S] fp32."""
    B, S, H, d = q.shape
    if o is None:
        o = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((B, H, S), dtype=torch.float32, device=q.device)
    _same_layout(q, k, v, o)
    if lse.dtype != torch.float32 or not lse.is_contiguous() or tuple(lse.shape) != (B, H, S):
        raise ValueError("lse must be contiguous fp32 [B,H,S]")
    desc = make_desc(q, scale)
    st = lib().memo_attn_fwd(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                             o.data_ptr(), lse.data_ptr(), _stream_ptr(stream))
    _check(st, "memo_attn_fwd")
    return o, lse


def memo_attn_bwd_workspace_bytes(q, scale):
    desc = make_desc(q, scale)
    return int(lib().memo_attn_bwd_workspace_bytes(ctypes.byref(desc)))


def memo_attn_bwd(q, k, v, o, lse, d_o, scale, dq=None, dk=None, dv=None, workspace=None,
                  stream=None, stage_events=None):
    """dq, dk, dv for dL/dO = d_o.  `workspace`: uint8 device tensor (allocated if None).
    stage_events: optional 4 torch.cuda.Event(enable_timing=True), passed to memo_attn_bwd_staged."""
    if dq is None:
        dq = torch.empty_like(q)
    if dk is None:
        dk = torch.empty_like(q)
    if dv is None:
        dv = torch.empty_like(q)
    _same_layout(q, k, v, o, d_o, dq, dk, dv)
    desc = make_desc(q, scale)
    if workspace is None:
        need = int(lib().memo_attn_bwd_workspace_bytes(ctypes.byref(desc)))
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    args = (ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(),
            o.data_ptr(), lse.data_ptr(), d_o.data_ptr(),
            dq.data_ptr(), dk.data_ptr(), dv.data_ptr(),
            workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))
    if stage_events is None:
        st = lib().memo_attn_bwd(*args)
    else:
        if len(stage_events) != 4:
            raise ValueError("stage_events must hold 4 events")
        handles = (ctypes.c_void_p * 4)(*[_event_ptr(e, _stream_obj(stream)) for e in stage_events])
        st = lib().memo_attn_bwd_staged(*args, handles)
    _check(st, "memo_attn_bwd")
    return dq, dk, dv


def memo_attn_bwd_static(q, k, v, o, lse, d_o, scale, dq, dk, dv, stream=None):
    """memo_attn_bwd without a workspace and without any allocation: the caller passes every
    output; the library keeps D_i in its static device array (B*H*S <= 4 Mi rows)."""
    _same_layout(q, k, v, o, d_o, dq, dk, dv)
    desc = make_desc(q, scale)
    _check(lib().memo_attn_bwd_static(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                      o.data_ptr(), lse.data_ptr(), d_o.data_ptr(), dq.data_ptr(),
                                      dk.data_ptr(), dv.data_ptr(), _stream_ptr(stream)),
           "memo_attn_bwd_static")
    return dq, dk, dv


def memo_split_tokens(S, alpha):
    return int(lib().memo_split_tokens(int(S), float(alpha)))


def memo_swap_plan_make(S, row_bytes, alpha):
    plan = MemoSwapPlan()
    _check(lib().memo_swap_plan_make(int(S), int(row_bytes), float(alpha), ctypes.byref(plan)),
           "memo_swap_plan_make")
    return {name: int(getattr(plan, name)) for name, _ in MemoSwapPlan._fields_}


def _act_geometry(act):
    if act.dim() != 2 or not act.is_contiguous():
        raise ValueError("activation must be a contiguous [S, row] tensor")
    return act.shape[0], act.shape[1] * act.element_size()


def memo_swap_out(dev_act, alpha, host_pinned, copy_stream, wait_event=None, done_event=None):
    """Queues the D2H copy of the first floor(alpha*S) rows of dev_act [S,row] into the
    pinned host tensor on copy_stream."""
    S, row_bytes = _act_geometry(dev_act)
    if not host_pinned.is_pinned():
        raise ValueError("host store must be pinned memory")
    st = lib().memo_swap_out(dev_act.data_ptr(), S, row_bytes, float(alpha),
                             host_pinned.data_ptr(), host_pinned.numel() * host_pinned.element_size(),
                             _stream_ptr(copy_stream), _event_ptr(wait_event),
                             _event_ptr(done_event, _stream_obj(copy_stream)))
    _check(st, "memo_swap_out")


def memo_swap_in(dev_act, alpha, host_pinned, copy_stream, wait_event=None, done_event=None):
    """Queues the H2D copy of the swapped rows back into rows [0,k) of dev_act."""
    S, row_bytes = _act_geometry(dev_act)
    if not host_pinned.is_pinned():
        raise ValueError("host store must be pinned memory")
    st = lib().memo_swap_in(dev_act.data_ptr(), S, row_bytes, float(alpha),
                            host_pinned.data_ptr(), host_pinned.numel() * host_pinned.element_size(),
                            _stream_ptr(copy_stream), _event_ptr(wait_event),
                            _event_ptr(done_event, _stream_obj(copy_stream)))
    _check(st, "memo_swap_in")


def memo_solve_alpha(s_in, s_attn, s_oth, bandwidth, t_layer, n_layers, m_cpu):
    out = ctypes.c_double(0.0)
    _check(lib().memo_solve_alpha(float(s_in), float(s_attn), float(s_oth), float(bandwidth),
                                  float(t_layer), int(n_layers), float(m_cpu), ctypes.byref(out)),
           "memo_solve_alpha")
    return out.value


def _tensor_descs(tensors):
    arr = (MemoTensorDesc * len(tensors))()
    for i, (row_bytes, alpha) in enumerate(tensors):
        arr[i].row_bytes, arr[i].alpha = int(row_bytes), float(alpha)
    return arr


def memo_buffer_plan_make(S, tensors):
    """tensors: list of (row_bytes, alpha).  Returns (slots, dev_bytes, host_bytes)."""
    n = len(tensors)
    slots = (MemoTensorSlot * max(n, 1))()
    dev, host = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(lib().memo_buffer_plan_make(int(S), n, _tensor_descs(tensors) if n else None, slots,
                                       ctypes.byref(dev), ctypes.byref(host)),
           "memo_buffer_plan_make")
    out = [{name: int(getattr(slots[i], name)) for name, _ in MemoTensorSlot._fields_}
           for i in range(n)]
    return out, int(dev.value), int(host.value)


class MemoSched:
    """Handle of memo_sched_*: two rounding buffers over n layers.  Keeps the caller's
    buffers, host store and streams alive for as long as the handle lives."""

    def __init__(self, n_layers, S, tensors, dev_buffers, host_store, compute_stream,
                 offload_stream, prefetch_stream):
        b0, b1 = dev_buffers
        for b in (b0, b1):
            if b.dtype != torch.uint8 or not b.is_contiguous() or not b.is_cuda:
                raise ValueError("rounding buffers must be contiguous uint8 device tensors")
        _, dev_bytes, _ = memo_buffer_plan_make(S, tensors)
        if b0.numel() < dev_bytes or b1.numel() < dev_bytes:
            raise ValueError(f"rounding buffers must hold {dev_bytes} bytes each")
        if host_store is not None and not host_store.is_pinned():
            raise ValueError("host store must be pinned memory")
        self._keep = (b0, b1, host_store, compute_stream, offload_stream, prefetch_stream)
        self.n_layers = int(n_layers)
        handle = ctypes.c_void_p(None)
        cap = 0 if host_store is None else host_store.numel() * host_store.element_size()
        _check(lib().memo_sched_create(ctypes.byref(handle), self.n_layers, int(S), len(tensors),
                                       _tensor_descs(tensors), b0.data_ptr(), b1.data_ptr(),
                                       None if host_store is None else host_store.data_ptr(), cap,
                                       _stream_ptr(compute_stream), _stream_ptr(offload_stream),
                                       _stream_ptr(prefetch_stream)),
               "memo_sched_create")
        self._h = handle

    def forward_begin(self, layer):
        _check(lib().memo_sched_forward_begin(self._h, int(layer)), "memo_sched_forward_begin")

    def forward_end(self, layer):
        _check(lib().memo_sched_forward_end(self._h, int(layer)), "memo_sched_forward_end")

    def backward_begin(self, layer):
        _check(lib().memo_sched_backward_begin(self._h, int(layer)), "memo_sched_backward_begin")

    def backward_end(self, layer):
        _check(lib().memo_sched_backward_end(self._h, int(layer)), "memo_sched_backward_end")

    def buffer(self, layer):
        """The rounding buffer (uint8 tensor) of a layer."""
        return self._keep[int(layer) % 2]

    def buffer_ptr(self, layer):
        return lib().memo_sched_buffer(self._h, int(layer))

    def destroy(self):
        if self._h is not None and self._h.value:
            _check(lib().memo_sched_destroy(self._h), "memo_sched_destroy")
        self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def _row_range(rows, S):
    if rows is None:
        return 0, S
    b, e = rows
    return int(b), int(e)


def _bf16_2d(t, name):
    if t.dtype != torch.bfloat16 or t.dim() != 2 or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous 2-D bf16 tensor")


def memo_layernorm_rows(x, gamma, beta, eps, y=None, rows=None, stream=None):
    """y[r] = LayerNorm(x[r]) * gamma + beta for r in rows = (begin, end) (default: all rows).
    x, y: [S,h] bf16; other rows of y are left as they are."""
    _bf16_2d(x, "x")
    S, h = x.shape
    if y is None:
        y = torch.empty_like(x)
    _bf16_2d(y, "y")
    if y.shape != x.shape or gamma.shape != (h,) or beta.shape != (h,):
        raise ValueError("shape mismatch")
    if gamma.dtype != torch.bfloat16 or beta.dtype != torch.bfloat16:
        raise ValueError("gamma, beta must be bf16")
    b, e = _row_range(rows, S)
    _check(lib().memo_layernorm_rows(x.data_ptr(), gamma.data_ptr(), beta.data_ptr(), y.data_ptr(), S, h,
                                     float(eps), b, e, _stream_ptr(stream)), "memo_layernorm_rows")
    return y


def memo_linear_rows(a, w, bias=None, out=None, rows=None, stream=None):
    """out[r] = a[r] @ w.T + bias for r in rows = (begin, end) (default: all rows).
    a: [S,K] bf16, w: [N,K] bf16, bias: [N] bf16 or None, out: [S,N] bf16."""
    _bf16_2d(a, "a")
    _bf16_2d(w, "w")
    S, K = a.shape
    N = w.shape[0]
    if w.shape[1] != K:
        raise ValueError("w must be [N,K]")
    if out is None:
        out = torch.empty((S, N), dtype=torch.bfloat16, device=a.device)
    _bf16_2d(out, "out")
    if tuple(out.shape) != (S, N):
        raise ValueError("out must be [S,N]")
    if bias is not None and (bias.dtype != torch.bfloat16 or tuple(bias.shape) != (N,)):
        raise ValueError("bias must be bf16 [N]")
    b, e = _row_range(rows, S)
    _check(lib().memo_linear_rows(a.data_ptr(), w.data_ptr(), None if bias is None else bias.data_ptr(),
                                  out.data_ptr(), S, K, N, b, e, _stream_ptr(stream)), "memo_linear_rows")
    return out


def _requests(reqs):
    arr = (MemoDsaRequest * max(len(reqs), 1))()
    for i, (size, start, end) in enumerate(reqs):
        arr[i].size, arr[i].start, arr[i].end = int(size), int(start), int(end)
    return arr


def memo_trace_to_requests(events):
    """events: list of ("malloc" | "free", tensor_id (int), size).  Returns (requests, ids)."""
    n = len(events)
    flags = (ctypes.c_int32 * max(n, 1))(*[1 if e[0] == "malloc" else 0 for e in events])
    ids = (ctypes.c_int64 * max(n, 1))(*[int(e[1]) for e in events])
    sizes = (ctypes.c_int64 * max(n, 1))(*[int(e[2]) for e in events])
    req = (MemoDsaRequest * max(n, 1))()
    out_ids = (ctypes.c_int64 * max(n, 1))()
    cnt = ctypes.c_int32(0)
    _check(lib().memo_trace_to_requests(n, flags, ids, sizes, req, out_ids, ctypes.byref(cnt)),
           "memo_trace_to_requests")
    k = cnt.value
    return [(req[i].size, req[i].start, req[i].end) for i in range(k)], [out_ids[i] for i in range(k)]


def memo_dsa_plan(requests, align=1, node_limit=1_000_000):
    """requests: list of (size, start, end).  Returns (peak, addresses, proven_optimal)."""
    n = len(requests)
    addr = (ctypes.c_int64 * max(n, 1))()
    peak, opt = ctypes.c_int64(0), ctypes.c_int32(0)
    _check(lib().memo_dsa_plan(n, _requests(requests), int(align), int(node_limit), addr,
                               ctypes.byref(peak), ctypes.byref(opt)), "memo_dsa_plan")
    return peak.value, [addr[i] for i in range(n)], bool(opt.value)


def memo_dsa_plan_bilevel(layer_fwd, layer_bwd, fwd_ticks, bwd_ticks, outer, align=1, node_limit=1_000_000):
    """Two-level plan; returns a dict like the oracle's."""
    nl = len(fwd_ticks)
    if len(bwd_ticks) != nl:
        raise ValueError("fwd_ticks and bwd_ticks must have one entry per layer")
    arrs = {name: (ctypes.c_int64 * max(k, 1))() for name, k in
            (("fwd_offsets", len(layer_fwd)), ("bwd_offsets", len(layer_bwd)), ("fwd_base", nl),
             ("bwd_base", nl), ("outer_addr", len(outer)))}
    plan = MemoBilevelPlan()
    for name, arr in arrs.items():
        setattr(plan, name, ctypes.cast(arr, ctypes.POINTER(ctypes.c_int64)))
    ft = (ctypes.c_int32 * max(nl, 1))(*[int(t) for t in fwd_ticks])
    bt = (ctypes.c_int32 * max(nl, 1))(*[int(t) for t in bwd_ticks])
    _check(lib().memo_dsa_plan_bilevel(len(layer_fwd), _requests(layer_fwd), len(layer_bwd), _requests(layer_bwd),
                                       nl, ft, bt, len(outer), _requests(outer), int(align), int(node_limit),
                                       ctypes.byref(plan)), "memo_dsa_plan_bilevel")
    out = {name: [arr[i] for i in range(k)] for (name, arr), k in
           zip(arrs.items(), (len(layer_fwd), len(layer_bwd), nl, nl, len(outer)))}
    out.update(peak=plan.peak, fwd_peak=plan.fwd_peak, bwd_peak=plan.bwd_peak, optimal=bool(plan.optimal))
    return out
