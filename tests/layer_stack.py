"""A stack of stand-in transformer layers that drives the rounding-buffer schedule
(Section 4.1, Figure 5; Section 4.3.4).

Each layer is   q, k, v = a_q*x, a_k*rot(x, 37), a_v*rot(x, 74) ;  o = causal_attention(q, k, v) ;
x' = x + o,   with per-layer scalars a_* and rot = rotation of a token's feature vector (so that
q_i and k_i are not parallel, which would put all the softmax mass on the diagonal): the
token-wise producers stand in for LayerNorm + QKV projection (any row of q, k, v can be
regenerated from the same row of x), the attention is the real kernel.  Saved tensors of a layer, all [S, H*d] bf16 in one rounding buffer:
    0 input x (alpha 1)   1 o (alpha 1)   2..4 q, k, v (alpha)   5.. filler (alpha)
The filler tensors bring the layer to the 16 x (b*s*h) of Section 4.1 (norm outputs, MLP
activations, ...): they are copied like the rest but nothing reads them.  The logsumexp
([H,S] fp32 per layer, 1/256 of a layer's bytes at d = 128) stays on the device.

The caller-side arithmetic here (scalar multiplies, adds) is torch; attention and the
schedule are libmemo's.  There is no CPU fallback.
"""
import torch

from . import binding as mb

N_SAVED = 16          # tensors per layer, Section 4.1: 16*b*s*h elements in all


def layer_tensors(H, d, alpha, n_saved=N_SAVED):
    row = H * d * 2
    return [(row, 1.0), (row, 1.0)] + [(row, float(alpha))] * (n_saved - 2)


def layer_scalars(layer):
    """a_q, a_k, a_v of a layer: exact in bf16, different per layer."""
    return 1.0 + 0.125 * (layer % 3), 1.0 - 0.0625 * (layer % 5), 0.75 + 0.125 * (layer % 4)


SHIFTS = (0, 37, 74)   # feature rotation of q, k, v


def produce(x_rows, a, shift, out_rows):
    """out = a * rot(x, shift), row by row (token-wise)."""
    if shift == 0:
        torch.mul(x_rows, a, out=out_rows)
    else:
        torch.mul(x_rows[:, shift:], a, out=out_rows[:, :-shift])
        torch.mul(x_rows[:, :shift], a, out=out_rows[:, -shift:])


def accumulate(dx, g, a, shift):
    """dx += a * rot^-1(g): the backward of produce."""
    if shift == 0:
        dx.add_(g, alpha=a)
    else:
        dx[:, shift:].add_(g[:, :-shift], alpha=a)
        dx[:, :shift].add_(g[:, -shift:], alpha=a)


class LayerStack:
    """n layers over either two rounding buffers with swap (swap=True) or n resident
    buffers (swap=False; the reference the swapped run must reproduce bit for bit)."""

    def __init__(self, n_layers, S, H, d, alpha, scale, swap=True, n_saved=N_SAVED,
                 device="cuda:0", host=None, streams=None):
        """host: optional pinned uint8 tensor to use as the host store (allocated if None).
        streams: optional (compute, offload, prefetch) to reuse.  HIP multiplexes streams onto a
        few hardware queues (4 by default); two of the three landing on one queue would serialise
        copies and compute, so a caller that builds many stacks should create the streams once."""
        if d != 128:
            raise ValueError("the bf16 attention path needs d = 128")
        self.n, self.S, self.H, self.d, self.scale, self.swap = n_layers, S, H, d, scale, swap
        self.tensors = layer_tensors(H, d, alpha, n_saved)
        self.slots, self.dev_bytes, self.host_bytes = mb.memo_buffer_plan_make(S, self.tensors)
        dev = torch.device(device)
        if streams is None:
            streams = tuple(torch.cuda.Stream(device=dev) for _ in range(3))
        self.compute, self.offload, self.prefetch = streams
        n_buf = 2 if swap else n_layers
        self.buffers = [torch.empty(self.dev_bytes, dtype=torch.uint8, device=dev)
                        for _ in range(n_buf)]
        self.lse = [torch.empty((1, H, S), dtype=torch.float32, device=dev) for _ in range(n_layers)]
        self.sched = None
        self.host = None
        if swap:
            held = max(0, n_layers - 2) * self.host_bytes
            self.host = host if host is not None else \
                torch.empty(max(held, 256), dtype=torch.uint8, pin_memory=True)
            self.sched = mb.MemoSched(n_layers, S, self.tensors, self.buffers, self.host,
                                      self.compute, self.offload, self.prefetch)
        shape = (S, H * d)
        self.x_io = [torch.empty(shape, dtype=torch.bfloat16, device=dev) for _ in range(2)]
        self.grads = [torch.empty((1, S, H, d), dtype=torch.bfloat16, device=dev) for _ in range(3)]
        self.dx = torch.empty(shape, dtype=torch.bfloat16, device=dev)
        probe = self.grads[0]
        self.workspace = torch.empty(max(256, mb.memo_attn_bwd_workspace_bytes(probe, scale)),
                                     dtype=torch.uint8, device=dev)

    # ---- views into a layer's buffer
    def buffer(self, layer):
        return self.buffers[layer % 2] if self.swap else self.buffers[layer]

    def view(self, layer, t):
        s = self.slots[t]
        row = self.tensors[t][0]
        b = self.buffer(layer)[s["dev_offset"]: s["dev_offset"] + self.S * row]
        return b.view(torch.bfloat16).view(self.S, row // 2)

    def _heads(self, t2d):
        return t2d.view(1, self.S, self.H, self.d)

    # ---- one training iteration
    def forward(self, x0):
        """x0: [S, H*d] bf16 on the device.  Returns the output of the last layer; all work
        is queued on the stack's compute stream, behind what the current stream holds."""
        self.compute.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(self.compute):
            cur = self.x_io[0]
            cur.copy_(x0)
            for i in range(self.n):
                if self.sched:
                    self.sched.forward_begin(i)
                x, o = self.view(i, 0), self.view(i, 1)
                x.copy_(cur)
                for t, a, sh in zip((2, 3, 4), layer_scalars(i), SHIFTS):
                    produce(x, a, sh, self.view(i, t))
                mb.memo_attn_fwd(self._heads(self.view(i, 2)), self._heads(self.view(i, 3)),
                                 self._heads(self.view(i, 4)), self.scale, o=self._heads(o),
                                 lse=self.lse[i], stream=self.compute)
                nxt = self.x_io[(i + 1) % 2]
                torch.add(x, o, out=nxt)
                cur = nxt
                if self.sched:
                    self.sched.forward_end(i)
            return cur

    def backward(self, d_out, on_layer=None):
        """d_out: dL/d(output of the last layer).  Returns dL/dx0 (valid once the compute
        stream has finished).  on_layer(i) is called on the compute stream right before
        layer i's backward kernels, after the dropped rows were regenerated."""
        self.compute.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(self.compute):
            dx = self.dx
            dx.copy_(d_out)
            dq, dk, dv = self.grads
            for i in range(self.n - 1, -1, -1):
                if self.sched:
                    self.sched.backward_begin(i)
                x, o = self.view(i, 0), self.view(i, 1)
                scal = layer_scalars(i)
                if self.sched and i < self.n - 2:
                    for t, a, sh in zip((2, 3, 4), scal, SHIFTS):
                        k = self.slots[t]["k_swapped"]
                        if k < self.S:
                            produce(x[k:], a, sh, self.view(i, t)[k:])
                if on_layer is not None:
                    on_layer(i)
                mb.memo_attn_bwd(self._heads(self.view(i, 2)), self._heads(self.view(i, 3)),
                                 self._heads(self.view(i, 4)), self._heads(o), self.lse[i],
                                 self._heads(dx), self.scale, dq=dq, dk=dk, dv=dv,
                                 workspace=self.workspace, stream=self.compute)
                for g, a, sh in zip((dq, dk, dv), scal, SHIFTS):
                    accumulate(dx, g.view(self.S, self.H * self.d), a, sh)
                if self.sched:
                    self.sched.backward_end(i)
            return dx

    def close(self):
        torch.cuda.synchronize()
        if self.sched:
            self.sched.destroy()
            self.sched = None
