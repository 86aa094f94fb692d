"""Test and benchmark harness (not part of the library): a stack of stand-in transformer layers
that drives the rounding-buffer schedule (Section 4.1, Figure 5; Section 4.3.4) together with the
token-wise recomputation kernels.

Each layer is   norm = LayerNorm(x) ;  q, k, v = norm W_q^T + b_q, ... ;  o = causal_attention(q, k, v) ;
x' = x + o,   with per-layer gamma, beta, W_* [h, h], b_* drawn from a seed (h = H*d).  LayerNorm,
the projections, the attention and the schedule are libmemo's (memo_layernorm_rows,
memo_linear_rows, memo_attn_fwd/bwd, memo_sched_*); the residual add and the stand-in gradient
propagation below are torch arithmetic of this harness.  Saved tensors of a layer, all [S,h] bf16
in one rounding buffer:
    0 input x (alpha 1)   1 o (alpha 1)   2 norm (alpha)   3..5 q, k, v (alpha)   6.. filler (alpha)
which with 10 fillers is the 16 x (b*s*h) of Section 4.1 (MLP activations and the like: they are
copied like the rest but nothing reads them).  The logsumexp ([H,S] fp32 per layer, 1/256 of a
layer's bytes at d = 128) stays on the device.

Backward of a layer: rows [0,k) of norm, q, k, v come back from the host with the prefetch, rows
[k,S) are rebuilt from the stored layer input by the same kernels on that row range (the paper's
token-wise recomputation), then memo_attn_bwd runs.  The gradient that is passed down is a stand-in:
dx' = dx + dq W_q + dk W_k + dv W_v (the projections' input gradient, LayerNorm treated as
identity); the weight gradients and the LayerNorm Jacobian are outside this path.  What the tests
need from it is that every regenerated row feeds the result.  There is no CPU fallback.
"""
import torch

from paper_2407_12117_amd import binding as mb

N_SAVED = 16          # saved [S,h] tensors per layer, Section 4.1: 16*b*s*h elements in all
EPS = 1e-5


def layer_tensors(H, d, alpha, n_saved=N_SAVED):
    """(row_bytes, alpha) of a layer's saved tensors."""
    if n_saved < 6:
        raise ValueError("a layer saves at least x, o, norm, q, k, v")
    row = H * d * 2
    return [(row, 1.0), (row, 1.0)] + [(row, float(alpha))] * (n_saved - 2)


def layer_params(layer, h, device):
    """gamma, beta [h] and (W [h,h], b [h]) for q, k, v of a layer, bf16, from a per-layer seed."""
    g = torch.Generator().manual_seed(9000 + layer)
    gamma = (1.0 + 0.1 * torch.randn(h, generator=g)).to(torch.bfloat16).to(device)
    beta = (0.1 * torch.randn(h, generator=g)).to(torch.bfloat16).to(device)
    proj = [((torch.randn((h, h), generator=g) / h ** 0.5).to(torch.bfloat16).to(device),
             (0.1 * torch.randn(h, generator=g)).to(torch.bfloat16).to(device)) for _ in range(3)]
    return gamma, beta, proj


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
        if (H * d) % 512:
            raise ValueError("memo_layernorm_rows needs a hidden size that is a multiple of 512 (H % 4 == 0)")
        self.n, self.S, self.H, self.d, self.scale, self.swap = n_layers, S, H, d, scale, swap
        self.h = H * d
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
        self.params = [layer_params(i, self.h, dev) for i in range(n_layers)]
        self.sched = None
        self.host = None
        if swap:
            held = max(0, n_layers - 2) * self.host_bytes
            self.host = host if host is not None else \
                torch.empty(max(held, 256), dtype=torch.uint8, pin_memory=True)
            self.sched = mb.MemoSched(n_layers, S, self.tensors, self.buffers, self.host,
                                      self.compute, self.offload, self.prefetch)
        shape = (S, self.h)
        self.x_io = [torch.empty(shape, dtype=torch.bfloat16, device=dev) for _ in range(2)]
        self.grads = [torch.empty((1, S, H, d), dtype=torch.bfloat16, device=dev) for _ in range(3)]
        self.dx = torch.empty(shape, dtype=torch.bfloat16, device=dev)
        self.workspace = torch.empty(max(256, mb.memo_attn_bwd_workspace_bytes(self.grads[0], scale)),
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
                x, o, norm = (self.view(i, t) for t in range(3))
                gamma, beta, proj = self.params[i]
                x.copy_(cur)
                mb.memo_layernorm_rows(x, gamma, beta, EPS, y=norm, stream=self.compute)
                for t, (w, b) in zip((3, 4, 5), proj):
                    mb.memo_linear_rows(norm, w, b, out=self.view(i, t), stream=self.compute)
                mb.memo_attn_fwd(self._heads(self.view(i, 3)), self._heads(self.view(i, 4)),
                                 self._heads(self.view(i, 5)), self.scale, o=self._heads(o),
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
                x, o, norm = (self.view(i, t) for t in range(3))
                gamma, beta, proj = self.params[i]
                if self.sched and i < self.n - 2:
                    # token-wise recomputation: rows [k,S) of norm from x, then of q, k, v from norm
                    mb.memo_layernorm_rows(x, gamma, beta, EPS, y=norm, rows=(self.slots[2]["k_swapped"], self.S),
                                           stream=self.compute)
                    for t, (w, b) in zip((3, 4, 5), proj):
                        mb.memo_linear_rows(norm, w, b, out=self.view(i, t),
                                            rows=(self.slots[t]["k_swapped"], self.S), stream=self.compute)
                if on_layer is not None:
                    on_layer(i)
                mb.memo_attn_bwd(self._heads(self.view(i, 3)), self._heads(self.view(i, 4)),
                                 self._heads(self.view(i, 5)), self._heads(o), self.lse[i],
                                 self._heads(dx), self.scale, dq=dq, dk=dk, dv=dv,
                                 workspace=self.workspace, stream=self.compute)
                for g, (w, _) in zip((dq, dk, dv), proj):
                    dx.addmm_(g.view(self.S, self.h), w)
                if self.sched:
                    self.sched.backward_end(i)
            return dx

    def close(self):
        torch.cuda.synchronize()
        if self.sched:
            self.sched.destroy()
            self.sched = None
