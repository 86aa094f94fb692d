/*
 * memo.h -- C ABI of libmemo, the MI355X (gfx950) hot path of Memo
 * (arXiv 2407.12117): exact causal attention forward/backward and the
 * token-wise swap of saved activations.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers unless the name says "host".
 *     The caller owns every buffer; the library never frees or keeps a pointer
 *     after the call returns, but work queued on a stream may still read or
 *     write the buffers until that stream (or the done event) completes.
 *   - Streams and events are hipStream_t / hipEvent_t passed as void*
 *     (NULL stream = the default stream).
 *   - Argument errors are found on the host before anything is queued and are
 *     reported through the return value; nothing is thrown, nothing is printed.
 *     A failing HIP call gives MEMO_ERR_DEVICE.  Faults inside a kernel surface
 *     at the caller's next synchronisation, as with any HIP launch.
 *   - Calls are asynchronous with respect to the host.
 */
#ifndef MEMO_H
#define MEMO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MEMO_OK = 0,
    MEMO_ERR_INVALID_ARG = 1,   /* null pointer, bad size, alpha outside [0,1], ... */
    MEMO_ERR_UNSUPPORTED = 2,   /* head dim / dtype / stride combination not built */
    MEMO_ERR_HOST_CAPACITY = 3, /* host store smaller than the swapped bytes: the paper's
                                   host out-of-memory case (Section 4.1, second constraint) */
    MEMO_ERR_WORKSPACE = 4,     /* workspace missing or smaller than the query says */
    MEMO_ERR_DEVICE = 5         /* a HIP runtime call failed */
} memo_status;

typedef enum { MEMO_F32 = 0, MEMO_BF16 = 1 } memo_dtype;

/*
 * Problem statement of one attention call (Section 2.1.3: Q, K, V of shape
 * (b, s, h), O = softmax(Q K^T / sqrt(d)) V under the decoder's causal mask).
 * h is split into H heads of width d; element (b, s, h, c) of every tensor
 * lives at  b*stride_b + s*stride_s + h*stride_h + c  (strides in elements,
 * c contiguous).  The token-major layout [B,S,H,d] is stride_b = S*H*d,
 * stride_s = H*d, stride_h = d.  All of q, k, v, o, d_o, dq, dk, dv share
 * the strides.  lse and the like are [B,H,S] contiguous fp32.
 * Supported: MEMO_BF16 with d = 128 (fp32 accumulation, MFMA path);
 *            MEMO_F32 with d in {64, 128} (fp32 throughout).
 * S may be any positive length (ragged last tile is handled); causal must be 1.
 * Rows must be 16-byte aligned: base pointers 16-byte aligned and strides a
 * multiple of 8 (bf16) or 4 (fp32) elements.  MEMO_BF16: stride_s <= 2^24 elements and
 * about S * H * B < 2^40 (one workgroup per pair of 256-row tiles, in chunks of 32 pairs per head
 * rounded up to 8 chunks, must fit a 2^31 grid); MEMO_ERR_UNSUPPORTED otherwise.
 * Non-finite inputs: the kernels keep IEEE semantics, so a NaN or an infinity in q, k, v or d_o
 * reaches every output element that depends on it: a NaN in key row j makes o, lse, dq of all
 * query rows i >= j non-finite and, through them, all of dk and dv of that head.  It may also
 * reach rows that only share a tile with row j (masked probabilities are zeros that still meet
 * the NaN inside a contraction): rows within the same 256-row block.  Rows outside that block
 * that do not depend on the value, other heads and other batch entries are bit-identical to a
 * run without it.
 */
typedef struct {
    int32_t B, H, d;
    int64_t S;
    int32_t dtype;              /* memo_dtype */
    float scale;                /* the 1/sqrt(d) of the formula, passed explicitly */
    int64_t stride_b, stride_s, stride_h;
    int32_t causal;             /* must be 1: mask is inclusive, key j visible to query i iff j <= i */
    uint32_t flags;             /* bit 0: bit-reproducible dq requested (always the case: the backward
                                   uses no atomics, so the bit changes nothing); other bits must be 0 */
} memo_attn_desc;

/*
 * Forward (Section 2.1.3, FlashAttention: tiled, keeps only per-row state).
 *   o   [same layout as q]  = softmax(scale * q k^T, causal) v
 *   lse [B,H,S] fp32        = natural-log sum_j exp(scale * q_i . k_j), j <= i
 * Queued on `stream`.  Returns MEMO_OK or an error; on error nothing is queued.
 */
memo_status memo_attn_fwd(const memo_attn_desc *desc, const void *q, const void *k, const void *v,
                          void *o, float *lse, void *stream);

/*
 * Backward (Section 2.1.3: the intermediates are re-formed tile by tile).
 * Given d_o = dL/dO, writes dq, dk, dv (same layout and dtype as q).
 * Needs o and lse from the forward.  `workspace` is device memory of at least
 * memo_attn_bwd_workspace_bytes(desc) bytes, 256-byte aligned, owned by the
 * caller, contents undefined on entry and exit.  Deterministic: no atomics.
 */
size_t memo_attn_bwd_workspace_bytes(const memo_attn_desc *desc);
memo_status memo_attn_bwd(const memo_attn_desc *desc, const void *q, const void *k, const void *v,
                          const void *o, const float *lse, const void *d_o,
                          void *dq, void *dk, void *dv,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * Same as memo_attn_bwd, and additionally records caller-owned events on `stream` between the
 * stages of the backward, so that a profiler or benchmark can time each kernel where it runs:
 *   stage_events[0] before the first kernel,
 *   stage_events[1] after the D_i = sum_c dO_ic O_ic preprocess,
 *   stage_events[2] after the dK/dV kernel,
 *   stage_events[3] after the dQ kernel.
 * stage_events is a host array of 4 hipEvent_t (created with timing enabled), or NULL.
 */
memo_status memo_attn_bwd_staged(const memo_attn_desc *desc, const void *q, const void *k,
                                 const void *v, const void *o, const float *lse, const void *d_o,
                                 void *dq, void *dk, void *dv,
                                 void *workspace, size_t workspace_bytes, void *stream,
                                 void *const *stage_events);

/*
 * memo_attn_bwd for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and errors as memo_attn_bwd without the workspace: the D_i buffer lives in a static
 * device array inside the library (16 MiB per GPU the library runs on, held until the process
 * ends), so the call allocates nothing, on the device or through any library.
 * Limit: B * H * S <= MEMO_ATTN_BWD_STATIC_MAX_ROWS, else MEMO_ERR_WORKSPACE and nothing is queued.
 * Every call on one GPU uses that GPU's one array: calls that may overlap in time on the same GPU
 * (different streams, different host threads) race and must be serialised by the caller.  The
 * array keeps the previous call's contents; the backward overwrites what it reads, so no clearing
 * is needed.  The device must be the current one, as for every other entry point.
 */
#define MEMO_ATTN_BWD_STATIC_MAX_ROWS ((size_t)4 << 20)
memo_status memo_attn_bwd_static(const memo_attn_desc *desc, const void *q, const void *k,
                                 const void *v, const void *o, const float *lse, const void *d_o,
                                 void *dq, void *dk, void *dv, void *stream);

/*
 * Token split (Section 4.1, "at the token granularity ... we offload a fraction alpha
 * to CPU, while the remaining part is discarded").  k = floor(alpha * S) evaluated in
 * IEEE double; tokens [0,k) are swapped, tokens [k,S) are recomputed by the caller
 * before the layer's backward.  Returns k, or -1 if S < 0 or alpha is not in [0,1].
 */
int64_t memo_split_tokens(int64_t S, double alpha);

typedef struct {
    int64_t S, row_bytes;
    int64_t k_swapped;              /* tokens offloaded */
    int64_t n_recompute;            /* tokens dropped: S - k_swapped */
    int64_t bytes_swapped;          /* k_swapped * row_bytes */
    int64_t bytes_dropped;          /* n_recompute * row_bytes */
    int64_t recompute_byte_offset;  /* where the first dropped row starts in the activation */
} memo_swap_plan;

/* Fills *out for an activation of S token rows of row_bytes bytes each. */
memo_status memo_swap_plan_make(int64_t S, int64_t row_bytes, double alpha, memo_swap_plan *out);

/*
 * Swap-out (Section 4.1: after a layer's computation its saved activations are offloaded
 * on a separate stream, concurrently with the next computation; an event tells when the
 * device buffer may be rewritten).
 *   dev_act      device, [S, row_bytes] bytes, rows contiguous; only rows [0,k) are read
 *   host_pinned  HOST pinned memory of host_capacity_bytes; receives k*row_bytes bytes
 *   copy_stream  stream the copy is queued on (the offload stream)
 *   wait_event   nullable; the copy stream waits for it first (producer finished writing)
 *   done_event   nullable; recorded on copy_stream after the copy
 * alpha = 0 queues no copy (events are still honoured).  MEMO_ERR_HOST_CAPACITY if the
 * host store is too small; then nothing is queued.
 */
memo_status memo_swap_out(const void *dev_act, int64_t S, int64_t row_bytes, double alpha,
                          void *host_pinned, size_t host_capacity_bytes,
                          void *copy_stream, void *wait_event, void *done_event);

/*
 * Swap-in (Section 4.1 / 4.3.4: prefetch on a third stream before the layer's backward).
 * Mirror of memo_swap_out: rows [0,k) of dev_act are written from the host store, rows
 * [k,S) are not touched.
 */
memo_status memo_swap_in(void *dev_act, int64_t S, int64_t row_bytes, double alpha,
                         const void *host_pinned, size_t host_capacity_bytes,
                         void *copy_stream, void *wait_event, void *done_event);

/*
 * Largest alpha in [0,1] with (Section 4.1, the problem "max alpha"):
 *   (s_in + s_attn + alpha*s_oth) / bandwidth <= t_layer
 *   (n_layers - 2) * (s_in + s_attn + alpha*s_oth) <= m_cpu
 * Sizes in bytes, bandwidth in bytes/s, t_layer in s.  Host-side arithmetic only.
 * Returns MEMO_ERR_HOST_CAPACITY if alpha = 0 already breaks the memory constraint,
 * MEMO_ERR_UNSUPPORTED if alpha = 0 breaks the time constraint (the copy of the two
 * whole tensors cannot be hidden), MEMO_ERR_INVALID_ARG on non-positive inputs.
 */
memo_status memo_solve_alpha(double s_in, double s_attn, double s_oth, double bandwidth,
                             double t_layer, int32_t n_layers, double m_cpu, double *alpha_out);

/*
 * Two rounding buffers over n layers (Section 4.1, Figure 5; Section 4.3.4, the
 * three-stream schedule).
 *
 * A layer's saved tensors live together in one of two device buffers (layer i uses
 * buffer i % 2).  Each tensor t is [S, row_bytes[t]] bytes with its own fraction
 * alpha[t] (1 for the layer input and the attention output, the solved alpha for the
 * rest).  memo_buffer_plan_make lays them out: every tensor whole in the device buffer
 * at dev_offset, the swapped prefixes back to back in a per-layer host slot at
 * host_offset, both rounded up to 256 bytes (the paper does not specify a packing).
 */
typedef struct {
    int64_t row_bytes;          /* > 0 */
    double alpha;               /* finite, in [0,1] */
} memo_tensor_desc;

typedef struct {
    int64_t dev_offset;         /* byte offset of the tensor in a rounding buffer */
    int64_t host_offset;        /* byte offset of its swapped prefix in a layer's host slot */
    int64_t k_swapped;          /* rows [0,k) swapped, rows [k,S) to regenerate */
    size_t bytes_swapped;       /* k_swapped * row_bytes */
} memo_tensor_slot;

/*
 * Host-side arithmetic only.  slots_out has room for n_tensors entries; dev_bytes_out /
 * host_bytes_out receive the size of one rounding buffer / of one layer's host slot.
 * MEMO_ERR_INVALID_ARG on null pointers, n_tensors < 1, S < 1 or a bad descriptor.
 */
memo_status memo_buffer_plan_make(int64_t S, int32_t n_tensors, const memo_tensor_desc *tensors,
                                  memo_tensor_slot *slots_out, size_t *dev_bytes_out,
                                  size_t *host_bytes_out);

/*
 * The schedule itself.  A memo_sched owns 4*n_layers HIP events and nothing else; the
 * caller owns the two device buffers (dev_bytes each), the pinned host store and the
 * three streams (compute, offload, prefetch; all three must differ for the copies to
 * overlap, but any may coincide).  The host store must hold (n_layers - 2) layer
 * slots: MEMO_ERR_HOST_CAPACITY otherwise (the second constraint of the alpha problem).
 *
 * Per iteration the caller brackets each layer's work on the compute stream:
 *   for i = 0 .. n-1:   memo_sched_forward_begin(i);  <forward of layer i writes buffer i%2>
 *                       memo_sched_forward_end(i);
 *   for i = n-1 .. 0:   memo_sched_backward_begin(i); <regenerate rows [k,S); backward>
 *                       memo_sched_backward_end(i);
 * forward_begin(i)  makes the compute stream wait until layer i-2's offload has left
 *                   buffer i%2;
 * forward_end(i)    queues the offload of layer i's prefixes on the offload stream behind
 *                   the forward (not for the last two layers, which turn round at once);
 * backward_begin(i) makes the compute stream wait for the prefetch of layer i;
 * backward_end(i)   queues the prefetch of layer i-2 into buffer i%2 on the prefetch
 *                   stream behind this backward, so it runs under backward(i-1).
 * Calls out of this order give MEMO_ERR_INVALID_ARG and queue nothing.  Nothing blocks
 * the host.  memo_sched_buffer(i) is the device buffer of layer i.
 * MEMO_ERR_DEVICE from one of the four calls means a HIP call failed part-way: some of that
 * call's waits and copies may already be queued and its event may not be recorded.  The handle
 * is then dead (every later call but memo_sched_destroy returns MEMO_ERR_DEVICE): the caller
 * synchronises its three streams, treats both buffers and the host store as undefined for this
 * iteration, destroys the handle and starts the iteration again with a new one.
 */
typedef struct memo_sched memo_sched;

memo_status memo_sched_create(memo_sched **out, int32_t n_layers, int64_t S, int32_t n_tensors,
                              const memo_tensor_desc *tensors, void *dev_buffer0,
                              void *dev_buffer1, void *host_store, size_t host_capacity_bytes,
                              void *compute_stream, void *offload_stream, void *prefetch_stream);
memo_status memo_sched_forward_begin(memo_sched *s, int32_t layer);
memo_status memo_sched_forward_end(memo_sched *s, int32_t layer);
memo_status memo_sched_backward_begin(memo_sched *s, int32_t layer);
memo_status memo_sched_backward_end(memo_sched *s, int32_t layer);
void *memo_sched_buffer(const memo_sched *s, int32_t layer);
/* Waits for nothing: the caller synchronises its streams first.  NULL is accepted. */
memo_status memo_sched_destroy(memo_sched *s);

/*
 * Token-wise recomputation of the tensors that follow the stored layer input (Section 4.1:
 * the layer input is kept whole so that "input_norm", "q", "k", "v" can be rebuilt; the
 * swapped rows [0,k) come back from the host, the dropped rows [k,S) are recomputed).
 * Both operations work on a row range of token-major bf16 tensors and each output row
 * depends on its own input row only, computed in a fixed order: a row recomputed in any
 * range is bit-identical to the same row of a pass over all rows.
 *
 * memo_layernorm_rows:  y[r,:] = (x[r,:] - mean_r) / sqrt(var_r + eps) * gamma + beta for
 *   row_begin <= r < row_end; x, y device [S,h] bf16 contiguous, gamma, beta device [h] bf16;
 *   statistics in fp32 (biased variance).  h a multiple of 512, at most 8192.
 * memo_linear_rows:     out[r,:] = a[r,:] * w^T + bias for the same kind of range; a device
 *   [S,K] bf16, w device [N,K] bf16 (K contiguous), bias device [N] bf16 or NULL, out device
 *   [S,N] bf16; fp32 accumulation on the matrix cores.  K and N multiples of 128.
 * All pointers 16-byte aligned.  An empty range queues nothing.  Rows outside the range are
 * neither read nor written.  MEMO_ERR_INVALID_ARG / MEMO_ERR_UNSUPPORTED before any launch.
 */
memo_status memo_layernorm_rows(const void *x, const void *gamma, const void *beta, void *y,
                                int64_t S, int32_t h, float eps, int64_t row_begin,
                                int64_t row_end, void *hip_stream);
memo_status memo_linear_rows(const void *a, const void *w, const void *bias, void *out, int64_t S,
                             int32_t K, int32_t N, int64_t row_begin, int64_t row_end,
                             void *hip_stream);

/*
 * Offline storage allocation for the transient tensors and its two-level use over identical
 * layers (Section 4.2).  Host-side arithmetic only; nothing touches a GPU.
 *
 * A request is a tensor of `size` bytes alive during the ticks [start, end) of a profiled
 * memory request sequence.  memo_dsa_plan assigns every request an address such that requests
 * with overlapping lifespans do not share bytes and the peak  max(addr + size)  is minimal:
 * the optimum of the paper's mixed-integer programme, found by an exact search that is cut
 * off after `node_limit` search nodes (then the best plan found so far is returned and
 * *optimal_out is 0; it is 1 when the plan is proven optimal).  Sizes are rounded up to
 * `align` (a power of two) first; addresses are multiples of it.  addr_out has n entries.
 *
 * memo_trace_to_requests turns a sequence of "malloc tensor_id size" / "free tensor_id size"
 * events (is_malloc[t] != 0 for a malloc) into requests in order of allocation: start = index
 * of the malloc, end = index of the free (the sequence length if never freed).  req_out and
 * id_out need room for one entry per malloc.  A double malloc, a free without a live
 * allocation or with another size give MEMO_ERR_INVALID_ARG.
 *
 * memo_dsa_plan_bilevel: level 1 plans one layer's forward and one layer's backward request
 * sequence (every layer reuses the offsets); level 2 plans the rest of the model (`outer`)
 * together with one pseudo request per layer pass, of the level-1 peak, alive during the tick
 * [fwd_ticks[l], fwd_ticks[l] + 1) resp. [bwd_ticks[l], bwd_ticks[l] + 1) of the outer clock.
 * The address of tensor t of layer l's forward pass is fwd_base[l] + fwd_offsets[t].
 * The caller provides the arrays of memo_bilevel_plan (n_fwd, n_bwd, n_layers, n_layers,
 * n_outer entries); peaks and `optimal` are filled in.
 */
typedef struct {
    int64_t size;
    int32_t start, end;
} memo_dsa_request;

typedef struct {
    int64_t peak;               /* bytes needed for all transient tensors of the model */
    int64_t fwd_peak, bwd_peak; /* level 1: bytes of one layer's forward / backward pass */
    int64_t *fwd_offsets, *bwd_offsets, *fwd_base, *bwd_base, *outer_addr;
    int32_t optimal;            /* 1 if all three searches proved their optimum */
} memo_bilevel_plan;

memo_status memo_trace_to_requests(int32_t n_events, const int32_t *is_malloc,
                                   const int64_t *tensor_id, const int64_t *size,
                                   memo_dsa_request *req_out, int64_t *id_out,
                                   int32_t *n_requests_out);
memo_status memo_dsa_plan(int32_t n, const memo_dsa_request *requests, int64_t align,
                          int64_t node_limit, int64_t *addr_out, int64_t *peak_out,
                          int32_t *optimal_out);
memo_status memo_dsa_plan_bilevel(int32_t n_fwd, const memo_dsa_request *layer_fwd, int32_t n_bwd,
                                  const memo_dsa_request *layer_bwd, int32_t n_layers,
                                  const int32_t *fwd_ticks, const int32_t *bwd_ticks,
                                  int32_t n_outer, const memo_dsa_request *outer, int64_t align,
                                  int64_t node_limit, memo_bilevel_plan *out);

/* Pinned host memory helpers (hipHostMalloc / hipHostFree). */
memo_status memo_host_alloc(void **host_ptr, size_t bytes);
memo_status memo_host_free(void *host_ptr);

const char *memo_status_str(memo_status s);

#ifdef __cplusplus
}
#endif
#endif /* MEMO_H */
