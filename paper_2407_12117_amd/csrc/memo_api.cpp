// C-ABI front end of libmemo: argument checking, the token-split bookkeeping, the swap
// copies on the caller's side streams, and dispatch to the gfx950 kernels.
// The contract of every entry point is in include/memo.h.
#include "../../include/memo.h"
#include "memo_kernels.h"

#include <cmath>
#include <cstring>

namespace {

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Checks the problem statement; fills the kernel-side argument block.
memo_status check_desc(const memo_attn_desc *d, memo::AttnArgs *out)
{
    if (!d) return MEMO_ERR_INVALID_ARG;
    if (d->B <= 0 || d->H <= 0 || d->S <= 0 || d->d <= 0) return MEMO_ERR_INVALID_ARG;
    if (d->B > 65535 || d->H > 65535) return MEMO_ERR_INVALID_ARG;
    if (!(d->scale > 0.f) || !std::isfinite(d->scale)) return MEMO_ERR_INVALID_ARG;
    // flags bit 0 asks for bit-reproducible gradients: every path here is, so it is accepted and changes nothing
    if (d->causal != 1 || (d->flags & ~1u) != 0) return MEMO_ERR_UNSUPPORTED;
    if (d->dtype != MEMO_F32 && d->dtype != MEMO_BF16) return MEMO_ERR_UNSUPPORTED;
    if (d->dtype == MEMO_BF16 && d->d != 128) return MEMO_ERR_UNSUPPORTED;
    if (d->dtype == MEMO_F32 && d->d != 64 && d->d != 128) return MEMO_ERR_UNSUPPORTED;
    const int64_t vec = d->dtype == MEMO_BF16 ? 8 : 4;   // elements per 16 bytes
    if (d->stride_h < d->d || d->stride_s < d->d || d->stride_b < d->d) return MEMO_ERR_INVALID_ARG;
    if (d->stride_b % vec || d->stride_s % vec || d->stride_h % vec) return MEMO_ERR_UNSUPPORTED;
    // the tile index arithmetic is 64-bit; the row count per launch must fit the grid
    if (d->S > ((int64_t)1 << 31) - 1024) return MEMO_ERR_UNSUPPORTED;
    // every bf16 kernel launches one workgroup per pair of 256-row tiles, in chunks of 32 pairs per head
    // rounded up to a multiple of 8 chunks
    if (d->dtype == MEMO_BF16) {
        const int64_t hb = (int64_t)d->H * d->B;
        if (((((d->S + 255) / 256 + 1) / 2 + 31) / 32 * hb + 7) / 8 * 256 > 0x7fffffffLL) return MEMO_ERR_UNSUPPORTED;
    }
    // the bf16 tile fills address 64 rows with 32-bit per-lane byte offsets
    if (d->dtype == MEMO_BF16 && d->stride_s > ((int64_t)1 << 24)) return MEMO_ERR_UNSUPPORTED;
    std::memset(out, 0, sizeof(*out));
    out->B = d->B;
    out->H = d->H;
    out->d = d->d;
    out->S = d->S;
    out->scale = d->scale;
    out->sb = d->stride_b;
    out->ss = d->stride_s;
    out->sh = d->stride_h;
    return MEMO_OK;
}

inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

memo_status check_swap(const void *dev, int64_t S, int64_t row_bytes, double alpha,
                       const void *host, size_t cap, memo_swap_plan *plan)
{
    memo_status st = memo_swap_plan_make(S, row_bytes, alpha, plan);
    if (st != MEMO_OK) return st;
    if (!dev || !host) return MEMO_ERR_INVALID_ARG;
    if ((uint64_t)plan->bytes_swapped > (uint64_t)cap) return MEMO_ERR_HOST_CAPACITY;
    return MEMO_OK;
}

}  // namespace

extern "C" {

const char *memo_status_str(memo_status s)
{
    switch (s) {
    case MEMO_OK: return "ok";
    case MEMO_ERR_INVALID_ARG: return "invalid argument";
    case MEMO_ERR_UNSUPPORTED: return "unsupported shape, dtype or layout";
    case MEMO_ERR_HOST_CAPACITY: return "host store too small for the swapped tokens";
    case MEMO_ERR_WORKSPACE: return "workspace missing or too small";
    case MEMO_ERR_DEVICE: return "HIP runtime error";
    }
    return "unknown status";
}

memo_status memo_attn_fwd(const memo_attn_desc *desc, const void *q, const void *k, const void *v,
                          void *o, float *lse, void *stream)
{
    memo::AttnArgs a;
    memo_status st = check_desc(desc, &a);
    if (st != MEMO_OK) return st;
    if (!q || !k || !v || !o || !lse) return MEMO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return MEMO_ERR_UNSUPPORTED;
    a.q = q;
    a.k = k;
    a.v = v;
    a.o_out = o;
    a.lse = lse;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    hipError_t e = desc->dtype == MEMO_BF16 ? memo::launch_attn_fwd_bf16(a, hs)
                                            : memo::launch_attn_fwd_f32(a, hs);
    return e == hipSuccess ? MEMO_OK : MEMO_ERR_DEVICE;
}

size_t memo_attn_bwd_workspace_bytes(const memo_attn_desc *desc)
{
    memo::AttnArgs a;
    if (check_desc(desc, &a) != MEMO_OK) return 0;
    // D_i = sum_c dO_ic O_ic, one fp32 per (b, h, i)
    return round_up((size_t)desc->B * desc->H * (size_t)desc->S * sizeof(float), 256);
}

memo_status memo_attn_bwd(const memo_attn_desc *desc, const void *q, const void *k, const void *v,
                          const void *o, const float *lse, const void *d_o,
                          void *dq, void *dk, void *dv,
                          void *workspace, size_t workspace_bytes, void *stream)
{
    return memo_attn_bwd_staged(desc, q, k, v, o, lse, d_o, dq, dk, dv, workspace, workspace_bytes,
                                stream, nullptr);
}

memo_status memo_attn_bwd_staged(const memo_attn_desc *desc, const void *q, const void *k,
                                 const void *v, const void *o, const float *lse, const void *d_o,
                                 void *dq, void *dk, void *dv,
                                 void *workspace, size_t workspace_bytes, void *stream,
                                 void *const *stage_events)
{
    memo::AttnArgs a;
    memo_status st = check_desc(desc, &a);
    if (st != MEMO_OK) return st;
    if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv) return MEMO_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(d_o) ||
        !aligned16(dq) || !aligned16(dk) || !aligned16(dv))
        return MEMO_ERR_UNSUPPORTED;
    const size_t need = memo_attn_bwd_workspace_bytes(desc);
    if (!workspace || workspace_bytes < need) return MEMO_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return MEMO_ERR_WORKSPACE;
    a.q = q;
    a.k = k;
    a.v = v;
    a.o_in = o;
    a.d_o = d_o;
    a.dq = dq;
    a.dk = dk;
    a.dv = dv;
    a.lse = const_cast<float *>(lse);
    a.delta = static_cast<float *>(workspace);
    hipEvent_t events[4];
    if (stage_events) {
        for (int n = 0; n < 4; ++n) {
            if (!stage_events[n]) return MEMO_ERR_INVALID_ARG;
            events[n] = static_cast<hipEvent_t>(stage_events[n]);
        }
        a.stage_events = events;
    }
    hipStream_t hs = static_cast<hipStream_t>(stream);
    hipError_t e = desc->dtype == MEMO_BF16 ? memo::launch_attn_bwd_bf16(a, hs)
                                            : memo::launch_attn_bwd_f32(a, hs);
    return e == hipSuccess ? MEMO_OK : MEMO_ERR_DEVICE;
}

int64_t memo_split_tokens(int64_t S, double alpha)
{
    if (S < 0 || std::isnan(alpha) || alpha < 0.0 || alpha > 1.0) return -1;
    const double kf = std::floor(alpha * static_cast<double>(S));
    int64_t k = static_cast<int64_t>(kf);
    if (k > S) k = S;
    if (k < 0) k = 0;
    return k;
}

memo_status memo_swap_plan_make(int64_t S, int64_t row_bytes, double alpha, memo_swap_plan *out)
{
    if (!out || row_bytes <= 0) return MEMO_ERR_INVALID_ARG;
    const int64_t k = memo_split_tokens(S, alpha);
    if (k < 0) return MEMO_ERR_INVALID_ARG;
    if (S > 0 && row_bytes > INT64_MAX / S) return MEMO_ERR_INVALID_ARG;
    out->S = S;
    out->row_bytes = row_bytes;
    out->k_swapped = k;
    out->n_recompute = S - k;
    out->bytes_swapped = k * row_bytes;
    out->bytes_dropped = (S - k) * row_bytes;
    out->recompute_byte_offset = k * row_bytes;
    return MEMO_OK;
}

memo_status memo_swap_out(const void *dev_act, int64_t S, int64_t row_bytes, double alpha,
                          void *host_pinned, size_t host_capacity_bytes,
                          void *copy_stream, void *wait_event, void *done_event)
{
    memo_swap_plan plan;
    memo_status st = check_swap(dev_act, S, row_bytes, alpha, host_pinned, host_capacity_bytes, &plan);
    if (st != MEMO_OK) return st;
    hipStream_t cs = static_cast<hipStream_t>(copy_stream);
    if (wait_event &&
        hipStreamWaitEvent(cs, static_cast<hipEvent_t>(wait_event), 0) != hipSuccess)
        return MEMO_ERR_DEVICE;
    // the swapped tokens are the first k rows, which are one contiguous block
    if (plan.bytes_swapped > 0 &&
        hipMemcpyAsync(host_pinned, dev_act, (size_t)plan.bytes_swapped, hipMemcpyDeviceToHost, cs) !=
            hipSuccess)
        return MEMO_ERR_DEVICE;
    if (done_event && hipEventRecord(static_cast<hipEvent_t>(done_event), cs) != hipSuccess)
        return MEMO_ERR_DEVICE;
    return MEMO_OK;
}

memo_status memo_swap_in(void *dev_act, int64_t S, int64_t row_bytes, double alpha,
                         const void *host_pinned, size_t host_capacity_bytes,
                         void *copy_stream, void *wait_event, void *done_event)
{
    memo_swap_plan plan;
    memo_status st = check_swap(dev_act, S, row_bytes, alpha, host_pinned, host_capacity_bytes, &plan);
    if (st != MEMO_OK) return st;
    hipStream_t cs = static_cast<hipStream_t>(copy_stream);
    if (wait_event &&
        hipStreamWaitEvent(cs, static_cast<hipEvent_t>(wait_event), 0) != hipSuccess)
        return MEMO_ERR_DEVICE;
    if (plan.bytes_swapped > 0 &&
        hipMemcpyAsync(dev_act, host_pinned, (size_t)plan.bytes_swapped, hipMemcpyHostToDevice, cs) !=
            hipSuccess)
        return MEMO_ERR_DEVICE;
    if (done_event && hipEventRecord(static_cast<hipEvent_t>(done_event), cs) != hipSuccess)
        return MEMO_ERR_DEVICE;
    return MEMO_OK;
}

memo_status memo_solve_alpha(double s_in, double s_attn, double s_oth, double bandwidth,
                             double t_layer, int32_t n_layers, double m_cpu, double *alpha_out)
{
    if (!alpha_out) return MEMO_ERR_INVALID_ARG;
    if (!(s_in >= 0.0) || !(s_attn >= 0.0) || !(s_oth > 0.0) || !(bandwidth > 0.0) ||
        !(t_layer > 0.0) || n_layers < 1 || !(m_cpu >= 0.0))
        return MEMO_ERR_INVALID_ARG;
    if (!std::isfinite(s_in + s_attn + s_oth + bandwidth + t_layer + m_cpu)) return MEMO_ERR_INVALID_ARG;
    const double fixed = s_in + s_attn;   // the two tensors that are always offloaded whole
    // time constraint: fixed + alpha*s_oth <= t_layer * bandwidth
    double a = (t_layer * bandwidth - fixed) / s_oth;
    if (a < 0.0) return MEMO_ERR_UNSUPPORTED;
    // host memory constraint: the last two layers are never swapped
    if (n_layers > 2) {
        const double am = (m_cpu / static_cast<double>(n_layers - 2) - fixed) / s_oth;
        if (am < 0.0) return MEMO_ERR_HOST_CAPACITY;
        if (am < a) a = am;
    }
    *alpha_out = a > 1.0 ? 1.0 : a;
    return MEMO_OK;
}

memo_status memo_layernorm_rows(const void *x, const void *gamma, const void *beta, void *y,
                                int64_t S, int32_t h, float eps, int64_t row_begin,
                                int64_t row_end, void *hip_stream)
{
    if (!x || !gamma || !beta || !y || S < 1) return MEMO_ERR_INVALID_ARG;
    if (row_begin < 0 || row_end < row_begin || row_end > S) return MEMO_ERR_INVALID_ARG;
    if (!(eps >= 0.0f) || !std::isfinite(eps)) return MEMO_ERR_INVALID_ARG;
    if (h < 512 || h > 8192 || h % 512) return MEMO_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(gamma) || !aligned16(beta) || !aligned16(y)) return MEMO_ERR_UNSUPPORTED;
    const hipError_t e = memo::launch_layernorm_rows_bf16(x, gamma, beta, y, row_begin, row_end, h, eps,
                                                          static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MEMO_OK : MEMO_ERR_DEVICE;
}

memo_status memo_linear_rows(const void *a, const void *w, const void *bias, void *out, int64_t S,
                             int32_t K, int32_t N, int64_t row_begin, int64_t row_end,
                             void *hip_stream)
{
    if (!a || !w || !out || S < 1) return MEMO_ERR_INVALID_ARG;
    if (row_begin < 0 || row_end < row_begin || row_end > S) return MEMO_ERR_INVALID_ARG;
    if (K < 128 || N < 128 || K % 128 || N % 128) return MEMO_ERR_UNSUPPORTED;
    if (!aligned16(a) || !aligned16(w) || !aligned16(out) || (bias && !aligned16(bias))) return MEMO_ERR_UNSUPPORTED;
    const hipError_t e = memo::launch_linear_rows_bf16(a, w, bias, out, row_begin, row_end, K, N,
                                                       static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MEMO_OK : MEMO_ERR_DEVICE;
}

memo_status memo_host_alloc(void **host_ptr, size_t bytes)
{
    if (!host_ptr || bytes == 0) return MEMO_ERR_INVALID_ARG;
    *host_ptr = nullptr;
    return hipHostMalloc(host_ptr, bytes, hipHostMallocDefault) == hipSuccess ? MEMO_OK
                                                                              : MEMO_ERR_DEVICE;
}

memo_status memo_host_free(void *host_ptr)
{
    if (!host_ptr) return MEMO_ERR_INVALID_ARG;
    return hipHostFree(host_ptr) == hipSuccess ? MEMO_OK : MEMO_ERR_DEVICE;
}

}  // extern "C"
