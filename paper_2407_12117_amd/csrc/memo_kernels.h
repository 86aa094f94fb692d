// Internal interface between the C-ABI front end (memo_api.cpp) and the gfx950 kernels.
// Not installed; the public contract is include/memo.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace memo {

// One attention problem as the kernels see it.  Element (b, s, h, c) of q/k/v/o/d_o/dq/dk/dv
// is at b*sb + s*ss + h*sh + c (elements); lse and delta are [B,H,S] fp32.
struct AttnArgs {
    const void *q, *k, *v;
    const void *o_in;     // backward: forward output
    const void *d_o;      // backward: dL/dO
    void *o_out;          // forward: output
    void *dq, *dk, *dv;   // backward outputs
    float *lse;           // forward: written; backward: read
    float *delta;         // backward workspace: D_i = sum_c dO_ic O_ic, [B,H,S]
    int32_t B, H, d;
    int64_t S;
    float scale;
    int64_t sb, ss, sh;
    hipEvent_t *stage_events;   // backward only, nullable: 4 events recorded between the stages
};

inline hipError_t record_stage(const AttnArgs &a, int idx, hipStream_t st)
{
    return a.stage_events ? hipEventRecord(a.stage_events[idx], st) : hipSuccess;
}

// fp32 path (VALU arithmetic, fp32 throughout), d in {64, 128}
hipError_t launch_attn_fwd_f32(const AttnArgs &a, hipStream_t st);
hipError_t launch_attn_bwd_f32(const AttnArgs &a, hipStream_t st);

// bf16 path (bf16 MFMA contractions, fp32 accumulation and softmax), d = 128
hipError_t launch_attn_fwd_bf16(const AttnArgs &a, hipStream_t st);
hipError_t launch_attn_bwd_bf16(const AttnArgs &a, hipStream_t st);

// D_i = sum_c dO_ic * O_ic for either dtype (is_bf16 selects the element type)
hipError_t launch_attn_delta(const AttnArgs &a, bool is_bf16, hipStream_t st);

// Token-wise recomputation (bf16): LayerNorm of rows [row_begin,row_end) of x [S,h] and the
// projection out[rows, N] = a[rows, K] * w[N, K]^T + bias over the same kind of row range.
hipError_t launch_layernorm_rows_bf16(const void *x, const void *gamma, const void *beta, void *y,
                                      int64_t row_begin, int64_t row_end, int h, float eps, hipStream_t st);
hipError_t launch_linear_rows_bf16(const void *a, const void *w, const void *bias, void *out,
                                   int64_t row_begin, int64_t row_end, int K, int N, hipStream_t st);

}  // namespace memo
