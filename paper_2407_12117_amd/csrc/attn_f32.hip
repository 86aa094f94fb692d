// fp32 causal attention forward/backward for gfx950 (Section 2.1.3 of the paper: exact
// softmax attention computed tile by tile with per-row running state, intermediates
// re-formed in the backward).  This is the full-precision path: plain fp32 VALU
// arithmetic, no rounding of the probabilities.  It serves the small fp32 workload; the
// long-sequence work goes through the bf16 MFMA kernels.
//
// Work split: a workgroup of 256 threads owns 64 rows (query rows in the forward and the
// dQ kernel, key rows in the dK/dV kernel); 4 adjacent lanes share a row, lane `part`
// holding columns part, part+4, part+8, ... so that the 4 lanes read adjacent LDS banks.
// Dot products are completed with two xor-shuffles inside the 4-lane group.
#include "memo_kernels.h"
#include <hip/hip_bf16.h>

namespace memo {
namespace {

constexpr int kRows = 64;    // rows owned by a workgroup
constexpr int kT = 4;        // lanes per row
constexpr int kTile = 32;    // rows of the streamed operand staged in LDS per step

__device__ __forceinline__ float group4_sum(float x)
{
    x += __shfl_xor(x, 1);
    x += __shfl_xor(x, 2);
    return x;
}

// Stage `kTile` rows [r0, r0+kTile) of a [S, D] head view into LDS; rows >= S are zeroed.
template <int D>
__device__ __forceinline__ void stage_rows(float *dst, const float *src, int64_t ss, int64_t r0,
                                           int64_t S, int tid)
{
    constexpr int vec_per_row = D / 4;
    for (int idx = tid; idx < kTile * vec_per_row; idx += 256) {
        const int r = idx / vec_per_row, c4 = idx % vec_per_row;
        float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r0 + r < S) val = *reinterpret_cast<const float4 *>(src + (r0 + r) * ss + 4 * c4);
        *reinterpret_cast<float4 *>(dst + r * D + 4 * c4) = val;
    }
}

template <int D>
__global__ __launch_bounds__(256) void attn_fwd_f32_kernel(AttnArgs a)
{
    constexpr int DT = D / kT;
    __shared__ __attribute__((aligned(16))) float Ks[kTile * D];
    __shared__ __attribute__((aligned(16))) float Vs[kTile * D];
    const int tid = threadIdx.x, r = tid / kT, part = tid % kT;
    const int h = blockIdx.y, b = blockIdx.z;
    const int64_t row0 = (int64_t)blockIdx.x * kRows;
    const int64_t i = row0 + r;
    const bool live = i < a.S;
    const int64_t base = (int64_t)b * a.sb + (int64_t)h * a.sh;
    const float *q = static_cast<const float *>(a.q) + base;
    const float *k = static_cast<const float *>(a.k) + base;
    const float *v = static_cast<const float *>(a.v) + base;

    float qr[DT], acc[DT];
#pragma unroll
    for (int c = 0; c < DT; ++c) {
        qr[c] = live ? q[i * a.ss + c * kT + part] : 0.f;
        acc[c] = 0.f;
    }
    float m = -INFINITY, l = 0.f;
    const int64_t last_row = min(row0 + kRows, a.S) - 1;
    const int64_t ntiles = last_row / kTile + 1;

    for (int64_t t = 0; t < ntiles; ++t) {
        const int64_t j0 = t * kTile;
        __syncthreads();
        stage_rows<D>(Ks, k, a.ss, j0, a.S, tid);
        stage_rows<D>(Vs, v, a.ss, j0, a.S, tid);
        __syncthreads();
        float s[kTile];
        float mt = -INFINITY;
#pragma unroll
        for (int jj = 0; jj < kTile; ++jj) {
            float dot = 0.f;
#pragma unroll
            for (int c = 0; c < DT; ++c) dot += qr[c] * Ks[jj * D + c * kT + part];
            dot = group4_sum(dot) * a.scale;
            s[jj] = (j0 + jj <= i) ? dot : -INFINITY;
            mt = fmaxf(mt, s[jj]);
        }
        // the first tile always holds key 0, which every row sees, so m_new is finite
        // from the first tile on; only rows past S (not stored) can stay at -inf
        const float m_new = fmaxf(m, mt);
        const float corr = (m_new == -INFINITY) ? 1.f : __expf(m - m_new);
        l *= corr;
#pragma unroll
        for (int c = 0; c < DT; ++c) acc[c] *= corr;
#pragma unroll
        for (int jj = 0; jj < kTile; ++jj) {
            const float p = (s[jj] == -INFINITY) ? 0.f : __expf(s[jj] - m_new);
            l += p;
#pragma unroll
            for (int c = 0; c < DT; ++c) acc[c] += p * Vs[jj * D + c * kT + part];
        }
        m = m_new;
    }
    if (live) {
        float *o = static_cast<float *>(a.o_out) + base + i * a.ss;
        const float inv = 1.f / l;
#pragma unroll
        for (int c = 0; c < DT; ++c) o[c * kT + part] = acc[c] * inv;
        if (part == 0) a.lse[((int64_t)b * a.H + h) * a.S + i] = m + __logf(l);
    }
}

// dQ_i = scale * sum_{j<=i} dS_ij k_j, dS_ij = P_ij (dO_i.v_j - D_i), P_ij = exp(s_ij - LSE_i)
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dq_f32_kernel(AttnArgs a)
{
    constexpr int DT = D / kT;
    __shared__ __attribute__((aligned(16))) float Ks[kTile * D];
    __shared__ __attribute__((aligned(16))) float Vs[kTile * D];
    const int tid = threadIdx.x, r = tid / kT, part = tid % kT;
    const int h = blockIdx.y, b = blockIdx.z;
    const int64_t row0 = (int64_t)blockIdx.x * kRows;
    const int64_t i = row0 + r;
    const bool live = i < a.S;
    const int64_t base = (int64_t)b * a.sb + (int64_t)h * a.sh;
    const float *q = static_cast<const float *>(a.q) + base;
    const float *k = static_cast<const float *>(a.k) + base;
    const float *v = static_cast<const float *>(a.v) + base;
    const float *g = static_cast<const float *>(a.d_o) + base;
    const int64_t stat = ((int64_t)b * a.H + h) * a.S;

    float qr[DT], gr[DT], acc[DT];
#pragma unroll
    for (int c = 0; c < DT; ++c) {
        qr[c] = live ? q[i * a.ss + c * kT + part] : 0.f;
        gr[c] = live ? g[i * a.ss + c * kT + part] : 0.f;
        acc[c] = 0.f;
    }
    const float lse_i = live ? a.lse[stat + i] : 0.f;
    const float D_i = live ? a.delta[stat + i] : 0.f;
    const int64_t last_row = min(row0 + kRows, a.S) - 1;
    const int64_t ntiles = last_row / kTile + 1;

    for (int64_t t = 0; t < ntiles; ++t) {
        const int64_t j0 = t * kTile;
        __syncthreads();
        stage_rows<D>(Ks, k, a.ss, j0, a.S, tid);
        stage_rows<D>(Vs, v, a.ss, j0, a.S, tid);
        __syncthreads();
#pragma unroll 4
        for (int jj = 0; jj < kTile; ++jj) {
            float dot = 0.f, dp = 0.f;
#pragma unroll
            for (int c = 0; c < DT; ++c) {
                dot += qr[c] * Ks[jj * D + c * kT + part];
                dp += gr[c] * Vs[jj * D + c * kT + part];
            }
            dot = group4_sum(dot);
            dp = group4_sum(dp);
            const float p = (j0 + jj <= i) ? __expf(dot * a.scale - lse_i) : 0.f;
            const float ds = p * (dp - D_i);
#pragma unroll
            for (int c = 0; c < DT; ++c) acc[c] += ds * Ks[jj * D + c * kT + part];
        }
    }
    if (live) {
        float *dq = static_cast<float *>(a.dq) + base + i * a.ss;
#pragma unroll
        for (int c = 0; c < DT; ++c) dq[c * kT + part] = acc[c] * a.scale;
    }
}

// dV_j = sum_{i>=j} P_ij dO_i,  dK_j = scale * sum_{i>=j} dS_ij q_i
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dkdv_f32_kernel(AttnArgs a)
{
    constexpr int DT = D / kT;
    __shared__ __attribute__((aligned(16))) float Qs[kTile * D];
    __shared__ __attribute__((aligned(16))) float Gs[kTile * D];
    __shared__ float Ls[kTile], Ds[kTile];
    const int tid = threadIdx.x, r = tid / kT, part = tid % kT;
    const int h = blockIdx.y, b = blockIdx.z;
    const int64_t col0 = (int64_t)blockIdx.x * kRows;
    const int64_t j = col0 + r;
    const bool live = j < a.S;
    const int64_t base = (int64_t)b * a.sb + (int64_t)h * a.sh;
    const float *q = static_cast<const float *>(a.q) + base;
    const float *k = static_cast<const float *>(a.k) + base;
    const float *v = static_cast<const float *>(a.v) + base;
    const float *g = static_cast<const float *>(a.d_o) + base;
    const int64_t stat = ((int64_t)b * a.H + h) * a.S;

    float kr[DT], vr[DT], dk[DT], dv[DT];
#pragma unroll
    for (int c = 0; c < DT; ++c) {
        kr[c] = live ? k[j * a.ss + c * kT + part] : 0.f;
        vr[c] = live ? v[j * a.ss + c * kT + part] : 0.f;
        dk[c] = 0.f;
        dv[c] = 0.f;
    }
    const int64_t t0 = col0 / kTile;
    const int64_t ntiles = (a.S + kTile - 1) / kTile;
    for (int64_t t = t0; t < ntiles; ++t) {
        const int64_t i0 = t * kTile;
        __syncthreads();
        stage_rows<D>(Qs, q, a.ss, i0, a.S, tid);
        stage_rows<D>(Gs, g, a.ss, i0, a.S, tid);
        if (tid < kTile) {
            const bool ok = i0 + tid < a.S;
            // rows past S get LSE = +inf so that their probability is exactly zero
            Ls[tid] = ok ? a.lse[stat + i0 + tid] : INFINITY;
            Ds[tid] = ok ? a.delta[stat + i0 + tid] : 0.f;
        }
        __syncthreads();
#pragma unroll 4
        for (int ii = 0; ii < kTile; ++ii) {
            float dot = 0.f, dp = 0.f;
#pragma unroll
            for (int c = 0; c < DT; ++c) {
                dot += kr[c] * Qs[ii * D + c * kT + part];
                dp += vr[c] * Gs[ii * D + c * kT + part];
            }
            dot = group4_sum(dot);
            dp = group4_sum(dp);
            const float p = (i0 + ii >= j) ? __expf(dot * a.scale - Ls[ii]) : 0.f;
            const float ds = p * (dp - Ds[ii]);
#pragma unroll
            for (int c = 0; c < DT; ++c) {
                dv[c] += p * Gs[ii * D + c * kT + part];
                dk[c] += ds * Qs[ii * D + c * kT + part];
            }
        }
    }
    if (live) {
        float *pdk = static_cast<float *>(a.dk) + base + j * a.ss;
        float *pdv = static_cast<float *>(a.dv) + base + j * a.ss;
#pragma unroll
        for (int c = 0; c < DT; ++c) {
            pdk[c * kT + part] = dk[c] * a.scale;
            pdv[c * kT + part] = dv[c];
        }
    }
}

// D_i = sum_c dO_ic O_ic.  16 lanes per row, 16 rows per 256-thread workgroup.
template <typename T, int D>
__global__ __launch_bounds__(256) void attn_delta_kernel(AttnArgs a)
{
    const int tid = threadIdx.x, r = tid / 16, part = tid % 16;
    const int h = blockIdx.y, b = blockIdx.z;
    const int64_t i = (int64_t)blockIdx.x * 16 + r;
    const int64_t base = (int64_t)b * a.sb + (int64_t)h * a.sh;
    float sum = 0.f;
    if (i < a.S) {
        const T *o = static_cast<const T *>(a.o_in) + base + i * a.ss;
        const T *g = static_cast<const T *>(a.d_o) + base + i * a.ss;
        constexpr int per = D / 16;
#pragma unroll
        for (int c = 0; c < per; ++c)
            sum += static_cast<float>(o[part * per + c]) * static_cast<float>(g[part * per + c]);
    }
    sum += __shfl_xor(sum, 1);
    sum += __shfl_xor(sum, 2);
    sum += __shfl_xor(sum, 4);
    sum += __shfl_xor(sum, 8);
    if (i < a.S && part == 0) a.delta[((int64_t)b * a.H + h) * a.S + i] = sum;
}

inline dim3 row_grid(const AttnArgs &a, int rows)
{
    return dim3((unsigned)((a.S + rows - 1) / rows), (unsigned)a.H, (unsigned)a.B);
}

}  // namespace

hipError_t launch_attn_fwd_f32(const AttnArgs &a, hipStream_t st)
{
    if (a.d == 64)
        attn_fwd_f32_kernel<64><<<row_grid(a, kRows), 256, 0, st>>>(a);
    else
        attn_fwd_f32_kernel<128><<<row_grid(a, kRows), 256, 0, st>>>(a);
    return hipGetLastError();
}

hipError_t launch_attn_delta(const AttnArgs &a, bool is_bf16, hipStream_t st)
{
    const dim3 grid = row_grid(a, 16);
    if (is_bf16) {
        if (a.d == 64)
            attn_delta_kernel<__hip_bfloat16, 64><<<grid, 256, 0, st>>>(a);
        else
            attn_delta_kernel<__hip_bfloat16, 128><<<grid, 256, 0, st>>>(a);
    } else {
        if (a.d == 64)
            attn_delta_kernel<float, 64><<<grid, 256, 0, st>>>(a);
        else
            attn_delta_kernel<float, 128><<<grid, 256, 0, st>>>(a);
    }
    return hipGetLastError();
}

hipError_t launch_attn_bwd_f32(const AttnArgs &a, hipStream_t st)
{
    hipError_t e = record_stage(a, 0, st);
    if (e != hipSuccess) return e;
    e = launch_attn_delta(a, false, st);
    if (e != hipSuccess) return e;
    if ((e = record_stage(a, 1, st)) != hipSuccess) return e;
    if (a.d == 64)
        attn_bwd_dkdv_f32_kernel<64><<<row_grid(a, kRows), 256, 0, st>>>(a);
    else
        attn_bwd_dkdv_f32_kernel<128><<<row_grid(a, kRows), 256, 0, st>>>(a);
    if ((e = record_stage(a, 2, st)) != hipSuccess) return e;
    if (a.d == 64)
        attn_bwd_dq_f32_kernel<64><<<row_grid(a, kRows), 256, 0, st>>>(a);
    else
        attn_bwd_dq_f32_kernel<128><<<row_grid(a, kRows), 256, 0, st>>>(a);
    if ((e = record_stage(a, 3, st)) != hipSuccess) return e;
    return hipGetLastError();
}

}  // namespace memo
