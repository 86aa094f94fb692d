// Token-wise recomputation of the first saved tensors of a layer (Section 4.1 of the paper:
// the stored layer input is what "input_norm", "q", "k", "v" are rebuilt from): LayerNorm over
// the hidden dimension and the projection that follows it, both restricted to a row range
// [row_begin, row_end) so that only the dropped tokens are recomputed.  Each output row depends
// on its own input row only and is accumulated in a fixed order, so a row recomputed in any
// range is bit-identical to the same row of a full pass.
#include "bf16_tiles.h"

namespace memo {
namespace {

// ---------------------------------------------------------------------------- LayerNorm
// One wave per row, 8 consecutive elements per lane and 512-element chunk; fp32 statistics in two
// passes over the registers (mean, then centred sum of squares).  HBM-bound: 2*h*2 bytes per row.
constexpr int kLnMaxChunks = 16;            // h <= 8192

__global__ __launch_bounds__(256) void layernorm_rows_bf16_kernel(const __bf16 *x, const __bf16 *gamma,
                                                                  const __bf16 *beta, __bf16 *y, int64_t row_begin,
                                                                  int64_t row_end, int h, float eps)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = row_begin + (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= row_end) return;
    const int nch = h / 512;
    const __bf16 *xr = x + row * h;
    float v[kLnMaxChunks][8];
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < kLnMaxChunks; ++c) {
        if (c < nch) {
            const bf16x8 raw = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(xr + c * 512 + lane * 8));
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                v[c][e] = (float)raw[e];
                sum += v[c][e];
            }
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    const float mean = sum / (float)h;
    float sq = 0.f;
#pragma unroll
    for (int c = 0; c < kLnMaxChunks; ++c)
        if (c < nch)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float dlt = v[c][e] - mean;
                sq = fmaf(dlt, dlt, sq);
            }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sq += __shfl_xor(sq, o, 64);
    const float rstd = 1.0f / sqrtf(sq / (float)h + eps);
    __bf16 *yr = y + row * h;
#pragma unroll
    for (int c = 0; c < kLnMaxChunks; ++c) {
        if (c < nch) {
            const bf16x8 gm = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(gamma + c * 512 + lane * 8));
            const bf16x8 bt = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(beta + c * 512 + lane * 8));
            bf16x8 out;
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                f32x2 two = {fmaf((v[c][e] - mean) * rstd, (float)gm[e], (float)bt[e]),
                             fmaf((v[c][e + 1] - mean) * rstd, (float)gm[e + 1], (float)bt[e + 1])};
                bf16x2 r = __builtin_convertvector(two, bf16x2);
                out[e] = r[0];
                out[e + 1] = r[1];
            }
            *reinterpret_cast<u32x4 *>(yr + c * 512 + lane * 8) = __builtin_bit_cast(u32x4, out);
        }
    }
}

// ---------------------------------------------------------------------------- projection
// out[token, feature] = sum_c a[token, c] * w[feature, c] + bias[feature]   (w as [N, K], K contiguous)
// Workgroup: 8 waves, 128 tokens x 128 features; K streamed in chunks of 128 through a
// double-buffered LDS ring of swizzled 64-row tiles (2 token tiles + 2 weight tiles per stage).
// Wave w owns tokens 32*(w%4).. and features 64*(w/4)..: D[feature, token] = W_rows * A_rows^T,
// so a lane holds one token and 4 consecutive features per register group (8-byte stores).
struct TripleSlot { bf16x8 b, a0, a1; };

template <int N>
__device__ __forceinline__ void lds_wait(TripleSlot &x)
{
    static_assert(N >= 0 && N <= 15, "lgkmcnt range");
    asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(x.b), "+v"(x.a0), "+v"(x.a1) : "n"(N));
}

constexpr int kLinBm = 128, kLinBn = 128, kLinBk = 128;

__global__ __launch_bounds__(512, 2) void linear_rows_bf16_kernel(const __bf16 *a, const __bf16 *w, const __bf16 *bias,
                                                                  __bf16 *out, int64_t row_begin, int64_t row_end,
                                                                  int K, int N)
{
    // token tiles [buf][2] in the first 64 KB, weight tiles [buf][2] in the second: each operand's
    // two buffers lie within the 64 KB an LDS immediate offset can reach from one address register
    __shared__ __attribute__((aligned(1024))) unsigned char smem[8 * kTileBytes];
    LDS_AS unsigned char *lds = (LDS_AS unsigned char *)smem;

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tb = wave & 3, fh = wave >> 2;
    const int ntn = N / kLinBn;
    const int64_t mt = blockIdx.x / ntn;              // consecutive workgroups share the token rows
    const int nt = (int)(blockIdx.x % ntn);
    const int64_t m0 = row_begin + mt * kLinBm;
    const int n0 = nt * kLinBn;
    const LaneAddr la = make_lane_addr(lane);
    const LdsAddr ad = make_lds_addr(lds, la);
    uint32_t tok_addr[8], wgt_addr[8];
#pragma unroll
    for (int kc = 0; kc < 8; ++kc) {
        tok_addr[kc] = ad.row[kc] + (uint32_t)(tb * 8192);
        wgt_addr[kc] = ad.row[kc] + (uint32_t)(4 * kTileBytes + fh * 16384);
    }
    const TileOffsets<8> toff = make_tile_offsets<8>(K, wave, lane);
    const bool full_rows = m0 + kLinBm <= row_end;
    const int nchunks = K / kLinBk;

    // queue the fill of K-chunk c into ring buffer `buf`
    auto fill_chunk = [&](int buf, int c) {
        LDS_AS unsigned char *tdst = lds + buf * 2 * kTileBytes, *wdst = lds + (4 + buf * 2) * kTileBytes;
        const char *wbase = reinterpret_cast<const char *>(w + (int64_t)n0 * K + (int64_t)c * kLinBk);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            if (full_rows) {
                const char *abase = reinterpret_cast<const char *>(a + (m0 + 64 * t) * K + (int64_t)c * kLinBk);
                fill_full_tile_part(tdst + t * kTileBytes, toff, 0, abase, wave);
                fill_full_tile_part(tdst + t * kTileBytes, toff, 1, abase, wave);
            } else {
                // rows past row_end re-read row row_end-1 (finite values, never stored)
                fill_ragged_tile<8>(tdst + t * kTileBytes, a + (int64_t)c * kLinBk, K, m0 + 64 * t, row_end, wave, lane);
            }
            const char *wt = wbase + (int64_t)(64 * t) * K * 2;
            fill_full_tile_part(wdst + t * kTileBytes, toff, 0, wt, wave);
            fill_full_tile_part(wdst + t * kTileBytes, toff, 1, wt, wave);
        }
    };

    f32x16 acc[2];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[cb][e] = 0.f;

    fill_chunk(0, 0);
    auto stage = [&](auto bufc, int c) {
        constexpr int BUF = decltype(bufc)::value;
        constexpr int off = BUF * 2 * kTileBytes;
        wait_fills();
        __syncthreads();          // chunk c is complete; nobody still reads the other buffer
        if (c + 1 < nchunks) fill_chunk(BUF ^ 1, c + 1);
        TripleSlot ring[3];
        auto issue = [&](auto n, TripleSlot &slot) {
            constexpr int kc = decltype(n)::value;
            lds_issue_b128<off>(slot.b, tok_addr[kc]);
            lds_issue_b128<off>(slot.a0, wgt_addr[kc]);
            lds_issue_b128<off + 8192>(slot.a1, wgt_addr[kc]);
        };
        lds_pipeline_prologue<8, 2, 3>(ring, issue);
        lds_pipeline_body<8, 2, 3>(ring, issue, [&](auto n, TripleSlot &slot) {
            acc[0] = mfma32(slot.a0, slot.b, acc[0]);
            acc[1] = mfma32(slot.a1, slot.b, acc[1]);
        });
    };
    for (int c = 0; c < nchunks; c += 2) {
        stage(IntC<0>{}, c);
        if (c + 1 < nchunks) stage(IntC<1>{}, c + 1);
    }

    // acc[cb][4g + r] = out[token m0 + 32 tb + l32][feature n0 + 64 fh + 32 cb + 8 g + 4 half + r]
    const int64_t token = m0 + 32 * tb + l32;
    if (token < row_end) {
        __bf16 *orow = out + token * N + n0 + 64 * fh + 4 * half;
        const __bf16 *brow = bias ? bias + n0 + 64 * fh + 4 * half : nullptr;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float b4[4] = {0.f, 0.f, 0.f, 0.f};
                if (brow) {
                    const u32x2 braw = *reinterpret_cast<const u32x2 *>(brow + 32 * cb + 8 * g);
                    // elements copied to scalars first: a bit cast applied to a vector element
                    // directly reads element 0 for both with this compiler
                    const uint32_t r0 = braw[0], r1 = braw[1];
                    const bf16x2 lo = __builtin_bit_cast(bf16x2, r0), hi = __builtin_bit_cast(bf16x2, r1);
                    b4[0] = (float)lo[0]; b4[1] = (float)lo[1]; b4[2] = (float)hi[0]; b4[3] = (float)hi[1];
                }
                f32x2 p = {acc[cb][4 * g] + b4[0], acc[cb][4 * g + 1] + b4[1]};
                f32x2 q = {acc[cb][4 * g + 2] + b4[2], acc[cb][4 * g + 3] + b4[3]};
                u32x2 wv;
                wv[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(p, bf16x2));
                wv[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(q, bf16x2));
                *reinterpret_cast<u32x2 *>(orow + 32 * cb + 8 * g) = wv;
            }
    }
}

}  // namespace

hipError_t launch_layernorm_rows_bf16(const void *x, const void *gamma, const void *beta, void *y, int64_t row_begin,
                                      int64_t row_end, int h, float eps, hipStream_t st)
{
    const int64_t rows = row_end - row_begin;
    if (rows <= 0) return hipSuccess;
    const int64_t blocks = (rows + 3) / 4;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    layernorm_rows_bf16_kernel<<<dim3((unsigned)blocks), 256, 0, st>>>(
        static_cast<const __bf16 *>(x), static_cast<const __bf16 *>(gamma), static_cast<const __bf16 *>(beta),
        static_cast<__bf16 *>(y), row_begin, row_end, h, eps);
    return hipGetLastError();
}

hipError_t launch_linear_rows_bf16(const void *a, const void *w, const void *bias, void *out, int64_t row_begin,
                                   int64_t row_end, int K, int N, hipStream_t st)
{
    const int64_t rows = row_end - row_begin;
    if (rows <= 0) return hipSuccess;
    const int64_t blocks = ((rows + kLinBm - 1) / kLinBm) * (N / kLinBn);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    linear_rows_bf16_kernel<<<dim3((unsigned)blocks), 512, 0, st>>>(
        static_cast<const __bf16 *>(a), static_cast<const __bf16 *>(w), static_cast<const __bf16 *>(bias),
        static_cast<__bf16 *>(out), row_begin, row_end, K, N);
    return hipGetLastError();
}

}  // namespace memo
