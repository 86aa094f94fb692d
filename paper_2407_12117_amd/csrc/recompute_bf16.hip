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

template <int NCH>                          // h = 512 * NCH: the row lives in 8 * NCH registers per lane
__global__ __launch_bounds__(256) void layernorm_rows_bf16_kernel(const __bf16 *x, const __bf16 *gamma,
                                                                  const __bf16 *beta, __bf16 *y, int64_t row_begin,
                                                                  int64_t row_end, int h, float eps)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = row_begin + (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= row_end) return;
    constexpr int nch = NCH;
    const __bf16 *xr = x + row * h;
    float v[NCH][8];
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
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
    for (int c = 0; c < NCH; ++c)
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
    for (int c = 0; c < NCH; ++c) {
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
// Workgroup: 8 waves, 256 tokens x 256 features; K streamed in chunks of 64 through a double-buffered
// LDS ring (32 KB of token rows + 32 KB of weight rows per stage).  The fills are what bounds this
// kernel (bytes into LDS per MFMA), hence the large tile.  Wave w owns tokens 64*(w%4).. (4 blocks
// of 16) and features 128*(w/4).. (8 blocks of 16): D[feature, token] = W_rows * A_rows^T on
// v_mfma_f32_16x16x32_bf16, so a lane holds one token and 4 consecutive features per accumulator
// (8-byte stores); per 32-wide k-step a wave reads 4 + 8 operands for 32 MFMAs.  The 16x16x32
// shape is chosen over 32x32x16 because the chip is power-limited on random data and sustains
// about an eighth more flops per second with it; the operand traffic from LDS is the same for
// the same wave tile.
//
// Operand conventions of the 16x16x32 MFMA, D = A(16xK32) * B(K32x16), lane = 16*g4 + l16:
//   A : lane holds row l16, k = 8*g4 .. 8*g4+7;  B : lane holds col l16, k = 8*g4 .. 8*g4+7;
//   D : lane holds col l16, rows 4*g4 + r for register r (4 fp32).
//
// LDS rows here are 128 bytes (64 bf16): chunk c (16 bytes) of row r sits at position
// c ^ ((r >> 1) & 7), which keeps 16 lanes reading one chunk column of 16 consecutive rows on
// distinct banks.  One global_load_lds_dwordx4 moves 8 rows.
constexpr int kLinBm = 256, kLinBn = 256, kLinBk = 64;
constexpr int kLinTile = 256 * 128;          // bytes of one operand's stage

struct TwelveSlot { bf16x8 b[4], a[8]; };

template <int N>
__device__ __forceinline__ void lds_wait(TwelveSlot &x)
{
    static_assert(N >= 0 && N <= 15, "lgkmcnt range");
    asm volatile("s_waitcnt lgkmcnt(%12)"
                 : "+v"(x.b[0]), "+v"(x.b[1]), "+v"(x.b[2]), "+v"(x.b[3]), "+v"(x.a[0]), "+v"(x.a[1]), "+v"(x.a[2]),
                   "+v"(x.a[3]), "+v"(x.a[4]), "+v"(x.a[5]), "+v"(x.a[6]), "+v"(x.a[7])
                 : "n"(N));
}

__global__ __launch_bounds__(512, 2) void linear_rows_bf16_kernel(const __bf16 *a, const __bf16 *w, const __bf16 *bias,
                                                                    __bf16 *out, int64_t row_begin, int64_t row_end,
                                                                    int K, int N)
{
    // token rows [buf] in the first 64 KB, weight rows [buf] in the second: each operand's two buffers
    // lie within the 64 KB an LDS immediate offset can reach from one address register
    __shared__ __attribute__((aligned(1024))) unsigned char smem[4 * kLinTile];
    LDS_AS unsigned char *lds = (LDS_AS unsigned char *)smem;

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, g4 = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tb = wave & 3, fh = wave >> 2;
    const int ntn = (N + kLinBn - 1) / kLinBn;
    // Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.  The ids are remapped so
    // that every XCD works through a contiguous range of (token tile, feature tile) pairs with the
    // feature tile running fastest: the workgroups that share a token tile then run on one XCD close
    // in time, and the token rows are fetched from HBM once instead of once per feature tile.
    const int64_t nblk = gridDim.x, per = nblk / 8, rem = nblk % 8;
    const int64_t xcd = blockIdx.x % 8, idx = blockIdx.x / 8;
    const int64_t logical = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + idx;
    const int64_t mt = logical / ntn;
    const int nt = (int)(logical % ntn);
    const int64_t m0 = row_begin + mt * kLinBm;
    const int n0 = nt * kLinBn;

    // operand read addresses: row l16 of a 16-row block, chunk 4*ks + g4, ks = 0..1
    uint32_t tok_addr[2], wgt_addr[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const uint32_t in_block = (uint32_t)(l16 * 128 + ((((4 * ks + g4) ^ ((l16 >> 1) & 7))) << 4));
        tok_addr[ks] = (uint32_t)(uintptr_t)lds + in_block + (uint32_t)(tb * 64 * 128);
        wgt_addr[ks] = (uint32_t)(uintptr_t)lds + in_block + (uint32_t)(2 * kLinTile + fh * 128 * 128);
    }
    // fills: instruction n of this wave covers stage rows 8*(4*wave + n) + lane/8, position lane%8
    uint32_t tok_off[4], wgt_off[4];
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        const int row = 8 * (4 * wave + n) + (lane >> 3);
        const int chunk = (lane & 7) ^ ((row >> 1) & 7);
        int64_t tr = m0 + row, wr = n0 + row;
        tr = tr < row_end ? tr : row_end - 1;         // rows past the range repeat the last one, never stored
        wr = wr < N ? wr : N - 1;
        tok_off[n] = (uint32_t)((tr - m0) * K * 2 + chunk * 16);
        wgt_off[n] = (uint32_t)((wr - n0) * K * 2 + chunk * 16);
    }
    const char *abase = reinterpret_cast<const char *>(a + m0 * K);
    const char *wbase = reinterpret_cast<const char *>(w + (int64_t)n0 * K);
    const int nchunks = K / kLinBk;

    auto fill_chunk = [&](int buf, int c) {
        LDS_AS unsigned char *tdst = lds + buf * kLinTile + (4 * wave) * 1024;
        LDS_AS unsigned char *wdst = lds + (2 + buf) * kLinTile + (4 * wave) * 1024;
        const char *ab = abase + (int64_t)c * kLinBk * 2, *wb = wbase + (int64_t)c * kLinBk * 2;
#pragma unroll
        for (int n = 0; n < 4; ++n) {
            __builtin_amdgcn_global_load_lds((const GLB_AS void *)(ab + tok_off[n]), (LDS_AS void *)(tdst + n * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((const GLB_AS void *)(wb + wgt_off[n]), (LDS_AS void *)(wdst + n * 1024), 16, 0, 0);
        }
    };

    f32x4 acc[8][4];                                 // [feature block of 16][token block of 16]
#pragma unroll
    for (int fb = 0; fb < 8; ++fb)
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[fb][t][e] = 0.f;

    fill_chunk(0, 0);
    auto stage = [&](auto bufc, int c) {
        constexpr int BUF = decltype(bufc)::value;
        constexpr int off = BUF * kLinTile;
        wait_fills();
        __syncthreads();          // chunk c is complete; nobody still reads the other buffer
        if (c + 1 < nchunks) fill_chunk(BUF ^ 1, c + 1);
        TwelveSlot ring[2];
        auto issue = [&](auto n, TwelveSlot &slot) {
            constexpr int ks = decltype(n)::value;
            static_for<0, 4>([&](auto t) { lds_issue_b128<off + decltype(t)::value * 16 * 128>(slot.b[decltype(t)::value], tok_addr[ks]); });
            static_for<0, 8>([&](auto f) { lds_issue_b128<off + decltype(f)::value * 16 * 128>(slot.a[decltype(f)::value], wgt_addr[ks]); });
        };
        lds_pipeline_prologue<2, 1, 12>(ring, issue);
        lds_pipeline_body<2, 1, 12>(ring, issue, [&](auto n, TwelveSlot &slot) {
#pragma unroll
            for (int fb = 0; fb < 8; ++fb)
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    acc[fb][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(slot.a[fb], slot.b[t], acc[fb][t], 0, 0, 0);
        });
    };
    for (int c = 0; c < nchunks; c += 2) {
        stage(IntC<0>{}, c);
        if (c + 1 < nchunks) stage(IntC<1>{}, c + 1);
    }

    // acc[fb][t][r] = out[token m0 + 64 tb + 16 t + l16][feature n0 + 128 fh + 16 fb + 4 g4 + r]
    if (n0 + 128 * fh < N) {                          // N is a multiple of 128: a feature half is whole or absent
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int64_t token = m0 + 64 * tb + 16 * t + l16;
            if (token >= row_end) continue;
            __bf16 *orow = out + token * N + n0 + 128 * fh + 4 * g4;
            const __bf16 *brow = bias ? bias + n0 + 128 * fh + 4 * g4 : nullptr;
#pragma unroll
            for (int fb = 0; fb < 8; ++fb) {
                float b4[4] = {0.f, 0.f, 0.f, 0.f};
                if (brow) {
                    const u32x2 braw = *reinterpret_cast<const u32x2 *>(brow + 16 * fb);
                    // elements copied to scalars first: a bit cast applied to a vector element
                    // directly reads element 0 for both with this compiler
                    const uint32_t r0 = braw[0], r1 = braw[1];
                    const bf16x2 lo = __builtin_bit_cast(bf16x2, r0), hi = __builtin_bit_cast(bf16x2, r1);
                    b4[0] = (float)lo[0]; b4[1] = (float)lo[1]; b4[2] = (float)hi[0]; b4[3] = (float)hi[1];
                }
                f32x2 p = {acc[fb][t][0] + b4[0], acc[fb][t][1] + b4[1]};
                f32x2 q = {acc[fb][t][2] + b4[2], acc[fb][t][3] + b4[3]};
                u32x2 wv;
                wv[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(p, bf16x2));
                wv[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(q, bf16x2));
                *reinterpret_cast<u32x2 *>(orow + 16 * fb) = wv;
            }
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
    if (blocks > 0x7fffffffLL || h % 512 || h / 512 > kLnMaxChunks) return hipErrorInvalidValue;
    const __bf16 *xp = static_cast<const __bf16 *>(x), *gp = static_cast<const __bf16 *>(gamma);
    const __bf16 *bp = static_cast<const __bf16 *>(beta);
    __bf16 *yp = static_cast<__bf16 *>(y);
    const dim3 grid((unsigned)blocks);
    switch (h / 512) {
#define MEMO_LN_CASE(n) \
    case n: layernorm_rows_bf16_kernel<n><<<grid, 256, 0, st>>>(xp, gp, bp, yp, row_begin, row_end, h, eps); break;
        MEMO_LN_CASE(1) MEMO_LN_CASE(2) MEMO_LN_CASE(3) MEMO_LN_CASE(4) MEMO_LN_CASE(5) MEMO_LN_CASE(6)
        MEMO_LN_CASE(7) MEMO_LN_CASE(8) MEMO_LN_CASE(9) MEMO_LN_CASE(10) MEMO_LN_CASE(11) MEMO_LN_CASE(12)
        MEMO_LN_CASE(13) MEMO_LN_CASE(14) MEMO_LN_CASE(15) MEMO_LN_CASE(16)
#undef MEMO_LN_CASE
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_linear_rows_bf16(const void *a, const void *w, const void *bias, void *out, int64_t row_begin,
                                   int64_t row_end, int K, int N, hipStream_t st)
{
    const int64_t rows = row_end - row_begin;
    if (rows <= 0) return hipSuccess;
    const int64_t blocks = ((rows + kLinBm - 1) / kLinBm) * ((N + kLinBn - 1) / kLinBn);
    // 256 rows of either operand must span < 4 GiB (32-bit per-lane offsets)
    if ((int64_t)kLinBm * K * 2 >= (1LL << 32)) return hipErrorInvalidValue;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    linear_rows_bf16_kernel<<<dim3((unsigned)blocks), 512, 0, st>>>(
        static_cast<const __bf16 *>(a), static_cast<const __bf16 *>(w), static_cast<const __bf16 *>(bias),
        static_cast<__bf16 *>(out), row_begin, row_end, K, N);
    return hipGetLastError();
}

}  // namespace memo
