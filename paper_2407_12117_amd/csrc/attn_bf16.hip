// bf16 causal attention forward/backward for gfx950 (CDNA4), head dim 128.
//
// What is computed (Section 2.1.3 of the paper): O = softmax(scale Q K^T) V under the causal
// mask, tile by tile with per-row running maximum and sum ("compact states"), plus the
// per-row logsumexp; the backward re-forms the probabilities from Q, K and the logsumexp.
//
// Contractions run on the matrix cores with v_mfma_f32_32x32x16_bf16 (fp32 accumulate);
// softmax runs in fp32 on the VALU with exp2 (scale*log2 e folded into one fma).
// Probabilities and dS are rounded to bf16 before their second contraction.
//
// Operand conventions of the 32x32x16 MFMA, D = A(32xK16) * B(K16x32), lane = 32*half + l32:
//   A : lane holds row  l32, k = 8*half .. 8*half+7      (8 bf16)
//   B : lane holds col  l32, k = 8*half .. 8*half+7      (8 bf16)
//   D : lane holds col  l32, rows 8*g + 4*half + r for register v = 4*g + r (16 fp32)
// Every product is arranged so that the per-row softmax quantities sit in ONE lane: the
// score tile is produced with the key index along D's rows and the query index along D's
// columns in the forward and the dQ kernel, and the other way round in the dK/dV kernel.
// The fp32 D registers of the score tile, rounded to bf16, are then directly a B operand
// of the next contraction, whose contraction slot e (0..7) of 16-row chunk q is tile row
//   16*q + 8*(e/4) + 4*half + e%4.
// The matching A operand is a TRANSPOSED read of a row-major LDS tile, done by the LDS
// transpose load ds_read_b64_tr_b16 (two per operand: rows 4*half+0..3 and 8+4*half+0..3).
// All operand reads are issued by hand several MFMAs ahead (see lds_pipeline_* below).
//
// LDS tiles are 64 rows x 128 bf16, row-major, 256 bytes per row, no padding; the sixteen
// 16-byte chunks of row r are stored at chunk position  c ^ swz(r),
//   swz(r) = ((r & 3) << 2) | ((r >> 2) & 3),
// which makes both access patterns bank-conflict free: 16 lanes reading the same chunk of
// 16 consecutive rows (row-major operand), and 32 lanes reading 4 rows x 64 contiguous
// bytes (transposed operand).
#include "bf16_tiles.h"

namespace memo {
namespace {

// ============================================================================ forward
// Workgroup: kFwdWaves waves, 32 query rows per wave; keys/values streamed in tiles of 64 through
// a double-buffered LDS ring filled asynchronously (one barrier per tile).  The more query rows
// share a K/V tile, the less fill traffic (L2 -> LDS) each MFMA has to pay for.
constexpr int kFwdWaves = 8;                 // waves per workgroup in the forward and dQ kernels
constexpr int kFwdBq = 32 * kFwdWaves, kBk = 64;

__global__ __launch_bounds__(64 * kFwdWaves) void attn_fwd_bf16_kernel(AttnArgs a)
{
    __shared__ __attribute__((aligned(1024))) unsigned char smem[4 * kTileBytes];
    LDS_AS unsigned char *lds = (LDS_AS unsigned char *)smem;   // [buf][K|V] tiles

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: lives in a scalar register
    const LaneAddr la = make_lane_addr(lane);
    const int64_t nqt = (a.S + kFwdBq - 1) / kFwdBq;
    const TileId t = decode_block(a, nqt, true);      // heaviest query tiles first
    const int64_t row0 = t.tile * kFwdBq, i0w = row0 + 32 * wave, i = i0w + l32;
    const int64_t base = (int64_t)t.b * a.sb + (int64_t)t.h * a.sh;
    const __bf16 *q = static_cast<const __bf16 *>(a.q) + base;
    const __bf16 *k = static_cast<const __bf16 *>(a.k) + base;
    const __bf16 *v = static_cast<const __bf16 *>(a.v) + base;
    TileStream<kFwdWaves> ks = make_tile_stream<kFwdWaves>(k, a.ss, 0, wave, lane);
    TileStream<kFwdWaves> vs = make_tile_stream<kFwdWaves>(v, a.ss, 0, wave, lane);

    const int64_t last_row = min(row0 + kFwdBq, a.S) - 1;
    const int ntiles = (int)(last_row / kBk) + 1;
    fill_tile_async(lds, ks, k, a.ss, 0, a.S, wave, lane);
    fill_tile_async(lds + kTileBytes, vs, v, a.ss, 0, a.S, wave, lane);

    // Q^T as B operand: lane = query row i, 8 head-dim values per 16-wide chunk
    bf16x8 qB[8];
    {
        const int64_t iq = i < a.S ? i : a.S - 1;     // rows past S are computed and never stored
#pragma unroll
        for (int kc = 0; kc < 8; ++kc)
            qB[kc] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(q + iq * a.ss + 16 * kc + 8 * half));
    }

    f32x16 accO[4];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int e = 0; e < 16; ++e) accO[cb][e] = 0.f;
    float m = -INFINITY, mc = -INFINITY, lsum = 0.f;   // running max of raw dots (and times c), running sum
    const float c = a.scale * kLog2e;
    const int wave_first_tile_masked = (int)((i0w + 31) / kBk) + 1;   // tiles >= this are fully masked
    const int wave_first_diag = (int)(i0w / kBk);                     // tiles >= this need the mask
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const LdsAddr ad = make_lds_addr(lds, la);
    const uint32_t (&row_addr)[8] = ad.row;
    const uint32_t (&tr_addr)[4][2] = ad.tr;

    // One key/value tile.  BUF is a compile-time buffer index, so every LDS address below is
    // a per-lane register plus an immediate offset.
    auto tile_step = [&](auto bufc, int jt) {
        constexpr int BUF = decltype(bufc)::value;
        constexpr int kOff = BUF * 2 * kTileBytes, vOff = kOff + kTileBytes;
        constexpr int nOff = (BUF ^ 1) * 2 * kTileBytes;
        wait_fills();
        __syncthreads();          // tile jt is complete; nobody still reads the other buffer
        if (jt + 1 < ntiles) {
            fill_tile_async(lds + nOff, ks, k, a.ss, (int64_t)(jt + 1) * kBk, a.S, wave, lane);
            fill_tile_async(lds + nOff + kTileBytes, vs, v, a.ss, (int64_t)(jt + 1) * kBk, a.S, wave, lane);
        }
        if (jt >= wave_first_tile_masked) return;     // every key of this tile is masked for this wave

        // S^T tile: rows = 64 keys (2 blocks of 32), cols = this wave's 32 queries.
        // item n = (jb = n%2, kc = n/2): one row operand of K, read 2 MFMAs ahead; the two key blocks
        // alternate, so that no MFMA accumulates onto the result of the one issued right before it
        f32x16 s[2];
        {
            bf16x8 ring[3];
            auto issue = [&](auto n, bf16x8 &slot) {
                constexpr int jb = decltype(n)::value % 2, kc = decltype(n)::value / 2;
                lds_issue_b128<jb * 8192 + kOff>(slot, row_addr[kc]);
            };
            lds_pipeline_prologue<16, 2, 1>(ring, issue);
            lds_pipeline_body<16, 2, 1>(ring, issue, [&](auto n, bf16x8 &slot) {
                constexpr int jb = decltype(n)::value % 2, kc = decltype(n)::value / 2;
                s[jb] = mfma32(slot, qB[kc], kc == 0 ? zero : s[jb]);
            });
        }
        // the first V^T operands are requested now: their latency hides behind the softmax
        TrSlot vring[3];
        auto v_issue = [&](auto n, TrSlot &slot) {
            constexpr int kj = decltype(n)::value / 4, cb = decltype(n)::value % 4;
            lds_issue_tr<kj * 4096 + vOff>(slot, tr_addr[cb][0], tr_addr[cb][1]);
        };
        lds_pipeline_prologue<16, 2, 2>(vring, v_issue);
        if (jt >= wave_first_diag) {                  // diagonal tile: mask keys j > i
            const int thr = (int)(i - (int64_t)jt * kBk) - 4 * half;    // key offset e' is visible iff e' <= thr
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    if (32 * jb + 8 * (e >> 2) + (e & 3) > thr) s[jb][e] = -INFINITY;
        }
        // 32 values in 16 three-input maxima (two chains)
        float mt = fmaxf(fmaxf(s[0][0], s[0][1]), s[0][2]), mu = fmaxf(fmaxf(s[1][0], s[1][1]), s[1][2]);
#pragma unroll
        for (int e = 3; e < 15; e += 2) {
            mt = fmaxf(fmaxf(mt, s[0][e]), s[0][e + 1]);
            mu = fmaxf(fmaxf(mu, s[1][e]), s[1][e + 1]);
        }
        mt = fmaxf(fmaxf(mt, s[0][15]), fmaxf(mu, s[1][15]));
        mt = max_across_halves(mt);
        // Rescale only when some row of the wave sees a new maximum (rare after the first tiles).
        // Every processed tile has key j0 visible to all 32 rows, so the maximum is finite.
        if (__builtin_amdgcn_ballot_w64(mt > m) != 0) {
            const float m_new = fmaxf(m, mt);
            const float corr = __builtin_amdgcn_exp2f((m - m_new) * c);
            m = m_new;
            mc = m_new * c;
            lsum *= corr;
#pragma unroll
            for (int cb = 0; cb < 4; ++cb)
#pragma unroll
                for (int e = 0; e < 16; ++e) accO[cb][e] *= corr;
        }
        float psum0 = 0.f, psum1 = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            s[0][e] = __builtin_amdgcn_exp2f(fmaf(s[0][e], c, -mc));
            s[1][e] = __builtin_amdgcn_exp2f(fmaf(s[1][e], c, -mc));
            psum0 += s[0][e];
            psum1 += s[1][e];
        }
        lsum += psum0 + psum1;

        // O^T += V^T P^T : A = V^T (transposed LDS read), B = P^T straight from the score registers.
        // item n = (kj = n/4, cb = n%4)
        bf16x8 pB[4];
#pragma unroll
        for (int kj = 0; kj < 4; ++kj) pB[kj] = pack8(s[kj >> 1], 8 * (kj & 1));
        lds_pipeline_body<16, 2, 2>(vring, v_issue, [&](auto n, TrSlot &slot) {
            constexpr int kj = decltype(n)::value / 4, cb = decltype(n)::value % 4;
            accO[cb] = mfma32(tr_operand(slot), pB[kj], accO[cb]);
        });
    };

    for (int jt = 0; jt < ntiles; jt += 2) {
        tile_step(IntC<0>{}, jt);
        if (jt + 1 < ntiles) tile_step(IntC<1>{}, jt + 1);
    }

    const float ltot = add_across_halves(lsum);
    if (i < a.S) {
        __bf16 *o = static_cast<__bf16 *>(a.o_out) + base + i * a.ss;
        store_acc_T(o, accO, 1.f / ltot, half);
        if (half == 0)
            a.lse[((int64_t)t.b * a.H + t.h) * a.S + i] = (mc + __builtin_amdgcn_logf(ltot)) * kLn2;
    }
}

// ============================================================================ backward: dQ
// Same shape as the forward: 32 query rows per wave, keys/values streamed.
//   S^T = K Q^T, dP^T = V dO^T, P = exp(S - LSE), dS = P (dP - D), dQ^T += K^T dS^T
__global__ __launch_bounds__(64 * kFwdWaves) void attn_bwd_dq_bf16_kernel(AttnArgs a)
{
    __shared__ __attribute__((aligned(1024))) unsigned char smem[4 * kTileBytes];
    LDS_AS unsigned char *lds = (LDS_AS unsigned char *)smem;   // [buf][K|V] tiles

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: lives in a scalar register
    const LaneAddr la = make_lane_addr(lane);
    const int64_t nqt = (a.S + kFwdBq - 1) / kFwdBq;
    const TileId t = decode_block(a, nqt, true);
    const int64_t row0 = t.tile * kFwdBq, i0w = row0 + 32 * wave, i = i0w + l32;
    const int64_t base = (int64_t)t.b * a.sb + (int64_t)t.h * a.sh;
    const __bf16 *q = static_cast<const __bf16 *>(a.q) + base;
    const __bf16 *k = static_cast<const __bf16 *>(a.k) + base;
    const __bf16 *v = static_cast<const __bf16 *>(a.v) + base;
    const __bf16 *g = static_cast<const __bf16 *>(a.d_o) + base;
    const int64_t stat = ((int64_t)t.b * a.H + t.h) * a.S;
    TileStream<kFwdWaves> ks = make_tile_stream<kFwdWaves>(k, a.ss, 0, wave, lane);
    TileStream<kFwdWaves> vs = make_tile_stream<kFwdWaves>(v, a.ss, 0, wave, lane);

    const int64_t last_row = min(row0 + kFwdBq, a.S) - 1;
    const int ntiles = (int)(last_row / kBk) + 1;
    fill_tile_async(lds, ks, k, a.ss, 0, a.S, wave, lane);
    fill_tile_async(lds + kTileBytes, vs, v, a.ss, 0, a.S, wave, lane);

    const int64_t iq = i < a.S ? i : a.S - 1;         // rows past S are computed and never stored
    bf16x8 qB[8], gB[8];
#pragma unroll
    for (int kc = 0; kc < 8; ++kc) {
        qB[kc] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(q + iq * a.ss + 16 * kc + 8 * half));
        gB[kc] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(g + iq * a.ss + 16 * kc + 8 * half));
    }
    const float c = a.scale * kLog2e;
    const float lse2 = a.lse[stat + iq] * kLog2e;
    // -D_i in all 16 registers of an accumulator: dP^T starts from it, so dP - D_i costs nothing
    const float neg_di = -a.delta[stat + iq];
    f32x16 neg_d;
#pragma unroll
    for (int e = 0; e < 16; ++e) neg_d[e] = neg_di;

    f32x16 accQ[4];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int e = 0; e < 16; ++e) accQ[cb][e] = 0.f;
    const int wave_first_tile_masked = (int)((i0w + 31) / kBk) + 1;
    const int wave_first_diag = (int)(i0w / kBk);
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    const LdsAddr ad = make_lds_addr(lds, la);
    const uint32_t (&row_addr)[8] = ad.row;
    const uint32_t (&tr_addr)[4][2] = ad.tr;

    auto tile_step = [&](auto bufc, int jt) {
        constexpr int BUF = decltype(bufc)::value;
        constexpr int kOff = BUF * 2 * kTileBytes, vOff = kOff + kTileBytes;
        constexpr int nOff = (BUF ^ 1) * 2 * kTileBytes;
        wait_fills();
        __syncthreads();
        if (jt + 1 < ntiles) {
            fill_tile_async(lds + nOff, ks, k, a.ss, (int64_t)(jt + 1) * kBk, a.S, wave, lane);
            fill_tile_async(lds + nOff + kTileBytes, vs, v, a.ss, (int64_t)(jt + 1) * kBk, a.S, wave, lane);
        }
        if (jt >= wave_first_tile_masked) return;
        const bool diag = jt >= wave_first_diag;
        const int thr = (int)(i - (int64_t)jt * kBk) - 4 * half;
        static_for<0, 2>([&](auto jbc) {
            constexpr int jb = decltype(jbc)::value;
            // S^T and dP^T blocks: item n = (kc = n/2, K or V = n%2), row operands read 2 MFMAs ahead
            f32x16 s, dp;
            {
                bf16x8 ring[3];
                auto issue = [&](auto n, bf16x8 &slot) {
                    constexpr int kc = decltype(n)::value / 2, isv = decltype(n)::value % 2;
                    lds_issue_b128<jb * 8192 + (isv ? vOff : kOff)>(slot, row_addr[kc]);
                };
                lds_pipeline_prologue<16, 2, 1>(ring, issue);
                lds_pipeline_body<16, 2, 1>(ring, issue, [&](auto n, bf16x8 &slot) {
                    constexpr int kc = decltype(n)::value / 2, isv = decltype(n)::value % 2;
                    if constexpr (isv) dp = mfma32(slot, gB[kc], kc == 0 ? neg_d : dp);
                    else s = mfma32(slot, qB[kc], kc == 0 ? zero : s);
                });
            }
            // dQ^T += K^T dS^T : A = K^T (transposed read of the same K tile), B = dS^T registers.
            // item n = (sub = n/4, cb = n%4); the first operands are requested before the VALU work
            TrSlot kring[3];
            auto k_issue = [&](auto n, TrSlot &slot) {
                constexpr int sub = decltype(n)::value / 4, cb = decltype(n)::value % 4;
                lds_issue_tr<(2 * jb + sub) * 4096 + kOff>(slot, tr_addr[cb][0], tr_addr[cb][1]);
            };
            lds_pipeline_prologue<8, 2, 2>(kring, k_issue);
            // the mask sits in a block of its own behind a wave-uniform branch: folded into the loop
            // below it became a compare and a select per element on every tile
            if (diag) {
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    if (32 * jb + 8 * (e >> 2) + (e & 3) > thr) s[e] = -INFINITY;
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = __builtin_amdgcn_exp2f(fmaf(s[e], c, -lse2));
                s[e] = p * dp[e];                  // dS (dp already holds dP - D_i)
            }
            bf16x8 dsB[2];
            dsB[0] = pack8(s, 0);
            dsB[1] = pack8(s, 8);
            lds_pipeline_body<8, 2, 2>(kring, k_issue, [&](auto n, TrSlot &slot) {
                constexpr int sub = decltype(n)::value / 4, cb = decltype(n)::value % 4;
                accQ[cb] = mfma32(tr_operand(slot), dsB[sub], accQ[cb]);
            });
        });
    };
    for (int jt = 0; jt < ntiles; jt += 2) {
        tile_step(IntC<0>{}, jt);
        if (jt + 1 < ntiles) tile_step(IntC<1>{}, jt + 1);
    }
    if (i < a.S) {
        __bf16 *dq = static_cast<__bf16 *>(a.dq) + base + i * a.ss;
        store_acc_T(dq, accQ, a.scale, half);
    }
}

constexpr int kBwdBk = 128, kBq = 64;

// ============================================================================ backward: dK, dV
// Workgroup: 8 waves, 128 key rows whose K and V stay in LDS for the workgroup's lifetime;
// queries streamed in tiles of 64 through the double-buffered ring (one barrier per tile).
// Wave w owns the 32 x 32 block (queries 32*(w/4).., keys 32*(w%4)..) of every tile and runs
// all four contractions on it, so nothing passes between waves inside the loop:
//   S = Q K^T, dP = dO V^T (both operands from LDS, the two accumulation chains interleaved)
//   P = exp(S - LSE_i), dS = P (dP - D_i)         (lane = key, 16 query rows per lane)
//   dV^T += dO^T P,  dK^T += Q^T dS                (transposed LDS reads, P / dS from registers)
// Waves w and w+4 hold partial sums for the same keys over disjoint queries; they are added
// through LDS once, after the loop (wave w finishes dV, wave w+4 finishes dK).  No atomics.
struct PairSlot { bf16x8 a, b; };

template <int N>
__device__ __forceinline__ void lds_wait(PairSlot &x)
{
    static_assert(N >= 0 && N <= 15, "lgkmcnt range");
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(x.a), "+v"(x.b) : "n"(N));
}

__global__ __launch_bounds__(512, 2) void attn_bwd_dkdv_bf16_kernel(AttnArgs a)
{
    constexpr int kKsOff = 4 * kTileBytes, kVsOff = 6 * kTileBytes, kStatOff = 8 * kTileBytes;
    // [buf][Q|dO] ring, K rows, V rows (128 x 256 B each), [buf][LSE*log2e | D] rows
    __shared__ __attribute__((aligned(1024))) unsigned char smem[8 * kTileBytes + 1024];
    LDS_AS unsigned char *lds = (LDS_AS unsigned char *)smem;
    LDS_AS float *Stat = (LDS_AS float *)(lds + kStatOff);      // [buf][2][64]

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kb = wave & 3, qh = wave >> 2;
    const LaneAddr la = make_lane_addr(lane);
    const int64_t nkt = (a.S + kBwdBk - 1) / kBwdBk;
    const TileId t = decode_block(a, nkt, false);     // key tile 0 sees every query: heaviest first
    const int64_t col0 = t.tile * kBwdBk, j0w = col0 + 32 * kb, j = j0w + l32;
    const int64_t base = (int64_t)t.b * a.sb + (int64_t)t.h * a.sh;
    const __bf16 *q = static_cast<const __bf16 *>(a.q) + base;
    const __bf16 *g = static_cast<const __bf16 *>(a.d_o) + base;
    const int64_t stat = ((int64_t)t.b * a.H + t.h) * a.S;

    const int it0 = (int)(col0 / kBq);
    const int nit = (int)((a.S + kBq - 1) / kBq);
    {   // resident K and V rows of this key tile (rows past S repeat row S-1, never stored)
        const __bf16 *kp = static_cast<const __bf16 *>(a.k) + base;
        const __bf16 *vp = static_cast<const __bf16 *>(a.v) + base;
        TileStream<8> ks = make_tile_stream<8>(kp, a.ss, col0, wave, lane);
        TileStream<8> vs = make_tile_stream<8>(vp, a.ss, col0, wave, lane);
        fill_tile_async(lds + kKsOff, ks, kp, a.ss, col0, a.S, wave, lane);
        fill_tile_async(lds + kKsOff + kTileBytes, ks, kp, a.ss, col0 + 64, a.S, wave, lane);
        fill_tile_async(lds + kVsOff, vs, vp, a.ss, col0, a.S, wave, lane);
        fill_tile_async(lds + kVsOff + kTileBytes, vs, vp, a.ss, col0 + 64, a.S, wave, lane);
    }
    const TileOffsets<8> toff = make_tile_offsets<8>(a.ss, wave, lane);
    const int64_t tile_step_bytes = kBq * a.ss * 2;
    auto fill_tile = [&](LDS_AS unsigned char *dst, const __bf16 *src, int64_t r0) {
        if (r0 + kBq <= a.S) {
            const char *tb = reinterpret_cast<const char *>(src) + (r0 / kBq) * tile_step_bytes;
            fill_full_tile_part(dst, toff, 0, tb, wave);
            fill_full_tile_part(dst, toff, 1, tb, wave);
        } else {
            fill_ragged_tile<8>(dst, src, a.ss, r0, a.S, wave, lane);
        }
    };
    fill_tile(lds, q, (int64_t)it0 * kBq);
    fill_tile(lds + kTileBytes, g, (int64_t)it0 * kBq);

    const float c = a.scale * kLog2e;
    f32x16 accV[4], accK[4];                          // dV^T, dK^T: lane = key, rows = head dim
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int e = 0; e < 16; ++e) accV[cb][e] = accK[cb][e] = 0.f;
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    // per-row statistics of a query tile: threads 0..63 LSE*log2e, threads 64..127 D_i.
    // rows past S: LSE = +inf makes their probabilities exactly zero
    // The value is loaded raw and only scaled when it is written to LDS a tile later, so that
    // nothing waits for the load (and for the fills queued before it) right after issuing it.
    const float *stat_src = (tid < 64 ? a.lse : a.delta) + stat;
    // D_i is kept negated: it then serves as the initial accumulator of dP, and dP - D_i costs nothing
    const float stat_pad = tid < 64 ? INFINITY : 0.f, stat_mul = tid < 64 ? kLog2e : -1.f;
    auto load_stat = [&](int it) -> float {
        const int64_t r = (int64_t)it * kBq + (tid & 63);
        return (tid < 128 && r < a.S) ? stat_src[r] : stat_pad;
    };
    float sreg = load_stat(it0);
    if (tid < 128) Stat[tid] = sreg * stat_mul;

    const LdsAddr ad = make_lds_addr(lds, la);
    const uint32_t (&row_addr)[8] = ad.row;
    const uint32_t (&tr_addr)[4][2] = ad.tr;
    // this wave's rows of the resident operands and of the ring tiles
    uint32_t kv_addr[8];
#pragma unroll
    for (int kc = 0; kc < 8; ++kc) kv_addr[kc] = row_addr[kc] + (uint32_t)(kKsOff + kb * 8192);

    auto tile_step = [&](auto bufc, int it) {
        constexpr int BUF = decltype(bufc)::value;
        constexpr int qOff = BUF * 2 * kTileBytes, gOff = qOff + kTileBytes;
        constexpr int nOff = (BUF ^ 1) * 2 * kTileBytes;
        const LDS_AS float *Ls = Stat + BUF * 128, *Ds = Ls + 64;
        wait_fills();
        __syncthreads();          // tile `it` and its statistics are complete; the other buffers are free
        const bool more = it + 1 < nit;
        const int64_t rn = (int64_t)(it + 1) * kBq;
        if (more) sreg = load_stat(it + 1);
        // the four fill instructions of the next tile, queued one at a time between the MFMAs
        const int64_t i0 = (int64_t)it * kBq + 32 * qh;           // first query of this wave's block
        const bool active = i0 + 31 >= j0w;           // else all 32 queries precede this wave's keys
        // A full next tile is fetched by four fill instructions queued one at a time between the
        // MFMAs below; the ragged last tile (and a wave with nothing to compute) queues them here.
        const bool spread = more && active && rn + kBq <= a.S;
        if (more && !spread) {
            fill_tile(lds + nOff, q, rn);
            fill_tile(lds + nOff + kTileBytes, g, rn);
        }
        const char *nq = reinterpret_cast<const char *>(q) + (int64_t)(it + 1) * tile_step_bytes;
        const char *ng = reinterpret_cast<const char *>(g) + (int64_t)(it + 1) * tile_step_bytes;
        auto fill_part = [&](auto pc) {
            constexpr int part = decltype(pc)::value;
            if (!spread) return;
            fill_full_tile_part(lds + nOff + (part / 2) * kTileBytes, toff, part % 2, part < 2 ? nq : ng, wave);
        };
        if (active) {
            const bool diag = i0 < j0w + 31;
            const int thr = (int)(j - i0) - 4 * half; // query offset e' is visible iff e' >= thr
            f32x16 s, dp, neg_d;                        // neg_d[e] = -D of query row 8*(e/4) + 4*half + e%4
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const f32x4 d4 = *reinterpret_cast<const LDS_AS f32x4 *>(Ds + 32 * qh + 8 * gq + 4 * half);
#pragma unroll
                for (int r = 0; r < 4; ++r) neg_d[4 * gq + r] = d4[r];
            }
            {
                // item n: k-chunk n/2 of S (even n: Q rows x K rows) or of dP (odd n: dO rows x V rows)
                PairSlot ring[3];
                auto issue = [&](auto n, PairSlot &slot) {
                    constexpr int kc = decltype(n)::value / 2, which = decltype(n)::value % 2;
                    lds_issue_b128<(which ? gOff : qOff)>(slot.a, row_addr[kc] + (uint32_t)(qh * 8192));
                    lds_issue_b128<(which ? kVsOff - kKsOff : 0)>(slot.b, kv_addr[kc]);
                };
                lds_pipeline_prologue<16, 2, 2>(ring, issue);
                lds_pipeline_body<16, 2, 2>(ring, issue, [&](auto n, PairSlot &slot) {
                    constexpr int kc = decltype(n)::value / 2, which = decltype(n)::value % 2;
                    if constexpr (which == 0) s = mfma32(slot.a, slot.b, kc == 0 ? zero : s);
                    else dp = mfma32(slot.a, slot.b, kc == 0 ? neg_d : dp);
                    if constexpr (decltype(n)::value % 4 == 1) fill_part(IntC<decltype(n)::value / 4>{});
                });
            }
            // item n < 8: dV^T block (sub = n/4, cb = n%4), A = dO^T; n >= 8: dK^T, A = Q^T
            TrSlot tring[3];
            auto t_issue = [&](auto n, TrSlot &slot) {
                constexpr int m = decltype(n)::value % 8, sub = m / 4, cb = m % 4;
                constexpr int off = (decltype(n)::value < 8 ? gOff : qOff) + sub * 4096;
                lds_issue_tr<off>(slot, tr_addr[cb][0] + (uint32_t)(qh * 8192), tr_addr[cb][1] + (uint32_t)(qh * 8192));
            };
            lds_pipeline_prologue<16, 2, 2>(tring, t_issue);
            // s, dp: lane = key j, register e = query row i0 + 8*(e/4) + 4*half + e%4
            // the mask sits in a block of its own behind a wave-uniform branch: folded into the loop
            // below it became a compare and a select per element on every tile
            if (diag) {
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    if (8 * (e >> 2) + (e & 3) < thr) s[e] = -INFINITY;
            }
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const f32x4 l4 = *reinterpret_cast<const LDS_AS f32x4 *>(Ls + 32 * qh + 8 * gq + 4 * half);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int e = 4 * gq + r;
                    const float p = __builtin_amdgcn_exp2f(fmaf(s[e], c, -l4[r]));
                    s[e] = p;
                    dp[e] = p * dp[e];                 // dp already holds dP - D_i
                }
            }
            bf16x8 pB[2], dsB[2];
            pB[0] = pack8(s, 0);
            pB[1] = pack8(s, 8);
            dsB[0] = pack8(dp, 0);
            dsB[1] = pack8(dp, 8);
            lds_pipeline_body<16, 2, 2>(tring, t_issue, [&](auto n, TrSlot &slot) {
                constexpr int m = decltype(n)::value % 8, sub = m / 4, cb = m % 4;
                if constexpr (decltype(n)::value < 8) accV[cb] = mfma32(tr_operand(slot), pB[sub], accV[cb]);
                else accK[cb] = mfma32(tr_operand(slot), dsB[sub], accK[cb]);
            });
        }
        if (more && tid < 128) Stat[(BUF ^ 1) * 128 + tid] = sreg * stat_mul;
    };
    for (int it = it0; it < nit; it += 2) {
        tile_step(IntC<0>{}, it);
        if (it + 1 < nit) tile_step(IntC<1>{}, it + 1);
    }

    // Add the two query halves: wave (kb, 0) hands its dK^T to wave (kb, 1) and takes that
    // wave's dV^T, as register images (lane l reads what lane l of the partner wrote).
    __syncthreads();              // every wave is done with the tiles
    {
        LDS_AS f32x4 *mine = (LDS_AS f32x4 *)lds + (size_t)wave * 1024 + lane;          // 16 KB per wave
        LDS_AS f32x4 *theirs = (LDS_AS f32x4 *)lds + (size_t)(wave ^ 4) * 1024 + lane;
        f32x16 (&give)[4] = qh == 0 ? accK : accV;
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const f32x4 x = {give[cb][4 * gq], give[cb][4 * gq + 1], give[cb][4 * gq + 2], give[cb][4 * gq + 3]};
                mine[(cb * 4 + gq) * 64] = x;
            }
        __syncthreads();
        f32x16 (&keep)[4] = qh == 0 ? accV : accK;
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const f32x4 x = theirs[(cb * 4 + gq) * 64];
#pragma unroll
                for (int r = 0; r < 4; ++r) keep[cb][4 * gq + r] += x[r];
            }
        if (j < a.S) {
            __bf16 *out = static_cast<__bf16 *>(qh == 0 ? a.dv : a.dk) + base + j * a.ss;
            store_acc_T(out, keep, qh == 0 ? 1.f : a.scale, half);
        }
    }
}

}  // namespace

hipError_t launch_attn_fwd_bf16(const AttnArgs &a, hipStream_t st)
{
    const int64_t nqt = (a.S + kFwdBq - 1) / kFwdBq;
    const int64_t blocks = nqt * a.H * a.B;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    attn_fwd_bf16_kernel<<<dim3((unsigned)blocks), 64 * kFwdWaves, 0, st>>>(a);
    return hipGetLastError();
}

hipError_t launch_attn_bwd_bf16(const AttnArgs &a, hipStream_t st)
{
    const int64_t nqt = (a.S + kFwdBq - 1) / kFwdBq;
    const int64_t nkt = (a.S + kBwdBk - 1) / kBwdBk;
    if (nkt * a.H * a.B > 0x7fffffffLL) return hipErrorInvalidValue;   // nkt >= nqt; the front end checks too
    hipError_t e = record_stage(a, 0, st);
    if (e != hipSuccess) return e;
    if ((e = launch_attn_delta(a, true, st)) != hipSuccess) return e;
    if ((e = record_stage(a, 1, st)) != hipSuccess) return e;
    attn_bwd_dkdv_bf16_kernel<<<dim3((unsigned)(nkt * a.H * a.B)), 512, 0, st>>>(a);
    if ((e = record_stage(a, 2, st)) != hipSuccess) return e;
    attn_bwd_dq_bf16_kernel<<<dim3((unsigned)(nqt * a.H * a.B)), 64 * kFwdWaves, 0, st>>>(a);
    if ((e = record_stage(a, 3, st)) != hipSuccess) return e;
    return hipGetLastError();
}

}  // namespace memo
