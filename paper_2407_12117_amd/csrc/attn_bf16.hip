// bf16 causal attention forward for gfx950 (CDNA4), head dim 128 (the backward is attn_bwd_bf16.hip).
//
// What is computed (Section 2.1.3 of the paper): O = softmax(scale Q K^T) V under the causal
// mask, tile by tile with per-row running maximum and sum ("compact states"), plus the
// per-row logsumexp that the backward re-forms the probabilities from.
//
// Contractions run on the matrix cores with v_mfma_f32_32x32x16_bf16 (fp32 accumulate);
// softmax runs in fp32 on the VALU with exp2 (scale*log2 e folded into one fma).
// Probabilities are rounded to bf16 before the second contraction.
//
// Operand conventions of the 32x32x16 MFMA, D = A(32xK16) * B(K16x32), lane = 32*half + l32:
//   A : lane holds row  l32, k = 8*half .. 8*half+7      (8 bf16)
//   B : lane holds col  l32, k = 8*half .. 8*half+7      (8 bf16)
//   D : lane holds col  l32, rows 8*g + 4*half + r for register v = 4*g + r (16 fp32)
// Every product is arranged so that the per-row softmax quantities sit in ONE lane: the
// score tile is produced with the key index along D's rows and the query index along D's
// columns.
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
constexpr int kFwdWaves = 8;                 // waves per workgroup
constexpr int kFwdBq = 32 * kFwdWaves, kBk = 64;
// A lane's 32 exponentials of a tile may sum to this much before the running maximum is brought up to
// date: 2^40 per tile leaves the row sum over 2^20 keys and the output accumulators far inside fp32.
constexpr float kRescaleAbove = 1099511627776.f;

__global__ __launch_bounds__(64 * kFwdWaves) void attn_fwd_bf16_kernel(AttnArgs a)
{
    __shared__ __attribute__((aligned(1024))) unsigned char smem[4 * kTileBytes];
    LDS_AS unsigned char *lds = (LDS_AS unsigned char *)smem;   // [buf][K|V] tiles

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: lives in a scalar register
    const LaneAddr la = make_lane_addr(lane);
    const int64_t nqt = (a.S + kFwdBq - 1) / kFwdBq;
    const PairId t = decode_block_folded(a, nqt);
    if (t.first < 0) return;
    const int64_t base = (int64_t)t.b * a.sb + (int64_t)t.h * a.sh;
    const __bf16 *q = static_cast<const __bf16 *>(a.q) + base;
    const __bf16 *k = static_cast<const __bf16 *>(a.k) + base;
    const __bf16 *v = static_cast<const __bf16 *>(a.v) + base;
    const float c = a.scale * kLog2e;
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const LdsAddr ad = make_lds_addr(lds, la);
    const uint32_t (&row_addr)[8] = ad.row;
    const uint32_t (&tr_addr)[4][2] = ad.tr;

    // the heavy tile of the pair sweeps the keys upwards from row 0, the light one downwards to row 0
    // (online softmax takes the key tiles in any order)
    for (int pass = 0; pass < 2; ++pass) {
    const int64_t tile = pass == 0 ? (t.second >= 0 ? t.second : t.first) : (t.second >= 0 ? t.first : -1);
    if (tile < 0) break;
    const int64_t row0 = tile * kFwdBq, i0w = row0 + 32 * wave, i = i0w + l32;
    const int64_t last_row = min(row0 + kFwdBq, a.S) - 1;
    const int ntiles = (int)(last_row / kBk) + 1;
    const int jfirst = pass ? ntiles - 1 : 0, jstep = pass ? -1 : 1;
    if (pass) __syncthreads();    // every wave has left the first tile's last LDS buffer
    TileStream<kFwdWaves> ks = make_tile_stream<kFwdWaves>(k, a.ss, (int64_t)jfirst * kBk, wave, lane);
    TileStream<kFwdWaves> vs = make_tile_stream<kFwdWaves>(v, a.ss, (int64_t)jfirst * kBk, wave, lane);
    fill_tile_async(lds, ks, k, a.ss, (int64_t)jfirst * kBk, a.S, wave, lane, jstep);
    fill_tile_async(lds + kTileBytes, vs, v, a.ss, (int64_t)jfirst * kBk, a.S, wave, lane, jstep);

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
    const int wave_first_tile_masked = (int)((i0w + 31) / kBk) + 1;   // tiles >= this are fully masked
    const int wave_first_diag = (int)(i0w / kBk);                     // tiles >= this need the mask

    // One key/value tile.  BUF is a compile-time buffer index, so every LDS address below is
    // a per-lane register plus an immediate offset.
    auto tile_step = [&](auto bufc, int jt) {
        constexpr int BUF = decltype(bufc)::value;
        constexpr int kOff = BUF * 2 * kTileBytes, vOff = kOff + kTileBytes;
        constexpr int nOff = (BUF ^ 1) * 2 * kTileBytes;
        wait_fills();
        __syncthreads();          // tile jt is complete; nobody still reads the other buffer
        const int jn = jt + jstep;
        if (jn >= 0 && jn < ntiles) {
            fill_tile_async(lds + nOff, ks, k, a.ss, (int64_t)jn * kBk, a.S, wave, lane, jstep);
            fill_tile_async(lds + nOff + kTileBytes, vs, v, a.ss, (int64_t)jn * kBk, a.S, wave, lane, jstep);
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
        // P^T = exp2(c S^T - c m) against the running maximum m AS IT STANDS, rounded to bf16 for the second
        // contraction, and its row sums.  Softmax does not need the true maximum, only one that keeps the
        // exponentials in range: O and the logsumexp come out of (accO, lsum, m) the same whatever m is, and
        // fp32 and bf16 keep their relative precision at any exponent.  So the maximum of the tile is not
        // formed at all (16 three-input maxima, an exchange between the half-waves, and the exponentials
        // waiting for both) unless some row sum shows a score far above m, which also covers the first
        // tile, where m = -inf gives +inf or NaN here.
        bf16x8 pB[4];
        float psum0, psum1;
        auto exponentials = [&]() __attribute__((always_inline)) {
            psum0 = psum1 = 0.f;
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int e = 0; e < 16; e += 2) {
                    const f32x2 two = {__builtin_amdgcn_exp2f(fmaf(s[jb][e], c, -mc)), __builtin_amdgcn_exp2f(fmaf(s[jb][e + 1], c, -mc))};
                    psum0 += two[0];
                    psum1 += two[1];
                    const bf16x2 r = __builtin_convertvector(two, bf16x2);
                    pB[2 * jb + (e >> 3)][e & 7] = r[0];
                    pB[2 * jb + (e >> 3)][(e & 7) + 1] = r[1];
                }
        };
        exponentials();
        // not (sum <= bound) rather than sum > bound: a NaN sum takes the careful path too
        if (__builtin_amdgcn_ballot_w64(!(psum0 + psum1 <= kRescaleAbove)) != 0) {
            // 32 values in 16 three-input maxima (two chains)
            float mt = fmaxf(fmaxf(s[0][0], s[0][1]), s[0][2]), mu = fmaxf(fmaxf(s[1][0], s[1][1]), s[1][2]);
#pragma unroll
            for (int e = 3; e < 15; e += 2) {
                mt = fmaxf(fmaxf(mt, s[0][e]), s[0][e + 1]);
                mu = fmaxf(fmaxf(mu, s[1][e]), s[1][e + 1]);
            }
            mt = fmaxf(fmaxf(mt, s[0][15]), fmaxf(mu, s[1][15]));
            mt = max_across_halves(mt);
            // Every processed tile has key j0 visible to all 32 rows, so the maximum is finite.
            const float m_new = fmaxf(m, mt);
            const float corr = __builtin_amdgcn_exp2f((m - m_new) * c);
            m = m_new;
            mc = m_new * c;
            lsum *= corr;
#pragma unroll
            for (int cb = 0; cb < 4; ++cb)
#pragma unroll
                for (int e = 0; e < 16; ++e) accO[cb][e] *= corr;
            exponentials();
        }
        lsum += psum0 + psum1;

        // O^T += V^T P^T : A = V^T (transposed LDS read), B = P^T straight from the score registers.
        // item n = (kj = n/4, cb = n%4)
        lds_pipeline_body<16, 2, 2>(vring, v_issue, [&](auto n, TrSlot &slot) {
            constexpr int kj = decltype(n)::value / 4, cb = decltype(n)::value % 4;
            accO[cb] = mfma32(tr_operand(slot), pB[kj], accO[cb]);
        });
    };

    for (int n = 0; n < ntiles; n += 2) {
        tile_step(IntC<0>{}, jfirst + jstep * n);
        if (n + 1 < ntiles) tile_step(IntC<1>{}, jfirst + jstep * (n + 1));
    }

    const float ltot = add_across_halves(lsum);
    if (i < a.S) {
        __bf16 *o = static_cast<__bf16 *>(a.o_out) + base + i * a.ss;
        store_acc_T(o, accO, 1.f / ltot, half);
        if (half == 0)
            a.lse[((int64_t)t.b * a.H + t.h) * a.S + i] = (mc + __builtin_amdgcn_logf(ltot)) * kLn2;
    }
    }   // pass
}

}  // namespace

hipError_t launch_attn_fwd_bf16(const AttnArgs &a, hipStream_t st)
{
    const int64_t nqt = (a.S + kFwdBq - 1) / kFwdBq;
    const int64_t blocks = folded_grid(nqt, (int64_t)a.H * a.B);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    attn_fwd_bf16_kernel<<<dim3((unsigned)blocks), 64 * kFwdWaves, 0, st>>>(a);
    return hipGetLastError();
}

}  // namespace memo
