// bf16 causal attention backward for gfx950 (CDNA4), head dim 128, on v_mfma_f32_16x16x32_bf16.
//
// What is computed (Section 2.1.3 of the paper): with P = exp(S - LSE) re-formed from Q, K and the
// logsumexp of the forward, dV = P^T dO, dP = dO V^T, dS = P (dP - D), dK = scale dS^T Q,
// dQ = scale dS K, D_i = dO_i . O_i.  Two kernels: a key-stationary one for dK, dV and a
// query-stationary one for dQ; no atomics, so the gradients are bit-reproducible.  S and dP are
// formed in both (7 contractions for the method's 5): the alternative, one kernel that adds its dQ
// partials to global memory, needs 16 KB of fp32 atomic adds per 32-query step of a 256-key
// workgroup, and this chip retires those at 1.4 TB/s: 2.5 times slower than the dQ kernel they
// would replace.
//
// Why this MFMA shape: the chip is power-limited on random data and the 16x16x32 instruction
// spends less energy per flop than the 32x32x16 one (an MFMA-only loop sustains about an eighth
// more flops per second with it); the wave tiles, and with them the bytes read from LDS per flop,
// are what a 32x32x16 version has.  The backward kernels have no per-row reductions, so the
// smaller accumulator blocks cost no extra vector arithmetic (measured against a 32x32x16 version
// of both kernels: 7 to 10 % faster on N(0,1) inputs).
//
// Operand conventions of the 16x16x32 MFMA, D = A(16xK32) * B(K32x16), lane = 16*g4 + l16:
//   A : lane holds row l16, k = 8*g4 .. 8*g4+7      (8 bf16)
//   B : lane holds col l16, k = 8*g4 .. 8*g4+7      (8 bf16)
//   D : lane holds col l16, rows 4*g4 + r for register r (4 fp32)
// As in the forward kernel every score block is produced so that its fp32 D registers, rounded
// to bf16, are directly the B operand of the next contraction: two D blocks stacked along the
// rows give a lane the 8 contraction slots  e <-> row 16*(e/4) + 4*g4 + e%4  of a 32-row chunk,
// and the matching A operand is two transposed LDS reads (ds_read_b64_tr_b16) of rows
// 4*g4 .. 4*g4+3 and 16 + 4*g4 .. of that chunk.  LDS tiles are rows of 256 bytes (64 per K/V tile
// of the dQ kernel, 32 per Q/dO tile of the dK/dV kernel) with the SwzB chunk swizzle
// (bf16_tiles.h); all operand reads are issued by hand ahead of their MFMAs.
#include "bf16_tiles.h"

namespace memo {
namespace {

constexpr int kDqWaves = 8, kDqBq = 32 * kDqWaves, kBk = 64;
constexpr f32x4 kZero4 = {0.f, 0.f, 0.f, 0.f};

// ============================================================================ backward: dQ
// Workgroup: 8 waves, 32 query rows per wave (two blocks of 16); keys/values streamed in tiles
// of 64 through a double-buffered LDS ring filled asynchronously (one barrier per tile).
//   S^T = K Q^T, dP^T = V dO^T - D   (A = K / V rows from LDS, B = Q^T / dO^T from registers)
//   dS^T = exp(S^T - LSE) dP^T        (lane = query, registers = keys)
//   dQ^T += K^T dS^T                  (A = K^T, transposed LDS read; B = dS^T from registers)
// A tile is worked in two halves of 32 keys so that the element-wise work of one half can run
// under the MFMAs of the other wave of the SIMD.
__global__ __launch_bounds__(64 * kDqWaves) void attn_bwd_dq_bf16_kernel(AttnArgs a)
{
    __shared__ __attribute__((aligned(1024))) unsigned char smem[4 * kTileBytes];
    LDS_AS unsigned char *lds = (LDS_AS unsigned char *)smem;   // [buf][K|V] tiles

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, g4 = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t nqt = (a.S + kDqBq - 1) / kDqBq;
    const PairId t = decode_block_folded(a, nqt);
    if (t.first < 0) return;
    const int64_t base = (int64_t)t.b * a.sb + (int64_t)t.h * a.sh;
    const __bf16 *q = static_cast<const __bf16 *>(a.q) + base;
    const __bf16 *k = static_cast<const __bf16 *>(a.k) + base;
    const __bf16 *v = static_cast<const __bf16 *>(a.v) + base;
    const __bf16 *g = static_cast<const __bf16 *>(a.d_o) + base;
    const int64_t stat = ((int64_t)t.b * a.H + t.h) * a.S;
    const LdsAddr16 ad = make_lds_addr16(lds, lane);
    const float c = a.scale * kLog2e;

    // the heavy tile of the pair sweeps the keys upwards from row 0, the light one downwards to row 0
    for (int pass = 0; pass < 2; ++pass) {
    const int64_t tile = pass == 0 ? (t.second >= 0 ? t.second : t.first) : (t.second >= 0 ? t.first : -1);
    if (tile < 0) break;
    const bool down = pass == 1;
    const int64_t row0 = tile * kDqBq, i0w = row0 + 32 * wave;
    const int64_t last_row = min(row0 + kDqBq, a.S) - 1;
    const int ntiles = (int)(last_row / kBk) + 1;
    const int jfirst = down ? ntiles - 1 : 0, jstep = down ? -1 : 1;
    if (pass) __syncthreads();    // every wave has left the first tile's last LDS buffer
    TileStream<kDqWaves> ks = make_tile_stream<kDqWaves, SwzB>(k, a.ss, (int64_t)jfirst * kBk, wave, lane);
    TileStream<kDqWaves> vs = make_tile_stream<kDqWaves, SwzB>(v, a.ss, (int64_t)jfirst * kBk, wave, lane);
    fill_tile_async<kDqWaves, SwzB>(lds, ks, k, a.ss, (int64_t)jfirst * kBk, a.S, wave, lane, jstep);
    fill_tile_async<kDqWaves, SwzB>(lds + kTileBytes, vs, v, a.ss, (int64_t)jfirst * kBk, a.S, wave, lane, jstep);

    // Q^T and dO^T as B operands: lane = query 16*qt + l16, 8 head-dim values per 32-wide k step
    bf16x8 qB[2][4], gB[2][4];
    float lse2[2];
    f32x4 neg_d[2];               // -D_i in all four registers: dP^T starts from it
    int64_t iq[2];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        const int64_t i = i0w + 16 * qt + l16;
        iq[qt] = i < a.S ? i : a.S - 1;               // rows past S are computed and never stored
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            qB[qt][kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(q + iq[qt] * a.ss + 32 * kk + 8 * g4));
            gB[qt][kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(g + iq[qt] * a.ss + 32 * kk + 8 * g4));
        }
        lse2[qt] = a.lse[stat + iq[qt]] * kLog2e;
        const float nd = -a.delta[stat + iq[qt]];
        neg_d[qt] = f32x4{nd, nd, nd, nd};
    }
    f32x4 accQ[8][2];             // dQ^T: [head-dim block of 16][query block]; lane = query, rows = head dim
#pragma unroll
    for (int dt = 0; dt < 8; ++dt)
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) accQ[dt][qt] = kZero4;
    const int wave_first_tile_masked = (int)((i0w + 31) / kBk) + 1;   // tiles >= this are fully masked
    const int wave_first_diag = (int)(i0w / kBk);                     // tiles >= this need the mask

    auto tile_step = [&](auto bufc, int jt) {
        constexpr int BUF = decltype(bufc)::value;
        constexpr int kOff = BUF * 2 * kTileBytes, vOff = kOff + kTileBytes;
        constexpr int nOff = (BUF ^ 1) * 2 * kTileBytes;
        wait_fills();
        __syncthreads();          // tile jt is complete; nobody still reads the other buffer
        const int jn = jt + jstep;
        if (jn >= 0 && jn < ntiles) {
            fill_tile_async<kDqWaves, SwzB>(lds + nOff, ks, k, a.ss, (int64_t)jn * kBk, a.S, wave, lane, jstep);
            fill_tile_async<kDqWaves, SwzB>(lds + nOff + kTileBytes, vs, v, a.ss, (int64_t)jn * kBk, a.S, wave, lane, jstep);
        }
        if (jt >= wave_first_tile_masked) return;
        const bool diag = jt >= wave_first_diag;
        static_for<0, 2>([&](auto hc) {
            constexpr int h = decltype(hc)::value;    // keys 32*h .. 32*h+31 of the tile: key blocks 2h, 2h+1
            f32x4 s[2][2], dp[2][2];                  // [key block of the half][query block]
            {
                // item n = (k step n/4, key block (n/2)%2, K or V = n%2): one row operand, two MFMAs
                bf16x8 ring[3];
                auto issue = [&](auto n, bf16x8 &slot) {
                    constexpr int kk = decltype(n)::value / 4, kt = (decltype(n)::value / 2) % 2, isv = decltype(n)::value % 2;
                    lds_issue_b128<(2 * h + kt) * 4096 + (isv ? vOff : kOff)>(slot, ad.row16[kk]);
                };
                lds_pipeline_prologue<16, 2, 1>(ring, issue);
                lds_pipeline_body<16, 2, 1>(ring, issue, [&](auto n, bf16x8 &slot) {
                    constexpr int kk = decltype(n)::value / 4, kt = (decltype(n)::value / 2) % 2, isv = decltype(n)::value % 2;
#pragma unroll
                    for (int qt = 0; qt < 2; ++qt) {
                        if constexpr (isv) dp[kt][qt] = mfma16(slot, gB[qt][kk], kk == 0 ? neg_d[qt] : dp[kt][qt]);
                        else s[kt][qt] = mfma16(slot, qB[qt][kk], kk == 0 ? kZero4 : s[kt][qt]);
                    }
                });
            }
            // dQ^T += K^T dS^T over the 32 keys of the half: item n = head-dim block dt, one transposed
            // operand (two reads), two MFMAs; the first operands are requested before the VALU work
            TrSlot kring[3];
            auto k_issue = [&](auto n, TrSlot &slot) {
                constexpr int dt = decltype(n)::value;
                lds_issue_tr_pair<h * 8192 + kOff>(slot, ad.tr16[dt]);
            };
            lds_pipeline_prologue<8, 2, 2>(kring, k_issue);
            if (diag) {           // mask keys beyond the query, behind a wave-uniform branch
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int qt = 0; qt < 2; ++qt) {
                        // key offset in the tile 32h + 16kt + 4g4 + r is visible iff <= query offset
                        const int thr = (int)(i0w + 16 * qt + l16 - (int64_t)jt * kBk) - (32 * h + 16 * kt + 4 * g4);
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (r > thr) s[kt][qt][r] = -INFINITY;
                    }
            }
            bf16x8 dsB[2];
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float p = __builtin_amdgcn_exp2f(fmaf(s[kt][qt][r], c, -lse2[qt]));
                        s[kt][qt][r] = p * dp[kt][qt][r];           // dS (dp already holds dP - D_i)
                    }
                dsB[qt] = pack44(s[0][qt], s[1][qt]);
            }
            lds_pipeline_body<8, 2, 2>(kring, k_issue, [&](auto n, TrSlot &slot) {
                constexpr int dt = decltype(n)::value;
#pragma unroll
                for (int qt = 0; qt < 2; ++qt) accQ[dt][qt] = mfma16(tr_operand(slot), dsB[qt], accQ[dt][qt]);
            });
        });
    };
    for (int n = 0; n < ntiles; n += 2) {
        tile_step(IntC<0>{}, jfirst + jstep * n);
        if (n + 1 < ntiles) tile_step(IntC<1>{}, jfirst + jstep * (n + 1));
    }
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        const int64_t i = i0w + 16 * qt + l16;
        if (i < a.S) {
            __bf16 *dq = static_cast<__bf16 *>(a.dq) + base + i * a.ss + 4 * g4;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) store4(dq + 16 * dt, accQ[dt][qt], a.scale);
        }
    }
    }   // pass
}


// ============================================================================ backward: dK, dV
// Workgroup: 8 waves, 256 key rows whose K and V stay in LDS for the workgroup's lifetime (128 KB);
// queries streamed in tiles of 32 through a double-buffered ring (Q and dO rows, 16 KB per stage,
// one barrier per tile): LDS is full to the byte (160 KB).  The bytes streamed per (query, key) pair
// are (Q + dO bytes per query) / (keys per workgroup): 256 resident keys halve the L2 -> LDS and the
// HBM traffic of a 128-key workgroup for the same work per wave and step.
// Wave w owns key rows 32*w .. 32*w+31 and all 32 queries of every tile, as 2 x 2 blocks of 16, and
// runs all four contractions on its block, so nothing passes between waves:
//   S = Q K^T - LSE/scale, dP = dO V^T - D   (both operands from LDS; lane = key, registers = queries;
//                                             -LSE_i/scale and -D_i are the initial accumulators)
//   P = exp2(scale log2e S), dS = P dP
//   dV^T += dO^T P,  dK^T += Q^T dS  (A = transposed LDS reads over the tile's 32 queries,
//                                     B = P / dS from registers; lane = key, rows = head dim)
// No atomics, no reduction across waves: every wave writes the dK and dV rows of its own keys.
// The row statistics do not pass through LDS (there is no room left): see "Row statistics" below.
constexpr int kBwdBk = 256, kBq = 32;
constexpr int kStageBytes = 2 * kBq * 256;            // Q rows, then dO rows
constexpr int kKvBlockBytes = 2 * 32 * 256;           // per wave: its 32 K rows, then its 32 V rows

struct QuadSlot { bf16x8 a0, a1, b0, b1; };

template <int N>
__device__ __forceinline__ void lds_wait(QuadSlot &x)
{
    static_assert(N >= 0 && N <= 15, "lgkmcnt range");
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(x.a0), "+v"(x.a1), "+v"(x.b0), "+v"(x.b1) : "n"(N));
}

__global__ __launch_bounds__(512, 2) void attn_bwd_dkdv_bf16_kernel(AttnArgs a)
{
    constexpr int kKvOff = 2 * kStageBytes;
    __shared__ __attribute__((aligned(1024))) unsigned char smem[kKvOff + 8 * kKvBlockBytes];   // 160 KB
    LDS_AS unsigned char *lds = (LDS_AS unsigned char *)smem;

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, g4 = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t nkt = (a.S + kBwdBk - 1) / kBwdBk;
    const PairId t = decode_block_folded(a, nkt);     // key tile p (long) and key tile nkt-1-p (short)
    if (t.first < 0) return;
    const int64_t base = (int64_t)t.b * a.sb + (int64_t)t.h * a.sh;
    const __bf16 *q = static_cast<const __bf16 *>(a.q) + base;
    const __bf16 *g = static_cast<const __bf16 *>(a.d_o) + base;
    const float *lse = a.lse + ((int64_t)t.b * a.H + t.h) * a.S;
    const float *dlt = a.delta + ((int64_t)t.b * a.H + t.h) * a.S;
    const int nit = (int)((a.S + kBq - 1) / kBq);
    const float c = a.scale * kLog2e, neg_inv_scale = -1.f / a.scale;
    const TileOffsets<16> toff = make_tile_offsets<16, SwzB>(a.ss, wave, lane);   // a 32-row ring tile is one fill instruction per wave
    const int64_t tile_step_bytes = kBq * a.ss * 2;
    const LdsAddr16 ad = make_lds_addr16(lds, lane);

    // The long tile walks the query tiles downwards from the last one to its diagonal, the short tile
    // upwards from its diagonal to the last one (the sums take the query tiles in any order): the
    // workgroups of a chunk, which share an XCD and its L2, then read the same Q/dO rows at about the
    // same time in both sweeps (bf16_tiles.h, folded order).
    for (int pass = 0; pass < 2; ++pass) {
    const int64_t tile = pass == 0 ? t.first : t.second;
    if (tile < 0) break;
    const int dir = pass == 0 ? -1 : 1;
    const int64_t col0 = tile * kBwdBk, j0w = col0 + 32 * wave;
    const int it0 = (int)(col0 / kBq);                // the tile's first query tile (its diagonal)
    const int it_first = dir > 0 ? it0 : nit - 1, nsteps = nit - it0;
    if (pass) __syncthreads();    // every wave has left the first tile's K, V and ring
    {   // resident K and V rows (rows past S repeat row S-1, never stored): 32-row pieces, 8 waves x 4 rows
        const __bf16 *kp = static_cast<const __bf16 *>(a.k) + base;
        const __bf16 *vp = static_cast<const __bf16 *>(a.v) + base;
        int ln = lane;            // opaque copy: these addresses are formed here, once per sweep, not kept in registers
        asm volatile("" : "+v"(ln));
#pragma unroll
        for (int blk = 0; blk < 8; ++blk) {
            fill_ragged_tile<16, SwzB>(lds + kKvOff + blk * kKvBlockBytes, kp, a.ss, col0 + 32 * blk, a.S, wave, ln);
            fill_ragged_tile<16, SwzB>(lds + kKvOff + blk * kKvBlockBytes + 8192, vp, a.ss, col0 + 32 * blk, a.S, wave, ln);
        }
    }
    auto fill_tile = [&](LDS_AS unsigned char *dst, const __bf16 *src, int64_t r0) {
        if (r0 + kBq <= a.S) {
            fill_full_tile_part(dst, toff, 0, reinterpret_cast<const char *>(src) + (r0 / kBq) * tile_step_bytes, wave);
        } else {
            int ln = lane;        // opaque copy: the addresses of this rare path are formed here, not kept in registers
            asm volatile("" : "+v"(ln));
            fill_ragged_tile<16, SwzB>(dst, src, a.ss, r0, a.S, wave, ln);
        }
    };
    fill_tile(lds, q, (int64_t)it_first * kBq);
    fill_tile(lds + kBq * 256, g, (int64_t)it_first * kBq);

    f32x4 accV[8][2], accK[8][2];                     // dV^T, dK^T: [head-dim block][key block]; lane = key
#pragma unroll
    for (int dt = 0; dt < 8; ++dt)
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) accV[dt][kt] = accK[dt][kt] = kZero4;

    // Row statistics.  The accumulator registers of lane 16*g4 + l16 stand for queries 4*g4 .. 4*g4+3 of a
    // 16-query block, so the lane needs -LSE_i/scale and -D_i of those four queries as the initial value
    // of S and dP: sixteen values per step.  Fetching them as such (from global memory or through LDS)
    // returns 64 bytes per lane and step to the registers, which costs the step 6 %.  Instead lane l
    // loads ONE value per block and statistic, that of query 4*(l/16) + l%4, and a 4x4x1 fp32 MFMA
    // (sixteen independent 4x4 outer products, block = l/4) spreads it: with B = the scaling constant in
    // every lane, register r of lane l receives A of lane 4*(l/4) + r, which is query 4*(l/16) + r.
    // The product is one fp32 multiplication, the same rounding as a v_mul.  Rows past S: LSE = +inf
    // makes their P exactly zero.
    const int stat_lane = 4 * g4 + (lane & 3);
    struct RawStats { float l[2], d[2]; };
    auto load_stats = [&](int it) {
        RawStats r;
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            const int64_t row = (int64_t)it * kBq + 16 * qt + stat_lane;
            r.l[qt] = row < a.S ? lse[row] : INFINITY;
            r.d[qt] = row < a.S ? dlt[row] : 0.f;
        }
        return r;
    };
    f32x4 nl[2], nd[2];           // -LSE_i/scale and -D_i of the tile about to be worked
    auto spread_stats = [&](const RawStats &r) {
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            nl[qt] = __builtin_amdgcn_mfma_f32_4x4x1f32(r.l[qt], neg_inv_scale, kZero4, 0, 0, 0);
            nd[qt] = __builtin_amdgcn_mfma_f32_4x4x1f32(r.d[qt], -1.f, kZero4, 0, 0, 0);
        }
    };
    RawStats raw = load_stats(it_first);

    uint32_t kv_row[4];                               // this wave's K rows; its V rows are 8192 bytes further
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) kv_row[kk] = ad.row16[kk] + (uint32_t)(kKvOff + wave * kKvBlockBytes);
    const uint32_t (&q_row)[4] = ad.row16;            // query rows of ring stage 0 (Q part)
    const uint32_t (&q_tr)[8] = ad.tr16;

    auto tile_step = [&](auto bufc, int it, bool more) {
        constexpr int BUF = decltype(bufc)::value;
        constexpr int qOff = BUF * kStageBytes, gOff = qOff + kBq * 256;
        constexpr int nOff = (BUF ^ 1) * kStageBytes;
        wait_fills();
        __syncthreads();          // tile `it` is complete; the other stage is free
        const int64_t rn = (int64_t)(it + dir) * kBq;   // first query of the next tile (if there is one)
        const int64_t i0 = (int64_t)it * kBq;         // first query of the tile
        const RawStats raw_now = raw;
        if (more) raw = load_stats(it + dir);         // four registers, used a whole step from now
        const bool active = i0 + 31 >= j0w;           // else all 32 queries precede this wave's keys
        // A full next tile is fetched by two fill instructions queued one at a time between the
        // MFMAs below; the ragged last tile (and a wave with nothing to compute) queues them here.
        const bool spread = more && active && rn + kBq <= a.S;
        if (more && !spread) {
            fill_tile(lds + nOff, q, rn);
            fill_tile(lds + nOff + kBq * 256, g, rn);
        }
        const char *nq = reinterpret_cast<const char *>(q) + (int64_t)(it + dir) * tile_step_bytes;
        const char *ng = reinterpret_cast<const char *>(g) + (int64_t)(it + dir) * tile_step_bytes;
        auto fill_part = [&](auto pc) {
            constexpr int part = decltype(pc)::value;
            if (!spread) return;
            fill_full_tile_part(lds + nOff + part * kBq * 256, toff, 0, part == 0 ? nq : ng, wave);
        };
        if (active) {
            spread_stats(raw_now);
            const bool diag = i0 < j0w + 31;
            f32x4 s[2][2], dp[2][2];                  // [query block][key block]; register r = query 16*qt + 4*g4 + r
            {
                // item n = (k step n/2, S or dP = n%2): the Q (dO) rows of both query blocks and the
                // K (V) rows of both key blocks, four MFMAs
                QuadSlot ring[2];
                auto issue = [&](auto n, QuadSlot &slot) {
                    constexpr int kk = decltype(n)::value / 2, which = decltype(n)::value % 2;
                    lds_issue_b128<(which ? gOff : qOff)>(slot.a0, q_row[kk]);
                    lds_issue_b128<(which ? gOff : qOff) + 4096>(slot.a1, q_row[kk]);
                    lds_issue_b128<(which ? 8192 : 0)>(slot.b0, kv_row[kk]);
                    lds_issue_b128<(which ? 8192 : 0) + 4096>(slot.b1, kv_row[kk]);
                };
                lds_pipeline_prologue<8, 1, 4>(ring, issue);
                lds_pipeline_body<8, 1, 4>(ring, issue, [&](auto n, QuadSlot &slot) {
                    constexpr int kk = decltype(n)::value / 2, which = decltype(n)::value % 2;
                    if constexpr (which == 0) {
                        s[0][0] = mfma16(slot.a0, slot.b0, kk == 0 ? nl[0] : s[0][0]);
                        s[0][1] = mfma16(slot.a0, slot.b1, kk == 0 ? nl[0] : s[0][1]);
                        s[1][0] = mfma16(slot.a1, slot.b0, kk == 0 ? nl[1] : s[1][0]);
                        s[1][1] = mfma16(slot.a1, slot.b1, kk == 0 ? nl[1] : s[1][1]);
                    } else {
                        dp[0][0] = mfma16(slot.a0, slot.b0, kk == 0 ? nd[0] : dp[0][0]);
                        dp[0][1] = mfma16(slot.a0, slot.b1, kk == 0 ? nd[0] : dp[0][1]);
                        dp[1][0] = mfma16(slot.a1, slot.b0, kk == 0 ? nd[1] : dp[1][0]);
                        dp[1][1] = mfma16(slot.a1, slot.b1, kk == 0 ? nd[1] : dp[1][1]);
                    }
                    if constexpr (decltype(n)::value == 3) fill_part(IntC<0>{});
                    if constexpr (decltype(n)::value == 7) fill_part(IntC<1>{});
                });
            }
            // item n < 8: dV^T head-dim block n, A = dO^T; n >= 8: dK^T block n - 8, A = Q^T
            TrSlot tring[3];
            auto t_issue = [&](auto n, TrSlot &slot) {
                constexpr int dt = decltype(n)::value % 8;
                constexpr int off = decltype(n)::value < 8 ? gOff : qOff;
                lds_issue_tr_pair<off>(slot, q_tr[dt]);
            };
            lds_pipeline_prologue<16, 2, 2>(tring, t_issue);
            if (diag) {           // the causal mask, behind a wave-uniform branch
#pragma unroll
                for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                    for (int kt = 0; kt < 2; ++kt) {
                        // query offset 16qt + 4g4 + r of the tile is visible to key j iff it is >= j - i0
                        const int thr = (int)(j0w + 16 * kt + l16 - i0) - (16 * qt + 4 * g4);
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (r < thr) s[qt][kt][r] = -INFINITY;
                    }
            }
#pragma unroll
            for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float p = __builtin_amdgcn_exp2f(s[qt][kt][r] * c);   // s already holds S - LSE_i/scale
                        s[qt][kt][r] = p;
                        dp[qt][kt][r] = p * dp[qt][kt][r];                          // dp already holds dP - D_i
                    }
            bf16x8 pB[2], dsB[2];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                pB[kt] = pack44(s[0][kt], s[1][kt]);
                dsB[kt] = pack44(dp[0][kt], dp[1][kt]);
            }
            lds_pipeline_body<16, 2, 2>(tring, t_issue, [&](auto n, TrSlot &slot) {
                constexpr int dt = decltype(n)::value % 8;
#pragma unroll
                for (int kt = 0; kt < 2; ++kt) {
                    if constexpr (decltype(n)::value < 8) accV[dt][kt] = mfma16(tr_operand(slot), pB[kt], accV[dt][kt]);
                    else accK[dt][kt] = mfma16(tr_operand(slot), dsB[kt], accK[dt][kt]);
                }
            });
        }
    };
    for (int n = 0; n < nsteps; n += 2) {
        tile_step(IntC<0>{}, it_first + dir * n, n + 1 < nsteps);
        if (n + 1 < nsteps) tile_step(IntC<1>{}, it_first + dir * (n + 1), n + 2 < nsteps);
    }

    int g4e = g4;                 // opaque copy: the output addresses are formed here, once per sweep, not kept in registers
    asm volatile("" : "+v"(g4e));
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
        const int64_t j = j0w + 16 * kt + l16;
        if (j < a.S) {
            __bf16 *dv = static_cast<__bf16 *>(a.dv) + base + j * a.ss + 4 * g4e;
            __bf16 *dk = static_cast<__bf16 *>(a.dk) + base + j * a.ss + 4 * g4e;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
                store4(dv + 16 * dt, accV[dt][kt], 1.f);
                store4(dk + 16 * dt, accK[dt][kt], a.scale);
            }
        }
    }
    }   // pass
}

}  // namespace

// D_i preprocess, then the key-stationary kernel (dK, dV), then the query-stationary one (dQ); events
// between the stages when the caller asked for them.
hipError_t launch_attn_bwd_bf16(const AttnArgs &a, hipStream_t st)
{
    const int64_t hb = (int64_t)a.H * a.B;
    const int64_t nkt = (a.S + kBwdBk - 1) / kBwdBk, nqt = (a.S + kDqBq - 1) / kDqBq;
    const int64_t dq_blocks = folded_grid(nqt, hb);
    const int64_t dkdv_blocks = folded_grid(nkt, hb);
    if (dkdv_blocks > 0x7fffffffLL || dq_blocks > 0x7fffffffLL) return hipErrorInvalidValue;   // the front end checks too
    hipError_t e = record_stage(a, 0, st);
    if (e != hipSuccess) return e;
    if ((e = launch_attn_delta(a, true, st)) != hipSuccess) return e;
    if ((e = record_stage(a, 1, st)) != hipSuccess) return e;
    attn_bwd_dkdv_bf16_kernel<<<dim3((unsigned)dkdv_blocks), 512, 0, st>>>(a);
    if ((e = record_stage(a, 2, st)) != hipSuccess) return e;
    attn_bwd_dq_bf16_kernel<<<dim3((unsigned)dq_blocks), 64 * kDqWaves, 0, st>>>(a);
    if ((e = record_stage(a, 3, st)) != hipSuccess) return e;
    return hipGetLastError();
}

}  // namespace memo
