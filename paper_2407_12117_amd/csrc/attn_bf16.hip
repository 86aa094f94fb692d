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
//
// LDS tiles are 64 rows x 128 bf16, row-major, 256 bytes per row, no padding; the sixteen
// 16-byte chunks of row r are stored at chunk position  c ^ swz(r),
//   swz(r) = ((r & 3) << 2) | ((r >> 2) & 3),
// which makes both access patterns bank-conflict free: 16 lanes reading the same chunk of
// 16 consecutive rows (row-major operand), and 32 lanes reading 4 rows x 64 contiguous
// bytes (transposed operand).
#include "memo_kernels.h"
#include <hip/hip_bf16.h>

namespace memo {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
#define LDS_AS __attribute__((address_space(3)))

constexpr int kTileBytes = 64 * 256;   // one 64 x 128 bf16 tile
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

// ---- per-lane LDS addressing ---------------------------------------------------------
struct LaneAddr {
    int row_op[8];      // row-major operand: byte offset of (row l32, chunk 2*kc+half), kc = 0..7
    int tr_op[4][2];    // transposed operand: [column block cb][second 4-row group]
};

__device__ __forceinline__ LaneAddr make_lane_addr(int lane)
{
    LaneAddr la;
    const int l32 = lane & 31, half = lane >> 5;
    const int hg = half ^ swz(l32);           // rows 32*b + l32 share swz(l32 & 15)
#pragma unroll
    for (int kc = 0; kc < 8; ++kc) la.row_op[kc] = l32 * 256 + (((2 * kc) ^ hg) << 4);
    // transposed read: inside each group of 16 lanes, lane i16 supplies the address of row
    // base + i16/4, columns 4*(i16%4).. of its 16-column slab, and receives column i16.
    const int i16 = lane & 15, slab = (lane >> 4) & 1;
    const int rr = i16 >> 2;                  // row within the 4-row group
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int sec = 0; sec < 2; ++sec) {
            const int row = 4 * half + rr + 8 * sec;               // + 16*q added by the caller
            const int chunk = 4 * cb + 2 * slab + ((i16 >> 1) & 1);
            la.tr_op[cb][sec] = row * 256 + ((chunk ^ swz(row)) << 4) + 8 * (i16 & 1);
        }
    return la;
}

__device__ __forceinline__ bf16x8 lds_row_operand(const LDS_AS unsigned char *tile, int off)
{
    return *reinterpret_cast<const LDS_AS bf16x8 *>(tile + off);
}

// 8 contraction slots of chunk q (16 tile rows) for tile column 32*cb + l32
__device__ __forceinline__ bf16x8 lds_tr_operand(const LDS_AS unsigned char *tile, const LaneAddr &la,
                                                 int cb, int q)
{
    // rows 16q .. 16q+15 keep swz() of rows 0..15, so q only adds 16*256 bytes
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (LDS_AS s16x4 *)(tile + la.tr_op[cb][0] + q * 4096));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (LDS_AS s16x4 *)(tile + la.tr_op[cb][1] + q * 4096));
    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

// 8 fp32 -> 8 bf16 (round to nearest even)
__device__ __forceinline__ bf16x8 pack8(const f32x16 &x, int first)
{
    bf16x8 out;
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
        f32x2 two = {x[first + e], x[first + e + 1]};
        bf16x2 r = __builtin_convertvector(two, bf16x2);
        out[e] = r[0];
        out[e + 1] = r[1];
    }
    return out;
}

// ---- staging of a 64-row x 128-col bf16 tile by 256 threads ---------------------------
// 16-byte global loads (16 lanes cover one 256-byte row), rows beyond S read as zero.
struct RowRegs { u32x4 r[4]; };

__device__ __forceinline__ void load_rows(RowRegs &t, const __bf16 *src, int64_t ss, int64_t r0,
                                          int64_t S, int tid)
{
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        const int r = 16 * n + (tid >> 4), c16 = tid & 15;
        t.r[n] = u32x4{0u, 0u, 0u, 0u};
        if (r0 + r < S) t.r[n] = *reinterpret_cast<const u32x4 *>(src + (r0 + r) * ss + c16 * 8);
    }
}

__device__ __forceinline__ void store_rows(LDS_AS unsigned char *tile, const RowRegs &t, int tid)
{
    // row 16n + tid/16 has the same swz() for every n
    const int r = tid >> 4, c16 = tid & 15;
    const int off = r * 256 + ((c16 ^ swz(r)) << 4);
#pragma unroll
    for (int n = 0; n < 4; ++n) *reinterpret_cast<LDS_AS u32x4 *>(tile + off + n * 4096) = t.r[n];
}

// Writes a 32(col i) x 128(row c) fp32 accumulator set held as acc[cb][v] (D layout with
// c along the rows) to out[i][c] as bf16, scaled.  4 consecutive c per 8-byte store.
__device__ __forceinline__ void store_acc_T(__bf16 *out_row, const f32x16 (&acc)[4], float mul,
                                            int half)
{
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            f32x2 a = {acc[cb][4 * g] * mul, acc[cb][4 * g + 1] * mul};
            f32x2 b = {acc[cb][4 * g + 2] * mul, acc[cb][4 * g + 3] * mul};
            u32x2 w;
            w[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(a, bf16x2));
            w[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(b, bf16x2));
            *reinterpret_cast<u32x2 *>(out_row + 32 * cb + 8 * g + 4 * half) = w;
        }
}

// Workgroup id -> (tile, head, batch).  Consecutive ids, which the dispatcher deals
// round-robin to the 8 XCDs, differ in the head, so with 1, 2, 4 or 8 heads every XCD's
// L2 streams one head's tensors.  `reverse` issues the highest tile index first.
struct TileId { int64_t tile; int h, b; };
__device__ __forceinline__ TileId decode_block(const AttnArgs &a, int64_t ntiles, bool reverse)
{
    const int64_t hb = (int64_t)a.H * a.B;
    const int64_t id = blockIdx.x;
    TileId t;
    const int64_t ord = id / hb;
    t.tile = reverse ? ntiles - 1 - ord : ord;
    const int rem = (int)(id % hb);
    t.h = rem % a.H;
    t.b = rem / a.H;
    return t;
}

// ============================================================================ forward
// Workgroup: 4 waves, 128 query rows (32 per wave); keys/values streamed in tiles of 64.
constexpr int kFwdBq = 128, kBk = 64;

__global__ __launch_bounds__(256, 2) void attn_fwd_bf16_kernel(AttnArgs a)
{
    __shared__ __attribute__((aligned(256))) unsigned char smem[2 * kTileBytes];
    LDS_AS unsigned char *Ks = (LDS_AS unsigned char *)smem;
    LDS_AS unsigned char *Vs = Ks + kTileBytes;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const LaneAddr la = make_lane_addr(lane);
    const int64_t nqt = (a.S + kFwdBq - 1) / kFwdBq;
    const TileId t = decode_block(a, nqt, true);      // heaviest query tiles first
    const int64_t row0 = t.tile * kFwdBq, i0w = row0 + 32 * wave, i = i0w + l32;
    const int64_t base = (int64_t)t.b * a.sb + (int64_t)t.h * a.sh;
    const __bf16 *q = static_cast<const __bf16 *>(a.q) + base;
    const __bf16 *k = static_cast<const __bf16 *>(a.k) + base;
    const __bf16 *v = static_cast<const __bf16 *>(a.v) + base;

    // Q^T as B operand: lane = query row i, 8 head-dim values per 16-wide chunk
    bf16x8 qB[8];
#pragma unroll
    for (int kc = 0; kc < 8; ++kc) {
        u32x4 raw = {0u, 0u, 0u, 0u};
        if (i < a.S) raw = *reinterpret_cast<const u32x4 *>(q + i * a.ss + 16 * kc + 8 * half);
        qB[kc] = __builtin_bit_cast(bf16x8, raw);
    }

    f32x16 accO[4];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int e = 0; e < 16; ++e) accO[cb][e] = 0.f;
    float m = -INFINITY, lsum = 0.f;          // running max of raw dots, running sum (per lane half)
    const float c = a.scale * kLog2e;

    const int64_t last_row = min(row0 + kFwdBq, a.S) - 1;
    const int64_t ntiles = last_row / kBk + 1;

    RowRegs kreg, vreg;
    load_rows(kreg, k, a.ss, 0, a.S, tid);
    load_rows(vreg, v, a.ss, 0, a.S, tid);

    for (int64_t jt = 0; jt < ntiles; ++jt) {
        const int64_t j0 = jt * kBk;
        __syncthreads();                      // previous tile fully consumed
        store_rows(Ks, kreg, tid);
        store_rows(Vs, vreg, tid);
        __syncthreads();
        if (jt + 1 < ntiles) {
            load_rows(kreg, k, a.ss, j0 + kBk, a.S, tid);
            load_rows(vreg, v, a.ss, j0 + kBk, a.S, tid);
        }
        if (j0 > i0w + 31) continue;          // every key of this tile is masked for this wave

        // S^T tile: rows = 64 keys (2 blocks of 32), cols = this wave's 32 queries
        f32x16 s[2];
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
#pragma unroll
            for (int e = 0; e < 16; ++e) s[jb][e] = 0.f;
#pragma unroll
            for (int kc = 0; kc < 8; ++kc)
                s[jb] = mfma32(lds_row_operand(Ks, la.row_op[kc] + jb * 8192), qB[kc], s[jb]);
        }
        if (j0 + kBk - 1 > i0w) {             // diagonal tile: mask keys j > i
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int64_t j = j0 + 32 * jb + 8 * (e >> 2) + 4 * half + (e & 3);
                    if (j > i) s[jb][e] = -INFINITY;
                }
        }
        float mt = s[0][0];
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int e = 0; e < 16; ++e) mt = fmaxf(mt, s[jb][e]);
        mt = fmaxf(mt, __shfl_xor(mt, 32));
        // every processed tile has j0 <= i for all 32 rows of the wave, so m_new is finite
        const float m_new = fmaxf(m, mt);
        const float corr = __builtin_amdgcn_exp2f((m - m_new) * c);
        const float mc = m_new * c;
        m = m_new;
        float psum = 0.f;
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                s[jb][e] = __builtin_amdgcn_exp2f(fmaf(s[jb][e], c, -mc));
                psum += s[jb][e];
            }
        lsum = lsum * corr + psum;
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
#pragma unroll
            for (int e = 0; e < 16; ++e) accO[cb][e] *= corr;

        // O^T += V^T P^T : A = V^T (transposed LDS read), B = P^T straight from the score registers
#pragma unroll
        for (int kj = 0; kj < 4; ++kj) {
            const bf16x8 pB = pack8(s[kj >> 1], 8 * (kj & 1));
#pragma unroll
            for (int cb = 0; cb < 4; ++cb)
                accO[cb] = mfma32(lds_tr_operand(Vs, la, cb, kj), pB, accO[cb]);
        }
    }

    const float ltot = lsum + __shfl_xor(lsum, 32);
    if (i < a.S) {
        __bf16 *o = static_cast<__bf16 *>(a.o_out) + base + i * a.ss;
        store_acc_T(o, accO, 1.f / ltot, half);
        if (half == 0)
            a.lse[((int64_t)t.b * a.H + t.h) * a.S + i] = (m * c + __builtin_amdgcn_logf(ltot)) * kLn2;
    }
}

// ============================================================================ backward: dQ
// Same shape as the forward: 128 query rows per workgroup, keys/values streamed.
//   S^T = K Q^T, dP^T = V dO^T, P = exp(S - LSE), dS = P (dP - D), dQ^T += K^T dS^T
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_bf16_kernel(AttnArgs a)
{
    __shared__ __attribute__((aligned(256))) unsigned char smem[2 * kTileBytes];
    LDS_AS unsigned char *Ks = (LDS_AS unsigned char *)smem;
    LDS_AS unsigned char *Vs = Ks + kTileBytes;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
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

    bf16x8 qB[8], gB[8];
#pragma unroll
    for (int kc = 0; kc < 8; ++kc) {
        u32x4 rq = {0u, 0u, 0u, 0u}, rg = rq;
        if (i < a.S) {
            rq = *reinterpret_cast<const u32x4 *>(q + i * a.ss + 16 * kc + 8 * half);
            rg = *reinterpret_cast<const u32x4 *>(g + i * a.ss + 16 * kc + 8 * half);
        }
        qB[kc] = __builtin_bit_cast(bf16x8, rq);
        gB[kc] = __builtin_bit_cast(bf16x8, rg);
    }
    const float c = a.scale * kLog2e;
    // rows past S: LSE = +inf makes their probabilities exactly zero
    const float lse2 = (i < a.S) ? a.lse[stat + i] * kLog2e : INFINITY;
    const float Di = (i < a.S) ? a.delta[stat + i] : 0.f;

    f32x16 accQ[4];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int e = 0; e < 16; ++e) accQ[cb][e] = 0.f;

    const int64_t last_row = min(row0 + kFwdBq, a.S) - 1;
    const int64_t ntiles = last_row / kBk + 1;

    RowRegs kreg, vreg;
    load_rows(kreg, k, a.ss, 0, a.S, tid);
    load_rows(vreg, v, a.ss, 0, a.S, tid);

    for (int64_t jt = 0; jt < ntiles; ++jt) {
        const int64_t j0 = jt * kBk;
        __syncthreads();
        store_rows(Ks, kreg, tid);
        store_rows(Vs, vreg, tid);
        __syncthreads();
        if (jt + 1 < ntiles) {
            load_rows(kreg, k, a.ss, j0 + kBk, a.S, tid);
            load_rows(vreg, v, a.ss, j0 + kBk, a.S, tid);
        }
        if (j0 > i0w + 31) continue;
        const bool diag = j0 + kBk - 1 > i0w;
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
            f32x16 s, dp;
#pragma unroll
            for (int e = 0; e < 16; ++e) { s[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
            for (int kc = 0; kc < 8; ++kc) {
                s = mfma32(lds_row_operand(Ks, la.row_op[kc] + jb * 8192), qB[kc], s);
                dp = mfma32(lds_row_operand(Vs, la.row_op[kc] + jb * 8192), gB[kc], dp);
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                float p = __builtin_amdgcn_exp2f(fmaf(s[e], c, -lse2));
                if (diag) {
                    const int64_t j = j0 + 32 * jb + 8 * (e >> 2) + 4 * half + (e & 3);
                    if (j > i) p = 0.f;
                }
                s[e] = p * (dp[e] - Di);           // dS
            }
            // dQ^T += K^T dS^T : A = K^T (transposed read of the same K tile), B = dS^T registers
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                const bf16x8 dsB = pack8(s, 8 * sub);
#pragma unroll
                for (int cb = 0; cb < 4; ++cb)
                    accQ[cb] = mfma32(lds_tr_operand(Ks, la, cb, 2 * jb + sub), dsB, accQ[cb]);
            }
        }
    }
    if (i < a.S) {
        __bf16 *dq = static_cast<__bf16 *>(a.dq) + base + i * a.ss;
        store_acc_T(dq, accQ, a.scale, half);
    }
}

// ============================================================================ backward: dK, dV
// Workgroup: 4 waves, 128 key rows (32 per wave) held in registers; queries streamed in
// tiles of 64 from the diagonal to the end of the sequence.
//   S = Q K^T, dP = dO V^T (key index per lane), P = exp(S - LSE_i), dS = P (dP - D_i),
//   dV^T += dO^T P, dK^T += Q^T dS      (no atomics: each key row has one owner)
constexpr int kBwdBk = 128, kBq = 64;

__global__ __launch_bounds__(256) void attn_bwd_dkdv_bf16_kernel(AttnArgs a)
{
    __shared__ __attribute__((aligned(256))) unsigned char smem[2 * kTileBytes + 512];
    LDS_AS unsigned char *Qs = (LDS_AS unsigned char *)smem;
    LDS_AS unsigned char *Gs = Qs + kTileBytes;
    LDS_AS float *Ls = (LDS_AS float *)(Gs + kTileBytes);   // 64 x LSE*log2e
    LDS_AS float *Ds = Ls + 64;                             // 64 x D_i

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const LaneAddr la = make_lane_addr(lane);
    const int64_t nkt = (a.S + kBwdBk - 1) / kBwdBk;
    const TileId t = decode_block(a, nkt, false);     // key tile 0 sees every query: heaviest first
    const int64_t col0 = t.tile * kBwdBk, j0w = col0 + 32 * wave, j = j0w + l32;
    const int64_t base = (int64_t)t.b * a.sb + (int64_t)t.h * a.sh;
    const __bf16 *q = static_cast<const __bf16 *>(a.q) + base;
    const __bf16 *k = static_cast<const __bf16 *>(a.k) + base;
    const __bf16 *v = static_cast<const __bf16 *>(a.v) + base;
    const __bf16 *g = static_cast<const __bf16 *>(a.d_o) + base;
    const int64_t stat = ((int64_t)t.b * a.H + t.h) * a.S;

    bf16x8 kB[8], vB[8];
#pragma unroll
    for (int kc = 0; kc < 8; ++kc) {
        u32x4 rk = {0u, 0u, 0u, 0u}, rv = rk;
        if (j < a.S) {
            rk = *reinterpret_cast<const u32x4 *>(k + j * a.ss + 16 * kc + 8 * half);
            rv = *reinterpret_cast<const u32x4 *>(v + j * a.ss + 16 * kc + 8 * half);
        }
        kB[kc] = __builtin_bit_cast(bf16x8, rk);
        vB[kc] = __builtin_bit_cast(bf16x8, rv);
    }
    const float c = a.scale * kLog2e;

    f32x16 accK[4], accV[4];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int e = 0; e < 16; ++e) { accK[cb][e] = 0.f; accV[cb][e] = 0.f; }

    const int64_t it0 = col0 / kBq;
    const int64_t nit = (a.S + kBq - 1) / kBq;

    RowRegs qreg, greg;
    float lreg = 0.f, dreg = 0.f;
    auto fetch = [&](int64_t i0) {
        load_rows(qreg, q, a.ss, i0, a.S, tid);
        load_rows(greg, g, a.ss, i0, a.S, tid);
        if (tid < 64) {
            const bool ok = i0 + tid < a.S;
            // rows past S: LSE = +inf makes their probabilities exactly zero
            lreg = ok ? a.lse[stat + i0 + tid] * kLog2e : INFINITY;
            dreg = ok ? a.delta[stat + i0 + tid] : 0.f;
        }
    };
    fetch(it0 * kBq);

    for (int64_t it = it0; it < nit; ++it) {
        const int64_t i0 = it * kBq;
        __syncthreads();
        store_rows(Qs, qreg, tid);
        store_rows(Gs, greg, tid);
        if (tid < 64) { Ls[tid] = lreg; Ds[tid] = dreg; }
        __syncthreads();
        if (it + 1 < nit) fetch(i0 + kBq);
        if (i0 + kBq - 1 < j0w) continue;       // all 64 queries precede this wave's keys
        const bool diag = i0 < j0w + 31;
#pragma unroll
        for (int ib = 0; ib < 2; ++ib) {
            f32x16 s, dp;
#pragma unroll
            for (int e = 0; e < 16; ++e) { s[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
            for (int kc = 0; kc < 8; ++kc) {
                s = mfma32(lds_row_operand(Qs, la.row_op[kc] + ib * 8192), kB[kc], s);
                dp = mfma32(lds_row_operand(Gs, la.row_op[kc] + ib * 8192), vB[kc], dp);
            }
            // s, dp: lane = key j, register e = query row 32*ib + 8*(e/4) + 4*half + e%4
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const f32x4 l4 = *reinterpret_cast<const LDS_AS f32x4 *>(Ls + 32 * ib + 8 * gq + 4 * half);
                const f32x4 d4 = *reinterpret_cast<const LDS_AS f32x4 *>(Ds + 32 * ib + 8 * gq + 4 * half);
                const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
                const float dl[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int e = 4 * gq + r;
                    float p = __builtin_amdgcn_exp2f(fmaf(s[e], c, -lv[r]));
                    if (diag) {
                        const int64_t ii = i0 + 32 * ib + 8 * gq + 4 * half + r;
                        if (ii < j) p = 0.f;
                    }
                    s[e] = p;
                    dp[e] = p * (dp[e] - dl[r]);    // dS
                }
            }
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                const bf16x8 pB = pack8(s, 8 * sub);
                const bf16x8 dsB = pack8(dp, 8 * sub);
#pragma unroll
                for (int cb = 0; cb < 4; ++cb) {
                    accV[cb] = mfma32(lds_tr_operand(Gs, la, cb, 2 * ib + sub), pB, accV[cb]);
                    accK[cb] = mfma32(lds_tr_operand(Qs, la, cb, 2 * ib + sub), dsB, accK[cb]);
                }
            }
        }
    }
    if (j < a.S) {
        store_acc_T(static_cast<__bf16 *>(a.dk) + base + j * a.ss, accK, a.scale, half);
        store_acc_T(static_cast<__bf16 *>(a.dv) + base + j * a.ss, accV, 1.f, half);
    }
}

}  // namespace

hipError_t launch_attn_fwd_bf16(const AttnArgs &a, hipStream_t st)
{
    const int64_t nqt = (a.S + kFwdBq - 1) / kFwdBq;
    const int64_t blocks = nqt * a.H * a.B;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    attn_fwd_bf16_kernel<<<dim3((unsigned)blocks), 256, 0, st>>>(a);
    return hipGetLastError();
}

hipError_t launch_attn_bwd_bf16(const AttnArgs &a, hipStream_t st)
{
    const int64_t nqt = (a.S + kFwdBq - 1) / kFwdBq;
    const int64_t nkt = (a.S + kBwdBk - 1) / kBwdBk;
    if (nqt * a.H * a.B > 0x7fffffffLL) return hipErrorInvalidValue;
    hipError_t e = record_stage(a, 0, st);
    if (e != hipSuccess) return e;
    if ((e = launch_attn_delta(a, true, st)) != hipSuccess) return e;
    if ((e = record_stage(a, 1, st)) != hipSuccess) return e;
    attn_bwd_dkdv_bf16_kernel<<<dim3((unsigned)(nkt * a.H * a.B)), 256, 0, st>>>(a);
    if ((e = record_stage(a, 2, st)) != hipSuccess) return e;
    attn_bwd_dq_bf16_kernel<<<dim3((unsigned)(nqt * a.H * a.B)), 256, 0, st>>>(a);
    if ((e = record_stage(a, 3, st)) != hipSuccess) return e;
    return hipGetLastError();
}

}  // namespace memo
