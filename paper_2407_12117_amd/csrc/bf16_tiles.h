// Building blocks shared by the bf16 MFMA kernels (gfx950): vector types, the 32x32x16 MFMA
// wrapper, the swizzled 64-row x 256-byte LDS tile and its per-lane addresses, asynchronous
// global -> LDS tile fills, and hand-issued, software-pipelined LDS operand reads.
// Included by the kernel sources only; everything has internal linkage.
#pragma once
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
#define GLB_AS __attribute__((address_space(1)))

constexpr int kTileBytes = 64 * 256;   // one 64 x 128 bf16 tile
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// Chunk swizzles of the 64-row x 256-byte LDS tile: the sixteen 16-byte chunks of row r are
// stored at chunk position c ^ f(r), f of period 16 in r.  SwzA serves the 32x32x16 kernels
// (lane 32*half + l32 reading chunk 2*kc + half of row l32; 32 lanes reading 4 rows x 64 bytes
// transposed).  SwzB serves the 16x16x32 kernels (lane 16*g4 + l16 reading chunk 4*ks + g4 of row
// l16; 16-lane groups reading rows 4*g4 .. 4*g4+3 x 32 bytes transposed).  Which lanes the LDS
// serves in one cycle, and so which f are free of bank conflicts for a pattern, was found by
// measurement (SQ_LDS_BANK_CONFLICT and read throughput over all 20160 invertible bit-linear f):
// SwzA conflicts two-way on both patterns of the 16x16x32 kernels; SwzB is free on both.
struct SwzA { static __device__ __forceinline__ int f(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); } };
struct SwzB { static __device__ __forceinline__ int f(int r) { return ((((r & 7) << 1) | ((r >> 3) & 1)) ^ (r & 8)) & 15; } };
__device__ __forceinline__ int swz(int r) { return SwzA::f(r); }

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

// the same offsets as absolute LDS byte addresses (for the hand-issued reads)
struct LdsAddr { uint32_t row[8]; uint32_t tr[4][2]; };
__device__ __forceinline__ LdsAddr make_lds_addr(const LDS_AS unsigned char *base, const LaneAddr &la)
{
    LdsAddr ad;
    const uint32_t b = (uint32_t)(uintptr_t)base;
#pragma unroll
    for (int kc = 0; kc < 8; ++kc) ad.row[kc] = b + (uint32_t)la.row_op[kc];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int sec = 0; sec < 2; ++sec) ad.tr[cb][sec] = b + (uint32_t)la.tr_op[cb][sec];
    return ad;
}

// Per-lane LDS addresses of the 16x16x32 kernels (SwzB tiles), lane = 16*g4 + l16:
//   row16[ks]  row-major operand: row l16 of a 16-row block, chunk 4*ks + g4 (k = 32*ks + 8*g4 ..)
//   tr16[ct]   transposed operand of the 16 columns 16*ct ..: this lane's address in the
//              ds_read_b64_tr_b16 of rows 4*g4 .. 4*g4+3 (lane i16 of a group supplies row i16/4,
//              columns 4*(i16%4) .. and receives column i16); + 16 rows = + 4096 bytes
struct LdsAddr16 { uint32_t row16[4]; uint32_t tr16[8]; };
__device__ __forceinline__ LdsAddr16 make_lds_addr16(const LDS_AS unsigned char *base, int lane)
{
    LdsAddr16 ad;
    const uint32_t b = (uint32_t)(uintptr_t)base;
    const int l16 = lane & 15, g4 = lane >> 4;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) ad.row16[ks] = b + (uint32_t)(l16 * 256 + (((4 * ks + g4) ^ SwzB::f(l16)) << 4));
    const int row = 4 * g4 + (l16 >> 2);
#pragma unroll
    for (int ct = 0; ct < 8; ++ct)
        ad.tr16[ct] = b + (uint32_t)(row * 256 + (((2 * ct + ((l16 & 3) >> 1)) ^ SwzB::f(row)) << 4) + 8 * (l16 & 1));
    return ad;
}

// 8 fp32 (two accumulator quartets) -> 8 bf16
__device__ __forceinline__ bf16x8 pack44(const f32x4 &lo, const f32x4 &hi)
{
    bf16x8 out;
    f32x2 t0 = {lo[0], lo[1]}, t1 = {lo[2], lo[3]}, t2 = {hi[0], hi[1]}, t3 = {hi[2], hi[3]};
    bf16x2 r0 = __builtin_convertvector(t0, bf16x2), r1 = __builtin_convertvector(t1, bf16x2);
    bf16x2 r2 = __builtin_convertvector(t2, bf16x2), r3 = __builtin_convertvector(t3, bf16x2);
    out[0] = r0[0]; out[1] = r0[1]; out[2] = r1[0]; out[3] = r1[1];
    out[4] = r2[0]; out[5] = r2[1]; out[6] = r3[0]; out[7] = r3[1];
    return out;
}

// 4 fp32 -> 4 bf16, stored as 8 bytes
__device__ __forceinline__ void store4(__bf16 *dst, const f32x4 &x, float mul)
{
    f32x2 a = {x[0] * mul, x[1] * mul}, b = {x[2] * mul, x[3] * mul};
    u32x2 w;
    w[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(a, bf16x2));
    w[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(b, bf16x2));
    *reinterpret_cast<u32x2 *>(dst) = w;
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

constexpr int kXcds = 8, kChunk = 32;   // XCDs per device; compute units (one workgroup each) per XCD

// Folded order of all three attention kernels.  Every workgroup of a head streams that head's K/V
// rows (forward, dQ) or Q/dO rows (dK/dV), and a tile's sweep is as long as its distance from the
// end of the causal triangle.  A workgroup works a PAIR of tiles of one head, the p-th longest and
// the p-th shortest, so every workgroup of a launch has the same length (ntiles + 1 tile units): a
// launch is a whole number of equal rounds and no compute unit waits for a straggler, whatever S
// is.  Chunks of kChunk consecutive pairs go to one XCD (the dispatcher deals consecutive workgroup
// ids round-robin to the 8 XCDs; an XCD has 32 compute units and these kernels run one workgroup
// per unit), chunks of one head to the 8 XCDs of a round.  The long tile is swept from the end all
// tiles share towards its own end, the short tile the other way round (forward and dQ: keys upwards
// from row 0, then downwards to row 0; dK/dV: queries downwards from row S-1, then upwards to it).
// Workgroup s of a chunk ends its first sweep a fixed number of steps per s before workgroup 0 and
// begins its second one as many steps further from the shared end, so the lengths cancel and the
// workgroups of an XCD read the same rows at about the same time in both sweeps, which is what
// lets that XCD's L2 serve most of those reads (measured: 32 workgroups, one fetch from the fabric,
// up to S = 256K; at S = 1M the forward keeps that, the two backward kernels drift apart over their
// 16384 steps and fetch about half of what they stream).
struct PairId { int64_t first, second; int h, b; };   // first < 0: nothing to do; second < 0: one tile only

__host__ __device__ inline int64_t folded_grid(int64_t ntiles, int64_t heads)
{
    const int64_t cph = ((ntiles + 1) / 2 + kChunk - 1) / kChunk;      // chunks per head
    return (cph * heads + kXcds - 1) / kXcds * kXcds * kChunk;
}

__device__ __forceinline__ PairId decode_block_folded(const AttnArgs &a, int64_t ntiles)
{
    const int64_t npairs = (ntiles + 1) / 2, cph = (npairs + kChunk - 1) / kChunk;
    const int64_t id = blockIdx.x;
    const int64_t chunk = id / (kXcds * kChunk) * kXcds + id % kXcds;  // round * 8 + xcd
    const int64_t p = (chunk % cph) * kChunk + (id / kXcds) % kChunk;
    const int64_t hbi = chunk / cph;
    const bool live = hbi < (int64_t)a.H * a.B && p < npairs;
    PairId t;
    t.first = live ? p : -1;                                           // tile p and tile ntiles-1-p
    t.second = (live && p != ntiles - 1 - p) ? ntiles - 1 - p : -1;
    t.h = (int)(hbi % a.H);
    t.b = (int)(hbi / a.H);
    return t;
}

// ---- asynchronous tile fill: global -> LDS without passing through registers -------------
// One global_load_lds_dwordx4 moves 64 x 16 bytes: lane l lands at LDS base + 16*l, i.e. four
// tile rows of sixteen chunks.  With NW waves sharing a tile, wave w issues instruction n for
// tile rows 4*(NI*w + n) + l/16 (NI = 16/NW); the lane at chunk position p = l%16 fetches
// logical chunk p ^ swz(row), so the swizzle is applied on the global side.  Each lane keeps
// the global address of its piece per instruction and steps it by one tile (a wave-uniform
// stride) after every fill: one 64-bit add per instruction and tile, nothing else.
template <int NW>
struct TileStream {
    static constexpr int kInstr = 16 / NW;
    const char *p[16 / NW];
};

template <int NW, typename SW = SwzA>
__device__ __forceinline__ TileStream<NW> make_tile_stream(const __bf16 *src, int64_t ss, int64_t r0,
                                                           int wave, int lane)
{
    TileStream<NW> f;
#pragma unroll
    for (int n = 0; n < TileStream<NW>::kInstr; ++n) {
        const int row = 4 * (TileStream<NW>::kInstr * wave + n) + (lane >> 4);
        const int chunk = (lane & 15) ^ SW::f(row);
        f.p[n] = reinterpret_cast<const char *>(src + (r0 + row) * ss + chunk * 8);
    }
    return f;
}

// Queues the fill of the 64-row tile the stream points at (rows r0..r0+63 of the head view
// `src`) and steps the stream to the next tile (the previous one with dir = -1).  A tile that reaches past row S-1 takes the
// slow path: rows past S re-read row S-1 (finite values; every consumer masks them).
template <int NW, typename SW = SwzA>
__device__ __forceinline__ void fill_tile_async(LDS_AS unsigned char *tile, TileStream<NW> &f,
                                                const __bf16 *src, int64_t ss, int64_t r0, int64_t S,
                                                int wave, int lane, int dir = 1)
{
    constexpr int NI = TileStream<NW>::kInstr;
    if (__builtin_expect(r0 + 64 <= S, 1)) {
#pragma unroll
        for (int n = 0; n < NI; ++n)
            __builtin_amdgcn_global_load_lds((const GLB_AS void *)f.p[n],
                                             (LDS_AS void *)(tile + (NI * wave + n) * 1024), 16, 0, 0);
    } else {
#pragma unroll
        for (int n = 0; n < NI; ++n) {
            const int row = 4 * (NI * wave + n) + (lane >> 4);
            const int chunk = (lane & 15) ^ SW::f(row);
            int64_t rg = r0 + row;
            rg = rg < S ? rg : S - 1;
            __builtin_amdgcn_global_load_lds((const GLB_AS void *)(src + rg * ss + chunk * 8),
                                             (LDS_AS void *)(tile + (NI * wave + n) * 1024), 16, 0, 0);
        }
    }
    const int64_t step = dir * 64 * ss * 2;       // dir = -1: the stream walks towards row 0
#pragma unroll
    for (int n = 0; n < NI; ++n) f.p[n] += step;
}

// The same fill addressed as a wave-uniform tile base (scalar registers, stepped once per tile)
// plus a per-lane 32-bit byte offset that never changes: half the address registers of
// TileStream and no per-tile vector adds.  Needs 64 rows of the view to span < 4 GiB.
template <int NW>
struct TileOffsets {
    static constexpr int kInstr = 16 / NW;
    uint32_t off[16 / NW];
};

template <int NW, typename SW = SwzA>
__device__ __forceinline__ TileOffsets<NW> make_tile_offsets(int64_t ss, int wave, int lane)
{
    TileOffsets<NW> f;
#pragma unroll
    for (int n = 0; n < TileOffsets<NW>::kInstr; ++n) {
        const int row = 4 * (TileOffsets<NW>::kInstr * wave + n) + (lane >> 4);
        const int chunk = (lane & 15) ^ SW::f(row);
        f.off[n] = (uint32_t)(row * ss * 2 + chunk * 16);
    }
    return f;
}

// instruction n of the fill of the full tile whose first row is at `tile_base`
template <int NW>
__device__ __forceinline__ void fill_full_tile_part(LDS_AS unsigned char *tile, const TileOffsets<NW> &f, int n,
                                                    const char *tile_base, int wave)
{
    __builtin_amdgcn_global_load_lds((const GLB_AS void *)(tile_base + f.off[n]),
                                     (LDS_AS void *)(tile + (TileOffsets<NW>::kInstr * wave + n) * 1024), 16, 0, 0);
}

// the ragged last tile: rows past S re-read row S-1 (finite values; every consumer masks them)
template <int NW, typename SW = SwzA>
__device__ __forceinline__ void fill_ragged_tile(LDS_AS unsigned char *tile, const __bf16 *src, int64_t ss,
                                                 int64_t r0, int64_t S, int wave, int lane)
{
    constexpr int NI = 16 / NW;
#pragma unroll
    for (int n = 0; n < NI; ++n) {
        const int row = 4 * (NI * wave + n) + (lane >> 4);
        const int chunk = (lane & 15) ^ SW::f(row);
        int64_t rg = r0 + row;
        rg = rg < S ? rg : S - 1;
        __builtin_amdgcn_global_load_lds((const GLB_AS void *)(src + rg * ss + chunk * 8),
                                         (LDS_AS void *)(tile + (NI * wave + n) * 1024), 16, 0, 0);
    }
}

// ---- software-pipelined LDS operand reads ---------------------------------------------------
// The compiler issues an LDS read right before the MFMA that consumes it and then waits for ALL
// outstanding LDS traffic, which exposes the full LDS latency once per MFMA.  The operand reads of
// the contractions are therefore issued by hand, several MFMAs ahead, through a small ring of
// registers, and each MFMA waits only until its own operand has landed.  LDS returns data in
// issue order, so "at most N reads still outstanding" (s_waitcnt lgkmcnt(N)) means that every
// read issued before the last N has completed; N counts only reads issued through these helpers
// after the wanted one, so any other LDS traffic in between can only make a wait longer, never
// too short.  The wait names the registers it guards as in/out operands, which orders it before
// their first use.
template <int N> struct IntC { static constexpr int value = N; };

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(IntC<I>{});
        static_for<I + 1, N>(f);
    }
}

struct TrSlot { s16x4 lo, hi; };      // the two halves of a transposed operand

template <int OFF>
__device__ __forceinline__ void lds_issue_b128(bf16x8 &dst, uint32_t addr)
{
    static_assert(OFF >= 0 && OFF < 65536, "LDS immediate offset");
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF) : "memory");
}

template <int OFF>
__device__ __forceinline__ void lds_issue_tr(TrSlot &dst, uint32_t addr_lo, uint32_t addr_hi)
{
    static_assert(OFF >= 0 && OFF < 65536, "LDS immediate offset");
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst.lo) : "v"(addr_lo), "n"(OFF) : "memory");
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst.hi) : "v"(addr_hi), "n"(OFF) : "memory");
}

// the two halves from one address register: rows +0 and +16 of a 32-row chunk (16x16x32 kernels)
template <int OFF>
__device__ __forceinline__ void lds_issue_tr_pair(TrSlot &dst, uint32_t addr)
{
    static_assert(OFF >= 0 && OFF + 4096 < 65536, "LDS immediate offset");
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst.lo) : "v"(addr), "n"(OFF) : "memory");
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst.hi) : "v"(addr), "n"(OFF + 4096) : "memory");
}

template <int N>
__device__ __forceinline__ void lds_wait(bf16x8 &x)
{
    static_assert(N >= 0 && N <= 15, "lgkmcnt range");
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(x) : "n"(N));
}

template <int N>
__device__ __forceinline__ void lds_wait(TrSlot &x)
{
    static_assert(N >= 0 && N <= 15, "lgkmcnt range");
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(x.lo), "+v"(x.hi) : "n"(N));
}

__device__ __forceinline__ bf16x8 tr_operand(const TrSlot &t)
{
    const s16x8 both = __builtin_shufflevector(t.lo, t.hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

// Runs items 0..N-1; item n's operand is read DEPTH items ahead of its use.  RPI = LDS reads per
// item (1 for a row operand, 2 for a transposed one).  issue(IntC<n>, slot&), use(IntC<n>, slot&).
// `ring` holds DEPTH+1 slots; the first `PRE` items may have been issued earlier by
// lds_pipeline_prologue (with nothing but other reads of these helpers in between).
template <int N, int DEPTH, int RPI, typename Slot, typename Issue>
__device__ __forceinline__ void lds_pipeline_prologue(Slot (&ring)[DEPTH + 1], Issue &&issue)
{
    static_for<0, (DEPTH < N ? DEPTH : N)>([&](auto n) { issue(n, ring[decltype(n)::value % (DEPTH + 1)]); });
}

template <int N, int DEPTH, int RPI, typename Slot, typename Issue, typename Use>
__device__ __forceinline__ void lds_pipeline_body(Slot (&ring)[DEPTH + 1], Issue &&issue, Use &&use)
{
    static_for<0, N>([&](auto n) {
        constexpr int i = decltype(n)::value;
        if constexpr (i + DEPTH < N) issue(IntC<i + DEPTH>{}, ring[(i + DEPTH) % (DEPTH + 1)]);
        constexpr int later = (i + DEPTH < N ? DEPTH : N - 1 - i) * RPI;
        lds_wait<later>(ring[i % (DEPTH + 1)]);
        use(n, ring[i % (DEPTH + 1)]);
    });
}

// All of this wave's queued fills have landed in LDS.
__device__ __forceinline__ void wait_fills() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// v_permlane32_swap exchanges lanes 32..63 of its first operand with lanes 0..31 of its second:
// fed two copies of x it leaves {x.lo, x.lo} and {x.hi, x.hi}.  The two results are copied to
// scalars before the bit cast: a bit cast applied to the vector element directly reads element 0
// for both with this compiler.
__device__ __forceinline__ void split_halves(float x, float &lo, float &hi)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const uint32_t r0 = r[0], r1 = r[1];
    lo = __builtin_bit_cast(float, r0);
    hi = __builtin_bit_cast(float, r1);
}

// max over the two 32-lane halves, result in every lane
__device__ __forceinline__ float max_across_halves(float x)
{
    float lo, hi;
    split_halves(x, lo, hi);
    return fmaxf(lo, hi);
}

__device__ __forceinline__ float add_across_halves(float x)
{
    float lo, hi;
    split_halves(x, lo, hi);
    return lo + hi;
}


}  // namespace
}  // namespace memo
