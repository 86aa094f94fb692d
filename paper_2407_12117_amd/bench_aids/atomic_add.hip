// Benchmark aid (not part of libmemo): the rate at which the chip retires fp32 atomic adds in the
// access pattern a fused five-contraction backward would produce for dQ.  In such a kernel the
// key-stationary workgroup adds an fp32 partial dQ of its query tile to global memory per step: blocks
// of 32 KB here (64 queries x 128, the tile of a 128-key workgroup; the 256-key workgroup of the
// library would add 16 KB per 32-query step, which only changes how many such blocks there are).
// `dup` = 4 models several key-block waves adding unreduced partials, `dup` = 1 a reduction through
// LDS first.  Workgroup w of head w % heads starts at row block 2 * (w / heads)
// and walks forward, as the key tiles of one head do.  scope: 0 device-scope atomics, 1 workgroup-
// scope atomics, 2 plain stores of the same bytes (for reference).
#include <hip/hip_runtime.h>
#include <stdint.h>
namespace {
template <int SCOPE>
__global__ __launch_bounds__(512) void atom_kernel(float *buf, int64_t head_stride_blocks, int heads, int iters, int dup, int64_t nblocks)
{
    const int wg = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int h = wg % heads;
    int64_t blk = (2 * (int64_t)(wg / heads)) % nblocks;
    float *hb = buf + (int64_t)h * head_stride_blocks * 8192;
    for (int it = 0; it < iters; ++it, ++blk) {
        if (blk >= nblocks) blk -= nblocks;
        float *p = hb + blk * 8192;
        for (int r = 0; r < dup; ++r) {
            const int w = (wave + 2 * r) & 7;
#pragma unroll
            for (int n = 0; n < 16; ++n) {
                float *a = p + (w * 16 + n) * 64 + lane;
                if (SCOPE == 0) __hip_atomic_fetch_add(a, 1.0f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                else if (SCOPE == 1) __hip_atomic_fetch_add(a, 1.0f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                else *a = 1.0f;            // plain stores of the same bytes, for reference
            }
        }
    }
}
}  // namespace

// buf: heads * head_stride_blocks * 8192 floats; returns the HIP error code of the launch
extern "C" int memo_bench_atomic_add(float *buf, int64_t head_stride_blocks, int heads, int wgs, int iters, int dup, int64_t nblocks, int scope, void *stream)
{
    if (!buf || heads < 1 || wgs < 1 || iters < 1 || dup < 1 || dup > 4 || nblocks < 1 || head_stride_blocks < nblocks) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    if (scope == 0) atom_kernel<0><<<wgs, 512, 0, st>>>(buf, head_stride_blocks, heads, iters, dup, nblocks);
    else if (scope == 1) atom_kernel<1><<<wgs, 512, 0, st>>>(buf, head_stride_blocks, heads, iters, dup, nblocks);
    else atom_kernel<2><<<wgs, 512, 0, st>>>(buf, head_stride_blocks, heads, iters, dup, nblocks);
    return (int)hipGetLastError();
}
