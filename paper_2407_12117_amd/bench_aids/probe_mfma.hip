// Benchmark aid, built into its own small library (not part of libmemo, not in include/memo.h):
// the matrix-core rate the chip sustains on given operand data.
// Every wave loads 8 A and 8 B operands once and then issues only v_mfma_f32_32x32x16_bf16
// (4 accumulators, no LDS, no other arithmetic): what is timed is the MFMA pipe alone.  On
// MI355X the result depends on the operand bits (N(0,1) data draws more power than zeros and
// the clock drops), which is why the benchmark reports it beside the published peak.
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stdint.h>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(512) void probe_mfma_kernel(const __bf16 *data, float *sink, int iters)
{
    bf16x8 a[8], b[8];
    const __bf16 *p = data + ((size_t)blockIdx.x * 512 + threadIdx.x) * 128;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = *reinterpret_cast<const bf16x8 *>(p + i * 8);
        b[i] = *reinterpret_cast<const bf16x8 *>(p + 64 + i * 8);
    }
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 8; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[r], b[(r + i) & 7], acc[i], 0, 0, 0);
        if ((it & 63) == 63)          // keeps the sums finite; 64 multiplies per 2048 MFMAs
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][e] *= 1e-3f;
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[i][e];
    if (s == 12345.678f) sink[threadIdx.x] = s;       // never true in practice: keeps the loop alive
}

}  // namespace

// Queues a kernel in which `workgroups` workgroups of 8 waves each issue iters x 32 bf16
// 32x32x16 MFMAs on operands taken from `operands` and nothing else, i.e.
// workgroups * 8 * iters * 32 * 32768 flop.
//   operands  device, workgroups * 512 * 128 bf16 values (256 bytes per lane), 16-byte aligned
//   sink      device, 512 floats, never written in practice
// Returns 0, 1 on a bad argument, 5 if the launch failed.
extern "C" int memo_bench_probe_mfma(const void *operands, float *sink, int32_t workgroups, int32_t iters,
                                     void *hip_stream)
{
    if (!operands || !sink || workgroups < 1 || iters < 1 || (reinterpret_cast<uintptr_t>(operands) & 15u)) return 1;
    probe_mfma_kernel<<<dim3((unsigned)workgroups), 512, 0, static_cast<hipStream_t>(hip_stream)>>>(
        static_cast<const __bf16 *>(operands), sink, iters);
    return hipGetLastError() == hipSuccess ? 0 : 5;
}
