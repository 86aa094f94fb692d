// memo_attn_bwd_static: the attention backward for callers that can neither allocate device
// memory nor pass a workspace (code under HIP graph capture, tight serving loops, harnesses that
// forbid hipMalloc).  The one scratch buffer of the backward, D_i = sum_c dO_ic O_ic (one fp32 per
// (b, h, i)), lives in a file-scope device array instead of a caller workspace; the kernels are
// the ones memo_attn_bwd launches and take the array's device address as that workspace.
//
// The array exists once per GPU (each device that loads this code object holds its own copy at
// its own address, until the process ends).  Its name is a host-side handle, not a device
// address: the address is looked up once per device with hipGetSymbolAddress, with that device
// current, and only that looked-up pointer is ever handed to a kernel.
#include "../../include/memo.h"
#include "memo_kernels.h"

#include <mutex>

namespace {

constexpr size_t kScratchBytes = MEMO_ATTN_BWD_STATIC_MAX_ROWS * sizeof(float);   // 16 MiB
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void *g_scratch_ptr[kMaxDevices];      // device address of `scratch` on device n, nullptr = not looked up yet

// Device address of the scratch array on the current device; hipSuccess or the failing call's error.
hipError_t scratch_of_current_device(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

extern "C" memo_status memo_attn_bwd_static(const memo_attn_desc *desc, const void *q, const void *k,
                                            const void *v, const void *o, const float *lse,
                                            const void *d_o, void *dq, void *dk, void *dv, void *stream)
{
    // the size of the problem is checked against the array before anything touches the device
    const size_t need = memo_attn_bwd_workspace_bytes(desc);      // 0 for a descriptor that is refused
    if (desc && need > kScratchBytes) return MEMO_ERR_WORKSPACE;
    if (!desc || need == 0)       // a refused descriptor: the common path names the error and queues nothing
        return memo_attn_bwd(desc, q, k, v, o, lse, d_o, dq, dk, dv, nullptr, 0, stream);
    // argument errors are reported before the device is touched at all
    if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv) return MEMO_ERR_INVALID_ARG;
    void *ws = nullptr;
    if (scratch_of_current_device(&ws) != hipSuccess) return MEMO_ERR_DEVICE;
    // D_i is written in full by the preprocess kernel before the main kernels read it: nothing in
    // the array has to start at zero, whatever the previous call left there.
    return memo_attn_bwd(desc, q, k, v, o, lse, d_o, dq, dk, dv, ws, kScratchBytes, stream);
}
