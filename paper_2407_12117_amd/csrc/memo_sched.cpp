// Two rounding buffers over n layers: packing plan and the three-stream schedule
// (Section 4.1, Figure 5; Section 4.3.4).  Host code only: the copies are the same
// prefix DMAs as memo_swap_out / memo_swap_in, ordered by HIP events.
#include <hip/hip_runtime.h>

#include <cmath>
#include <new>
#include <vector>

#include "../../include/memo.h"

namespace {

constexpr int64_t kAlign = 256;

inline int64_t round_up(int64_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

}  // namespace

struct memo_sched {
    int32_t n_layers = 0;
    std::vector<memo_tensor_slot> slots;
    size_t dev_bytes = 0, host_bytes = 0;
    char *buffer[2] = {nullptr, nullptr};
    char *host = nullptr;
    hipStream_t compute = nullptr, offload = nullptr, prefetch = nullptr;
    // one event of each kind per layer
    std::vector<hipEvent_t> fwd_done, offloaded, bwd_done, fetched;
    // position in the fixed call sequence of one iteration, 0 .. 4n-1
    int64_t pos = 0;
    // set when a HIP call failed inside a schedule call: some of that call's work may already be
    // queued, so the handle refuses every later call except memo_sched_destroy
    bool failed = false;

    bool swapped(int32_t layer) const { return layer < n_layers - 2; }
};

namespace {

void destroy_events(std::vector<hipEvent_t> &v)
{
    for (hipEvent_t e : v)
        if (e) (void)hipEventDestroy(e);
    v.clear();
}

bool create_events(std::vector<hipEvent_t> &v, int32_t n)
{
    v.assign(static_cast<size_t>(n), nullptr);
    for (int32_t i = 0; i < n; ++i)
        if (hipEventCreateWithFlags(&v[i], hipEventDisableTiming) != hipSuccess) return false;
    return true;
}

// Expected position of a call: forward i -> 2i (+1 for end); backward i -> 2n + 2(n-1-i) (+1).
memo_status take_position(memo_sched *s, int32_t layer, bool backward, bool end)
{
    if (!s || layer < 0 || layer >= s->n_layers) return MEMO_ERR_INVALID_ARG;
    if (s->failed) return MEMO_ERR_DEVICE;
    const int64_t n = s->n_layers;
    const int64_t want = (backward ? 2 * n + 2 * (n - 1 - layer) : 2 * static_cast<int64_t>(layer)) + (end ? 1 : 0);
    if (s->pos != want) return MEMO_ERR_INVALID_ARG;
    return MEMO_OK;
}

memo_status fail(memo_sched *s)
{
    s->failed = true;
    return MEMO_ERR_DEVICE;
}

void advance(memo_sched *s) { s->pos = (s->pos + 1) % (4 * static_cast<int64_t>(s->n_layers)); }

}  // namespace

extern "C" {

memo_status memo_buffer_plan_make(int64_t S, int32_t n_tensors, const memo_tensor_desc *tensors,
                                  memo_tensor_slot *slots_out, size_t *dev_bytes_out,
                                  size_t *host_bytes_out)
{
    if (!tensors || !slots_out || !dev_bytes_out || !host_bytes_out) return MEMO_ERR_INVALID_ARG;
    if (S < 1 || n_tensors < 1) return MEMO_ERR_INVALID_ARG;
    int64_t dev = 0, host = 0;
    for (int32_t t = 0; t < n_tensors; ++t) {
        memo_swap_plan p;
        const memo_status st = memo_swap_plan_make(S, tensors[t].row_bytes, tensors[t].alpha, &p);
        if (st != MEMO_OK) return st;
        slots_out[t].dev_offset = dev;
        slots_out[t].host_offset = host;
        slots_out[t].k_swapped = p.k_swapped;
        slots_out[t].bytes_swapped = p.bytes_swapped;
        dev = round_up(dev + S * tensors[t].row_bytes);
        host = round_up(host + static_cast<int64_t>(p.bytes_swapped));
    }
    *dev_bytes_out = static_cast<size_t>(dev);
    *host_bytes_out = static_cast<size_t>(host);
    return MEMO_OK;
}

memo_status memo_sched_create(memo_sched **out, int32_t n_layers, int64_t S, int32_t n_tensors,
                              const memo_tensor_desc *tensors, void *dev_buffer0,
                              void *dev_buffer1, void *host_store, size_t host_capacity_bytes,
                              void *compute_stream, void *offload_stream, void *prefetch_stream)
{
    if (!out) return MEMO_ERR_INVALID_ARG;
    *out = nullptr;
    if (n_layers < 1 || n_tensors < 1 || !tensors || !dev_buffer0 || !dev_buffer1)
        return MEMO_ERR_INVALID_ARG;
    memo_sched *s = new (std::nothrow) memo_sched;
    if (!s) return MEMO_ERR_DEVICE;
    s->n_layers = n_layers;
    s->slots.resize(static_cast<size_t>(n_tensors));
    memo_status st = memo_buffer_plan_make(S, n_tensors, tensors, s->slots.data(), &s->dev_bytes,
                                           &s->host_bytes);
    if (st != MEMO_OK) {
        delete s;
        return st;
    }
    const size_t held = n_layers > 2 ? static_cast<size_t>(n_layers - 2) : 0;
    if (held * s->host_bytes > host_capacity_bytes) {
        delete s;
        return MEMO_ERR_HOST_CAPACITY;
    }
    if (held * s->host_bytes > 0 && !host_store) {
        delete s;
        return MEMO_ERR_INVALID_ARG;
    }
    s->buffer[0] = static_cast<char *>(dev_buffer0);
    s->buffer[1] = static_cast<char *>(dev_buffer1);
    s->host = static_cast<char *>(host_store);
    s->compute = static_cast<hipStream_t>(compute_stream);
    s->offload = static_cast<hipStream_t>(offload_stream);
    s->prefetch = static_cast<hipStream_t>(prefetch_stream);
    if (!create_events(s->fwd_done, n_layers) || !create_events(s->offloaded, n_layers) ||
        !create_events(s->bwd_done, n_layers) || !create_events(s->fetched, n_layers)) {
        memo_sched_destroy(s);
        return MEMO_ERR_DEVICE;
    }
    *out = s;
    return MEMO_OK;
}

memo_status memo_sched_forward_begin(memo_sched *s, int32_t layer)
{
    memo_status st = take_position(s, layer, false, false);
    if (st != MEMO_OK) return st;
    // Buffer layer%2 was last read by the offload of layer-2: do not overwrite it earlier.
    if (layer >= 2 && hipStreamWaitEvent(s->compute, s->offloaded[layer - 2], 0) != hipSuccess)
        return fail(s);
    advance(s);
    return MEMO_OK;
}

memo_status memo_sched_forward_end(memo_sched *s, int32_t layer)
{
    memo_status st = take_position(s, layer, false, true);
    if (st != MEMO_OK) return st;
    if (s->swapped(layer)) {
        if (hipEventRecord(s->fwd_done[layer], s->compute) != hipSuccess) return fail(s);
        if (hipStreamWaitEvent(s->offload, s->fwd_done[layer], 0) != hipSuccess)
            return fail(s);
        const char *buf = s->buffer[layer % 2];
        char *slot = s->host + static_cast<size_t>(layer) * s->host_bytes;
        for (const memo_tensor_slot &t : s->slots) {
            if (t.bytes_swapped == 0) continue;
            if (hipMemcpyAsync(slot + t.host_offset, buf + t.dev_offset, t.bytes_swapped,
                               hipMemcpyDeviceToHost, s->offload) != hipSuccess)
                return fail(s);
        }
        if (hipEventRecord(s->offloaded[layer], s->offload) != hipSuccess) return fail(s);
    }
    advance(s);
    return MEMO_OK;
}

memo_status memo_sched_backward_begin(memo_sched *s, int32_t layer)
{
    memo_status st = take_position(s, layer, true, false);
    if (st != MEMO_OK) return st;
    if (s->swapped(layer) && hipStreamWaitEvent(s->compute, s->fetched[layer], 0) != hipSuccess)
        return fail(s);
    advance(s);
    return MEMO_OK;
}

memo_status memo_sched_backward_end(memo_sched *s, int32_t layer)
{
    memo_status st = take_position(s, layer, true, true);
    if (st != MEMO_OK) return st;
    const int32_t j = layer - 2;
    if (j >= 0) {
        // Buffer layer%2 is dead once this backward has finished: fetch layer j into it.
        // Layer j's offload finished long ago: forward(j+2) waited for it.
        if (hipEventRecord(s->bwd_done[layer], s->compute) != hipSuccess) return fail(s);
        if (hipStreamWaitEvent(s->prefetch, s->bwd_done[layer], 0) != hipSuccess)
            return fail(s);
        char *buf = s->buffer[j % 2];
        const char *slot = s->host + static_cast<size_t>(j) * s->host_bytes;
        for (const memo_tensor_slot &t : s->slots) {
            if (t.bytes_swapped == 0) continue;
            if (hipMemcpyAsync(buf + t.dev_offset, slot + t.host_offset, t.bytes_swapped,
                               hipMemcpyHostToDevice, s->prefetch) != hipSuccess)
                return fail(s);
        }
        if (hipEventRecord(s->fetched[j], s->prefetch) != hipSuccess) return fail(s);
    }
    advance(s);
    return MEMO_OK;
}

void *memo_sched_buffer(const memo_sched *s, int32_t layer)
{
    if (!s || layer < 0 || layer >= s->n_layers) return nullptr;
    return s->buffer[layer % 2];
}

memo_status memo_sched_destroy(memo_sched *s)
{
    if (!s) return MEMO_OK;
    destroy_events(s->fwd_done);
    destroy_events(s->offloaded);
    destroy_events(s->bwd_done);
    destroy_events(s->fetched);
    delete s;
    return MEMO_OK;
}

}  // extern "C"
