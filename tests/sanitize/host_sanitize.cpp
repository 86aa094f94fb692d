// Host-side sanitizer driver (test infrastructure): the CPU oracle (oracle/memo_oracle.c) and the
// library's host code (memo_api.cpp, memo_sched.cpp, memo_dsa.cpp) built with
// -fsanitize=address,undefined and run on the CPU.  No GPU and no HIP runtime is involved: the few
// HIP entry points the host code calls are replaced below by fakes that execute copies at once with
// memcpy, record nothing and can be told to fail, and the kernel launchers are stubs that count
// calls.  Any out-of-bounds access, use after free, leak, signed overflow or misaligned access in
// the code under test aborts the run; the checks below give those accesses something to do.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "../../include/memo.h"
#include "../../paper_2407_12117_amd/csrc/memo_kernels.h"

#define CHECK(cond)                                                                   \
    do {                                                                              \
        if (!(cond)) {                                                                \
            std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            std::exit(1);                                                             \
        }                                                                             \
    } while (0)

// ------------------------------------------------------------------ fake HIP runtime
namespace fake {
int events_alive = 0;
int copies = 0;
int fail_copy_at = -1;      // the copy with this index fails
int launches = 0;
}  // namespace fake

extern "C" {
hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned)
{
    *e = reinterpret_cast<hipEvent_t>(new int(0));
    ++fake::events_alive;
    return hipSuccess;
}
hipError_t hipEventDestroy(hipEvent_t e)
{
    delete reinterpret_cast<int *>(e);
    --fake::events_alive;
    return hipSuccess;
}
hipError_t hipEventRecord(hipEvent_t e, hipStream_t)
{
    ++*reinterpret_cast<int *>(e);
    return hipSuccess;
}
hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t e, unsigned)
{
    return *reinterpret_cast<int *>(e) >= 0 ? hipSuccess : hipErrorInvalidValue;
}
hipError_t hipMemcpyAsync(void *dst, const void *src, size_t n, hipMemcpyKind, hipStream_t)
{
    if (fake::copies++ == fake::fail_copy_at) return hipErrorInvalidValue;
    std::memcpy(dst, src, n);
    return hipSuccess;
}
hipError_t hipHostMalloc(void **p, size_t n, unsigned)
{
    *p = std::malloc(n);
    return *p ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipHostFree(void *p)
{
    std::free(p);
    return hipSuccess;
}
hipError_t hipGetLastError(void) { return hipSuccess; }
}

namespace memo {
hipError_t launch_attn_fwd_f32(const AttnArgs &, hipStream_t) { ++fake::launches; return hipSuccess; }
hipError_t launch_attn_bwd_f32(const AttnArgs &, hipStream_t) { ++fake::launches; return hipSuccess; }
hipError_t launch_attn_fwd_bf16(const AttnArgs &, hipStream_t) { ++fake::launches; return hipSuccess; }
hipError_t launch_attn_bwd_bf16(const AttnArgs &, hipStream_t) { ++fake::launches; return hipSuccess; }
hipError_t launch_attn_delta(const AttnArgs &, bool, hipStream_t) { ++fake::launches; return hipSuccess; }
hipError_t launch_layernorm_rows_bf16(const void *, const void *, const void *, void *, int64_t, int64_t, int,
                                      float, hipStream_t) { ++fake::launches; return hipSuccess; }
hipError_t launch_linear_rows_bf16(const void *, const void *, const void *, void *, int64_t, int64_t, int, int,
                                   hipStream_t) { ++fake::launches; return hipSuccess; }
}  // namespace memo

// ------------------------------------------------------------------ the oracle's C entry points
extern "C" {
void memo_oracle_attn_fwd(int, int64_t, int, int, double, const double *, const double *, const double *, double *,
                          double *);
void memo_oracle_attn_bwd(int, int64_t, int, int, double, const double *, const double *, const double *,
                          const double *, double *, double *, double *);
void memo_oracle_head_rows(int64_t, int, double, const double *, const double *, const double *, const double *,
                           int64_t, const int64_t *, double *, double *, double *, double *);
void memo_oracle_head_dkdv_tail(int64_t, int, double, const double *, const double *, const double *, const double *,
                                int64_t, double *, double *);
int64_t memo_oracle_split_tokens(int64_t, double);
int memo_oracle_swap_plan(int64_t, int64_t, double, int64_t[5]);
int64_t memo_oracle_swap_out(const unsigned char *, int64_t, int64_t, double, unsigned char *, int64_t);
int64_t memo_oracle_swap_in(unsigned char *, int64_t, int64_t, double, const unsigned char *, int64_t);
double memo_oracle_alpha_grid(double, double, double, double, double, int, double, int);
}

static std::mt19937_64 rng(20240712);

static std::vector<double> randn(size_t n)
{
    std::normal_distribution<double> d(0.0, 1.0);
    std::vector<double> v(n);
    for (double &x : v) x = d(rng);
    return v;
}

static void oracle_attention()
{
    const int B = 2, H = 2, d = 8;
    const int64_t S = 37;
    const size_t n = (size_t)B * S * H * d;
    const auto q = randn(n), k = randn(n), v = randn(n), g = randn(n);
    std::vector<double> o(n), lse((size_t)B * H * S), dq(n), dk(n), dv(n);
    memo_oracle_attn_fwd(B, S, H, d, 0.3, q.data(), k.data(), v.data(), o.data(), lse.data());
    memo_oracle_attn_bwd(B, S, H, d, 0.3, q.data(), k.data(), v.data(), g.data(), dq.data(), dk.data(), dv.data());
    for (double x : o) CHECK(std::isfinite(x));
    // the sampled entry points on head (0, 1) reproduce the dense ones exactly, buffers sized to the byte
    std::vector<double> qh((size_t)S * d), kh(qh), vh(qh), gh(qh);
    for (int64_t i = 0; i < S; ++i)
        for (int c = 0; c < d; ++c) {
            const size_t src = ((size_t)i * H + 1) * d + c;
            qh[i * d + c] = q[src], kh[i * d + c] = k[src], vh[i * d + c] = v[src], gh[i * d + c] = g[src];
        }
    const int64_t rows[3] = {0, 17, S - 1};
    std::vector<double> ro(3 * d), rl(3), rd(3), rq(3 * d);
    memo_oracle_head_rows(S, d, 0.3, qh.data(), kh.data(), vh.data(), gh.data(), 3, rows, ro.data(), rl.data(),
                          rd.data(), rq.data());
    for (int r = 0; r < 3; ++r)
        for (int c = 0; c < d; ++c) {
            CHECK(ro[r * d + c] == o[((size_t)rows[r] * H + 1) * d + c]);
            CHECK(rq[r * d + c] == dq[((size_t)rows[r] * H + 1) * d + c]);
        }
    const int64_t j0 = S - 5;
    std::vector<double> tk(5 * d), tv(5 * d);
    memo_oracle_head_dkdv_tail(S, d, 0.3, qh.data(), kh.data(), vh.data(), gh.data(), j0, tk.data(), tv.data());
    for (int t = 0; t < 5; ++t)
        for (int c = 0; c < d; ++c) {
            CHECK(tk[t * d + c] == dk[((size_t)(j0 + t) * H + 1) * d + c]);
            CHECK(tv[t * d + c] == dv[((size_t)(j0 + t) * H + 1) * d + c]);
        }
    // S = 1 and d_o = NULL
    std::vector<double> o1(d), l1(1);
    const int64_t r0 = 0;
    memo_oracle_head_rows(1, d, 1.0, qh.data(), kh.data(), vh.data(), nullptr, 1, &r0, o1.data(), l1.data(), nullptr,
                          nullptr);
    for (int c = 0; c < d; ++c) CHECK(o1[c] == vh[c]);
}

static void swap_both_sides()
{
    const double alphas[] = {0.0, 0.125, 0.5, 0.9, 1.0};
    for (double alpha : alphas)
        for (int64_t S : {1, 7, 100}) {
            const int64_t rb = 24;
            int64_t plan[5];
            CHECK(memo_oracle_swap_plan(S, rb, alpha, plan) == 0);
            memo_swap_plan lp;
            CHECK(memo_swap_plan_make(S, rb, alpha, &lp) == MEMO_OK);
            CHECK(lp.k_swapped == plan[0] && lp.n_recompute == plan[1] && lp.bytes_swapped == plan[2] &&
                  lp.bytes_dropped == plan[3] && lp.recompute_byte_offset == plan[4]);
            CHECK(memo_split_tokens(S, alpha) == memo_oracle_split_tokens(S, alpha));
            // buffers sized exactly: one byte too many copied is an address-sanitizer report
            std::vector<unsigned char> act((size_t)(S * rb)), host((size_t)plan[2]), back((size_t)(S * rb), 0x5A);
            for (size_t i = 0; i < act.size(); ++i) act[i] = (unsigned char)(i * 131 + 7);
            CHECK(memo_oracle_swap_out(act.data(), S, rb, alpha, host.data(), plan[2]) == plan[2]);
            CHECK(memo_oracle_swap_out(act.data(), S, rb, alpha, host.data(), plan[2] - 1) == -2);
            CHECK(memo_oracle_swap_in(back.data(), S, rb, alpha, host.data(), plan[2]) == plan[2]);
            // the library's copies through the fake runtime
            std::vector<unsigned char> host2((size_t)plan[2] + 1, 0xEE), back2((size_t)(S * rb), 0x5A);
            CHECK(memo_swap_out(act.data(), S, rb, alpha, host2.data(), (size_t)plan[2], nullptr, nullptr, nullptr) == MEMO_OK);
            CHECK(host2[(size_t)plan[2]] == 0xEE);
            CHECK(memo_swap_in(back2.data(), S, rb, alpha, host2.data(), (size_t)plan[2], nullptr, nullptr, nullptr) == MEMO_OK);
            CHECK(back == back2);
            if (plan[2] > 0)
                CHECK(memo_swap_out(act.data(), S, rb, alpha, host2.data(), (size_t)plan[2] - 1, nullptr, nullptr,
                                    nullptr) == MEMO_ERR_HOST_CAPACITY);
        }
    CHECK(memo_split_tokens(-1, 0.5) == -1 && memo_split_tokens(10, std::nan("")) == -1);
    CHECK(memo_oracle_split_tokens(10, 1.5) == -1);
    double a = -1.0;
    CHECK(memo_solve_alpha(1, 1, 14, 32, 1.0, 32, 1e9, &a) == MEMO_OK && a == 1.0);
    CHECK(memo_solve_alpha(1, 1, 14, 1, 9.0, 32, 1e9, &a) == MEMO_OK && std::fabs(a - 0.5) < 1e-12);
    CHECK(memo_oracle_alpha_grid(1, 1, 14, 1, 9.0, 32, 1e9, 1000) == 0.5);
    CHECK(memo_solve_alpha(1, 1, 14, 1, 1.0, 32, 1e9, &a) == MEMO_ERR_UNSUPPORTED);
    CHECK(memo_solve_alpha(1, 1, 14, 1e9, 1.0, 32, 1.0, &a) == MEMO_ERR_HOST_CAPACITY);
    CHECK(memo_solve_alpha(1, 1, 0, 1, 1.0, 32, 1.0, &a) == MEMO_ERR_INVALID_ARG);
}

static void attention_front_end()
{
    memo_attn_desc d{};
    d.B = 1, d.H = 2, d.d = 128, d.S = 300, d.dtype = MEMO_BF16, d.scale = 0.1f;
    d.stride_b = 300 * 256, d.stride_s = 256, d.stride_h = 128, d.causal = 1, d.flags = 0;
    alignas(256) static unsigned char buf[4096];
    void *p = buf;
    const int before = fake::launches;
    CHECK(memo_attn_fwd(&d, p, p, p, p, reinterpret_cast<float *>(p), nullptr) == MEMO_OK);
    const size_t need = memo_attn_bwd_workspace_bytes(&d);
    CHECK(need == 2560);
    CHECK(memo_attn_bwd(&d, p, p, p, p, reinterpret_cast<float *>(p), p, p, p, p, p, need, nullptr) == MEMO_OK);
    CHECK(fake::launches == before + 2);
    CHECK(memo_attn_bwd(&d, p, p, p, p, reinterpret_cast<float *>(p), p, p, p, p, p, need - 1, nullptr) == MEMO_ERR_WORKSPACE);
    void *ev[4] = {nullptr, nullptr, nullptr, nullptr};
    CHECK(memo_attn_bwd_staged(&d, p, p, p, p, reinterpret_cast<float *>(p), p, p, p, p, p, need, nullptr, ev) ==
          MEMO_ERR_INVALID_ARG);
    d.S = (int64_t)1 << 31;
    CHECK(memo_attn_fwd(&d, p, p, p, p, reinterpret_cast<float *>(p), nullptr) == MEMO_ERR_UNSUPPORTED);
    d.S = (int64_t)1 << 30, d.H = 1024;
    CHECK(memo_attn_fwd(&d, p, p, p, p, reinterpret_cast<float *>(p), nullptr) == MEMO_ERR_UNSUPPORTED);
    CHECK(fake::launches == before + 2);
    CHECK(memo_layernorm_rows(p, p, p, p, 10, 512, 1e-5f, 3, 10, nullptr) == MEMO_OK);
    CHECK(memo_layernorm_rows(p, p, p, p, 10, 500, 1e-5f, 3, 10, nullptr) == MEMO_ERR_UNSUPPORTED);
    CHECK(memo_linear_rows(p, p, nullptr, p, 10, 128, 256, 0, 11, nullptr) == MEMO_ERR_INVALID_ARG);
    void *hp = nullptr;
    CHECK(memo_host_alloc(&hp, 100) == MEMO_OK && hp);
    CHECK(memo_host_free(hp) == MEMO_OK);
    for (int s = 0; s < 7; ++s) CHECK(std::strlen(memo_status_str((memo_status)s)) > 0);
}

// One iteration of the rounding-buffer schedule over the fake runtime: what every backward finds
// in its buffer, then a copy that fails part-way and the handle's behaviour afterwards.
static void schedule(int n_layers, int fail_at)
{
    const int64_t S = 50;
    const memo_tensor_desc tens[3] = {{40, 1.0}, {24, 0.5}, {8, 0.0}};
    memo_tensor_slot slots[3];
    size_t dev_bytes = 0, host_bytes = 0;
    CHECK(memo_buffer_plan_make(S, 3, tens, slots, &dev_bytes, &host_bytes) == MEMO_OK);
    CHECK(slots[1].k_swapped == 25 && slots[2].bytes_swapped == 0 && dev_bytes % 256 == 0);
    std::vector<unsigned char> b0(dev_bytes), b1(dev_bytes);
    const size_t held = n_layers > 2 ? (size_t)(n_layers - 2) : 0;
    std::vector<unsigned char> host(held * host_bytes + 1);
    memo_sched *s = nullptr;
    if (held > 0)
        CHECK(memo_sched_create(&s, n_layers, S, 3, tens, b0.data(), b1.data(), host.data(), held * host_bytes - 1,
                                nullptr, nullptr, nullptr) == MEMO_ERR_HOST_CAPACITY);
    CHECK(memo_sched_create(&s, n_layers, S, 3, tens, b0.data(), b1.data(), host.data(), held * host_bytes, nullptr,
                            nullptr, nullptr) == MEMO_OK);
    fake::copies = 0;
    fake::fail_copy_at = fail_at;
    bool dead = false;
    auto expect = [&](memo_status st) {
        if (dead) {
            CHECK(st == MEMO_ERR_DEVICE);
        } else if (st == MEMO_ERR_DEVICE) {
            CHECK(fail_at >= 0);
            dead = true;
        } else {
            CHECK(st == MEMO_OK);
        }
    };
    CHECK(memo_sched_forward_end(s, 0) == MEMO_ERR_INVALID_ARG);      // out of order: refused, not fatal
    for (int i = 0; i < n_layers; ++i) {
        expect(memo_sched_forward_begin(s, i));
        unsigned char *buf = static_cast<unsigned char *>(memo_sched_buffer(s, i));
        CHECK(buf == (i % 2 ? b1.data() : b0.data()));
        if (!dead) std::memset(buf, 0x10 + i, dev_bytes);
        expect(memo_sched_forward_end(s, i));
    }
    for (int i = n_layers - 1; i >= 0; --i) {
        expect(memo_sched_backward_begin(s, i));
        if (!dead && i < n_layers - 2) {
            const unsigned char *buf = static_cast<unsigned char *>(memo_sched_buffer(s, i));
            for (int t = 0; t < 3; ++t)
                for (size_t x = 0; x < slots[t].bytes_swapped; ++x) CHECK(buf[slots[t].dev_offset + x] == 0x10 + i);
        }
        if (!dead) std::memset(memo_sched_buffer(s, i), 0xEE, dev_bytes);   // dead after its backward
        expect(memo_sched_backward_end(s, i));
    }
    CHECK(dead == (fail_at >= 0 && fail_at < (int)(4 * held)));
    if (!dead) CHECK(memo_sched_forward_begin(s, 0) == MEMO_OK);        // the next iteration starts
    CHECK(memo_sched_destroy(s) == MEMO_OK);
    CHECK(fake::events_alive == 0);
    fake::fail_copy_at = -1;
}

static void planner()
{
    std::uniform_int_distribution<int> sz(1, 9), tick(0, 7);
    for (int round = 0; round < 60; ++round) {
        const int n = 1 + round % 8;
        std::vector<memo_dsa_request> r(n);
        for (auto &q : r) {
            q.size = sz(rng) * 3;
            q.start = tick(rng);
            q.end = q.start + 1 + tick(rng) % 4;
        }
        std::vector<int64_t> addr(n);
        int64_t peak = 0;
        int32_t opt = 0;
        CHECK(memo_dsa_plan(n, r.data(), 4, round % 3 ? 100000 : 0, addr.data(), &peak, &opt) == MEMO_OK);
        for (int i = 0; i < n; ++i) {
            const int64_t si = (r[i].size + 3) / 4 * 4;
            CHECK(addr[i] % 4 == 0 && addr[i] + si <= peak);
            for (int j = 0; j < i; ++j) {
                const int64_t sj = (r[j].size + 3) / 4 * 4;
                const bool live = r[i].start < r[j].end && r[j].start < r[i].end;
                CHECK(!live || addr[i] + si <= addr[j] || addr[j] + sj <= addr[i]);
            }
        }
    }
    // request sequence -> requests, good and bad
    const int32_t is_malloc[6] = {1, 1, 0, 1, 0, 0};
    const int64_t ids[6] = {7, 8, 7, 9, 9, 8}, sizes[6] = {16, 32, 16, 8, 8, 32};
    memo_dsa_request req[6];
    int64_t out_ids[6];
    int32_t cnt = 0;
    CHECK(memo_trace_to_requests(6, is_malloc, ids, sizes, req, out_ids, &cnt) == MEMO_OK && cnt == 3);
    CHECK(req[0].start == 0 && req[0].end == 2 && req[1].end == 5 && req[2].start == 3);
    const int64_t bad_sizes[6] = {16, 32, 17, 8, 8, 32};
    CHECK(memo_trace_to_requests(6, is_malloc, ids, bad_sizes, req, out_ids, &cnt) == MEMO_ERR_INVALID_ARG);
    // two levels
    const memo_dsa_request fwd[3] = {{8, 0, 2}, {4, 1, 3}, {8, 2, 4}}, bwd[2] = {{6, 0, 2}, {6, 1, 2}};
    const memo_dsa_request outer[2] = {{10, 0, 9}, {5, 3, 6}};
    const int32_t ft[3] = {1, 2, 3}, bt[3] = {7, 6, 5};
    int64_t fo[3], bo[2], fb[3], bb[3], oa[2];
    memo_bilevel_plan plan{};
    plan.fwd_offsets = fo, plan.bwd_offsets = bo, plan.fwd_base = fb, plan.bwd_base = bb, plan.outer_addr = oa;
    CHECK(memo_dsa_plan_bilevel(3, fwd, 2, bwd, 3, ft, bt, 2, outer, 1, 100000, &plan) == MEMO_OK);
    CHECK(plan.fwd_peak == 12 && plan.bwd_peak == 12 && plan.peak >= 22 && plan.optimal == 1);
    CHECK(fb[0] == fb[1] && fb[1] == fb[2]);
}

int main()
{
    oracle_attention();
    swap_both_sides();
    attention_front_end();
    for (int n : {1, 2, 3, 5}) schedule(n, -1);
    for (int fail_at : {0, 1, 3, 6, 11, 12}) schedule(5, fail_at);
    planner();
    std::puts("host sanitizer run: ok");
    return 0;
}
