// Offline dynamic storage allocation for the transient tensors of a training iteration and
// its two-level use over identical layers (Section 4.2).  Host code only.
//
// The paper hands the mixed-integer programme to a commercial solver; here the same optimum
// is searched directly.  An optimal plan sorted by address is reproduced by placing the
// requests in that order, each at the lowest address free of the already placed requests it
// overlaps in time; so a depth-first search over placement orders with that rule is exact.
// It is pruned by the best peak found so far, by the load bound (largest sum of sizes alive
// at one instant) and by keeping addresses non-decreasing along an order (any other order
// reaches the same plan through a sorted one).  A node budget bounds the work: when it runs
// out the best plan found is returned and flagged as not proven optimal.
#include <algorithm>
#include <cstdint>
#include <numeric>
#include <vector>

#include "../../include/memo.h"

namespace {

struct Req { int64_t size; int32_t start, end; };

inline int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

struct Solver {
    std::vector<Req> req;                 // sizes already rounded up to the alignment
    std::vector<std::vector<int>> nb;     // time-overlapping neighbours
    int n = 0;
    int64_t lower = 0, best = 0, nodes = 0, node_limit = 0;
    std::vector<int64_t> addr, best_addr;
    std::vector<char> placed;
    bool exhausted = false;

    int64_t first_fit(int i) const
    {
        // lowest address at which request i clears every placed neighbour
        std::vector<std::pair<int64_t, int64_t>> busy;
        for (int j : nb[i])
            if (placed[j]) busy.emplace_back(addr[j], addr[j] + req[j].size);
        std::sort(busy.begin(), busy.end());
        int64_t x = 0;
        for (const auto &b : busy) {
            if (x + req[i].size <= b.first) break;
            x = std::max(x, b.second);
        }
        return x;
    }

    int64_t load_bound() const
    {
        int64_t lb = 0;
        for (int i = 0; i < n; ++i) {
            int64_t live = 0;
            for (int j = 0; j < n; ++j)
                if (req[j].start <= req[i].start && req[i].start < req[j].end) live += req[j].size;
            lb = std::max(lb, live);
        }
        return lb;
    }

    // one placement order, no search: an upper bound to start from
    void greedy(const std::vector<int> &order)
    {
        std::fill(placed.begin(), placed.end(), 0);
        int64_t peak = 0;
        for (int i : order) {
            addr[i] = first_fit(i);
            placed[i] = 1;
            peak = std::max(peak, addr[i] + req[i].size);
        }
        if (best_addr.empty() || peak < best) {
            best = peak;
            best_addr = addr;
        }
        std::fill(placed.begin(), placed.end(), 0);
    }

    void dfs(int depth, int64_t peak, int64_t last_addr)
    {
        if (best == lower || exhausted) return;
        if (depth == n) {
            if (peak < best) {
                best = peak;
                best_addr = addr;
            }
            return;
        }
        if (++nodes > node_limit) {
            exhausted = true;
            return;
        }
        // candidates: every unplaced request at its lowest address, lowest address first
        std::vector<std::pair<int64_t, int>> cand;
        for (int i = 0; i < n; ++i) {
            if (placed[i]) continue;
            const int64_t x = first_fit(i);
            if (x + req[i].size >= best) return;     // this request ends at or above x + size in every completion
            if (x >= last_addr) cand.emplace_back(x, i);
        }
        std::sort(cand.begin(), cand.end(), [&](const auto &a, const auto &b) {
            return a.first != b.first ? a.first < b.first : req[a.second].size > req[b.second].size;
        });
        for (const auto &c : cand) {
            const int i = c.second;
            addr[i] = c.first;
            placed[i] = 1;
            dfs(depth + 1, std::max(peak, c.first + req[i].size), c.first);
            placed[i] = 0;
            if (best == lower || exhausted) return;
        }
    }
};

memo_status solve(int32_t n, const memo_dsa_request *in, int64_t align, int64_t node_limit,
                  int64_t *addr_out, int64_t *peak_out, int32_t *optimal_out)
{
    if (n < 0 || (n > 0 && (!in || !addr_out)) || !peak_out) return MEMO_ERR_INVALID_ARG;
    if (align < 1 || (align & (align - 1)) || node_limit < 0) return MEMO_ERR_INVALID_ARG;
    Solver s;
    s.n = n;
    s.req.resize(n);
    for (int i = 0; i < n; ++i) {
        if (in[i].size < 0 || in[i].end <= in[i].start || in[i].start < 0) return MEMO_ERR_INVALID_ARG;
        if (in[i].size > (INT64_MAX >> 8) / std::max(n, 1)) return MEMO_ERR_INVALID_ARG;   // sums stay in range
        s.req[i] = {align_up(in[i].size, align), in[i].start, in[i].end};
    }
    s.nb.assign(n, {});
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j)
            if (i != j && s.req[i].start < s.req[j].end && s.req[j].start < s.req[i].end) s.nb[i].push_back(j);
    s.addr.assign(n, 0);
    s.placed.assign(n, 0);
    s.lower = s.load_bound();
    s.node_limit = node_limit;
    std::vector<int> order(n);
    std::iota(order.begin(), order.end(), 0);
    s.best = 0;
    if (n > 0) {
        // starting plans: by size, by size x lifetime, by start time (what an online allocator sees)
        auto by = [&](auto key) {
            std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return key(a) > key(b); });
            s.greedy(order);
        };
        by([&](int i) { return s.req[i].size; });
        by([&](int i) { return s.req[i].size * (int64_t)(s.req[i].end - s.req[i].start); });
        by([&](int i) { return -(int64_t)s.req[i].start; });
        s.dfs(0, 0, 0);
    }
    for (int i = 0; i < n; ++i) addr_out[i] = s.best_addr[i];
    *peak_out = n > 0 ? s.best : 0;
    if (optimal_out) *optimal_out = (n == 0 || s.best == s.lower || !s.exhausted) ? 1 : 0;
    return MEMO_OK;
}

}  // namespace

extern "C" {

memo_status memo_trace_to_requests(int32_t n_events, const int32_t *is_malloc, const int64_t *tensor_id,
                                   const int64_t *size, memo_dsa_request *req_out, int64_t *id_out,
                                   int32_t *n_requests_out)
{
    if (n_events < 0 || !n_requests_out ||
        (n_events > 0 && (!is_malloc || !tensor_id || !size || !req_out || !id_out)))
        return MEMO_ERR_INVALID_ARG;
    int32_t n = 0;
    for (int32_t t = 0; t < n_events; ++t) {
        if (size[t] < 0) return MEMO_ERR_INVALID_ARG;
        int32_t live = -1;
        for (int32_t r = 0; r < n; ++r)
            if (id_out[r] == tensor_id[t] && req_out[r].end < 0) live = r;
        if (is_malloc[t]) {
            if (live >= 0) return MEMO_ERR_INVALID_ARG;            // allocated twice
            req_out[n].size = size[t];
            req_out[n].start = t;
            req_out[n].end = -1;
            id_out[n] = tensor_id[t];
            ++n;
        } else {
            if (live < 0 || req_out[live].size != size[t]) return MEMO_ERR_INVALID_ARG;
            req_out[live].end = t;
        }
    }
    for (int32_t r = 0; r < n; ++r)
        if (req_out[r].end < 0) req_out[r].end = n_events;         // never freed: alive to the end
    *n_requests_out = n;
    return MEMO_OK;
}

memo_status memo_dsa_plan(int32_t n, const memo_dsa_request *requests, int64_t align, int64_t node_limit,
                          int64_t *addr_out, int64_t *peak_out, int32_t *optimal_out)
{
    return solve(n, requests, align, node_limit, addr_out, peak_out, optimal_out);
}

memo_status memo_dsa_plan_bilevel(int32_t n_fwd, const memo_dsa_request *layer_fwd, int32_t n_bwd,
                                  const memo_dsa_request *layer_bwd, int32_t n_layers, const int32_t *fwd_ticks,
                                  const int32_t *bwd_ticks, int32_t n_outer, const memo_dsa_request *outer,
                                  int64_t align, int64_t node_limit, memo_bilevel_plan *out)
{
    if (!out || n_layers < 0 || n_outer < 0 || (n_layers > 0 && (!fwd_ticks || !bwd_ticks))) return MEMO_ERR_INVALID_ARG;
    if (n_outer > 0 && !outer) return MEMO_ERR_INVALID_ARG;
    if ((n_fwd > 0 && !out->fwd_offsets) || (n_bwd > 0 && !out->bwd_offsets) ||
        (n_layers > 0 && (!out->fwd_base || !out->bwd_base)) || (n_outer > 0 && !out->outer_addr))
        return MEMO_ERR_INVALID_ARG;
    int32_t opt_f = 1, opt_b = 1, opt_2 = 1;
    memo_status st = solve(n_fwd, layer_fwd, align, node_limit, out->fwd_offsets, &out->fwd_peak, &opt_f);
    if (st != MEMO_OK) return st;
    st = solve(n_bwd, layer_bwd, align, node_limit, out->bwd_offsets, &out->bwd_peak, &opt_b);
    if (st != MEMO_OK) return st;
    // level 2: the rest of the model plus one pseudo request per layer pass
    const int32_t n2 = n_outer + 2 * n_layers;
    std::vector<memo_dsa_request> req(n2);
    for (int32_t i = 0; i < n_outer; ++i) req[i] = outer[i];
    for (int32_t l = 0; l < n_layers; ++l) {
        if (fwd_ticks[l] < 0 || bwd_ticks[l] < 0) return MEMO_ERR_INVALID_ARG;
        req[n_outer + l] = {out->fwd_peak > 0 ? out->fwd_peak : 0, fwd_ticks[l], fwd_ticks[l] + 1};
        req[n_outer + n_layers + l] = {out->bwd_peak > 0 ? out->bwd_peak : 0, bwd_ticks[l], bwd_ticks[l] + 1};
    }
    std::vector<int64_t> addr(n2);
    st = solve(n2, req.data(), align, node_limit, addr.data(), &out->peak, &opt_2);
    if (st != MEMO_OK) return st;
    for (int32_t i = 0; i < n_outer; ++i) out->outer_addr[i] = addr[i];
    for (int32_t l = 0; l < n_layers; ++l) {
        out->fwd_base[l] = addr[n_outer + l];
        out->bwd_base[l] = addr[n_outer + n_layers + l];
    }
    out->optimal = opt_f && opt_b && opt_2;
    return MEMO_OK;
}

}  // extern "C"
