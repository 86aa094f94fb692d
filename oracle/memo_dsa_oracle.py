"""Oracle of the offline dynamic-storage-allocation problem and its bi-level use
(Section 4.2: minimise the peak M subject to A_i + S_i <= M and, for every pair with
overlapping lifespans, one of A_i + S_i <= A_j or A_j + S_j <= A_i chosen by z_ij).

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  The exact solver here is the formulation written
out: every assignment of the binary variables z_ij is tried; for a fixed assignment the
smallest feasible addresses are longest paths in the "i lies below j" graph (an
assignment with a cycle is infeasible).  Exponential in the number of overlapping pairs,
so only for tiny instances.  A request is (size, start, end) with lifespan [start, end).
"""
import itertools


def overlapping_pairs(req):
    """E of the formulation: pairs whose lifespans intersect."""
    n = len(req)
    return [(i, j) for i in range(n) for j in range(i + 1, n)
            if req[i][1] < req[j][2] and req[j][1] < req[i][2]]


def load_lower_bound(req):
    """Largest sum of sizes alive at one instant: no plan can have a smaller peak."""
    points = sorted({r[1] for r in req})
    return max((sum(r[0] for r in req if r[1] <= t < r[2]) for t in points), default=0)


def check_plan(req, addr):
    """Peak of a plan; raises if two requests with overlapping lifespans share bytes."""
    for i, j in overlapping_pairs(req):
        if not (addr[i] + req[i][0] <= addr[j] or addr[j] + req[j][0] <= addr[i]):
            raise AssertionError(f"requests {i} and {j} overlap in time and in memory")
    if any(a < 0 for a in addr):
        raise AssertionError("negative address")
    return max((a + r[0] for a, r in zip(addr, req)), default=0)


def solve_exact(req):
    """(peak, addresses) minimising the peak, by enumeration of all z_ij."""
    n = len(req)
    pairs = overlapping_pairs(req)
    best = None
    for z in itertools.product((0, 1), repeat=len(pairs)):
        below = [[] for _ in range(n)]            # below[j] = requests that must lie under j
        for (i, j), zij in zip(pairs, z):
            if zij == 0:
                below[j].append(i)                # A_i + S_i <= A_j
            else:
                below[i].append(j)                # A_j + S_j <= A_i
        addr, state, ok = [0] * n, [0] * n, True

        def visit(v):
            nonlocal ok
            if state[v] == 1:
                ok = False                        # cycle: no addresses satisfy this z
                return
            if state[v] == 2 or not ok:
                return
            state[v] = 1
            a = 0
            for u in below[v]:
                visit(u)
                if not ok:
                    return
                a = max(a, addr[u] + req[u][0])
            addr[v] = a
            state[v] = 2

        for v in range(n):
            visit(v)
            if not ok:
                break
        if not ok:
            continue
        peak = max((addr[v] + req[v][0] for v in range(n)), default=0)
        if best is None or peak < best[0]:
            best = (peak, list(addr))
    return best if best is not None else (0, [])


def trace_to_requests(events):
    """events: list of ("malloc" | "free", tensor_id, size) in program order, the form of
    Section 4.2's memory request sequence.  Returns (requests, ids): lifespan = [index of the
    malloc event, index of the free event); a tensor never freed lives to the end."""
    start, size, order = {}, {}, []
    end = {}
    for t, (op, tid, sz) in enumerate(events):
        if op == "malloc":
            if tid in start:
                raise ValueError(f"tensor {tid} allocated twice")
            start[tid], size[tid] = t, sz
            order.append(tid)
        elif op == "free":
            if tid not in start or tid in end:
                raise ValueError(f"tensor {tid} freed without a live allocation")
            if sz != size[tid]:
                raise ValueError(f"tensor {tid} freed with another size")
            end[tid] = t
        else:
            raise ValueError(op)
    T = len(events)
    return [(size[t], start[t], end.get(t, T)) for t in order], order


def bilevel(layer_fwd, layer_bwd, fwd_ticks, bwd_ticks, outer, solve=solve_exact):
    """Two-level plan of Section 4.2.  layer_fwd / layer_bwd: request lists of ONE layer's
    forward / backward pass; level 1 solves each once, every layer reuses the offsets.  Level 2
    sees the pass of layer l as one pseudo request of the level-1 peak alive during
    [fwd_ticks[l], fwd_ticks[l] + 1) (resp. bwd_ticks), next to the requests `outer` of the
    rest of the model on the same clock.  Returns dict(peak, fwd_peak, bwd_peak, fwd_offsets,
    bwd_offsets, fwd_base[l], bwd_base[l], outer_addr[i])."""
    pf, off_f = solve(layer_fwd)
    pb, off_b = solve(layer_bwd)
    req = list(outer)
    req += [(pf, t, t + 1) for t in fwd_ticks]
    req += [(pb, t, t + 1) for t in bwd_ticks]
    peak, addr = solve(req)
    no, nf = len(outer), len(fwd_ticks)
    return dict(peak=peak, fwd_peak=pf, bwd_peak=pb, fwd_offsets=off_f, bwd_offsets=off_b,
                outer_addr=addr[:no], fwd_base=addr[no:no + nf], bwd_base=addr[no + nf:],
                level2_requests=req)
