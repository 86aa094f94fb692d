#!/usr/bin/env python3
"""Benchmark of the Memo hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input that is already
resident in HBM: token split plan, swap-out of the saved activation on the offload stream
overlapped with the attention forward, swap-in on the prefetch stream overlapped with the
attention backward (D_i preprocess, dK/dV kernel, dQ kernel).

Prints ONE JSON line: whole-job attention throughput in TFLOP/s (FlashAttention convention for
causal attention: forward 2*S^2*d*H, backward 5*S^2*d*H), the roofline of the dominant kernel
measured live with HIP events on the launch stream, the swap/compute overlap, and the CPU
oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "attn fwd+bwd TFLOP/s (% bf16 MFMA peak) at S=256K/1M; swap-overlap fraction"
BF16_MFMA_PEAK_TFLOPS = 2500.0     # MI355X dense bf16, published

# HBM bytes per launch (read + write) from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes
# over this same command, scaled by what the counters read for a copy kernel of known size
# (profiles/attn_c5_counters.md).  Counters cannot be read from inside the benchmark, so the
# figures are carried here per workload; a workload that was not profiled reports null.
GIB = float(1 << 30)
TRAFFIC_SOURCE = ("carried from profiles/attn_c5_counters.md (two rocprofv3 --pmc runs of this command), not read "
                  "in this run; it varies by tens of per cent between runs with the timing of the workgroups (how long the 32 workgroups of an XCD stay in step)")
MEASURED_HBM_TRAFFIC_BYTES = {
    "C5": {"attn_fwd_bf16_kernel": (1210.9 + 1.02) * GIB,
           "attn_bwd_dkdv_bf16_kernel": (1253.5 + 2.00) * GIB,
           "attn_bwd_dq_bf16_kernel": (2136.5 + 1.00) * GIB},
}


def cpu_baseline(cfg, q, k, v, g, scale, budget_s=15.0):
    """The oracle as it stands, timed on the host cores on a bounded sample of the workload:
    exact forward + dQ rows of head 0 at uniformly spaced query positions."""
    import numpy as np
    from oracle import memo_oracle
    S, d = cfg["S"], cfg["d"]
    f64 = lambda t: t[0, :, 0, :].to("cpu").double().numpy()
    qh, kh, vh, gh = f64(q), f64(k), f64(v), f64(g)
    threads = memo_oracle.num_threads()

    def rows_for(n):
        return np.unique(np.linspace(0, S - 1, n + 2)[1:-1].astype(np.int64))

    def run(rows):
        t0 = time.perf_counter()
        memo_oracle.head_rows(qh, kh, vh, gh, rows, scale)
        dt = time.perf_counter() - t0
        # per row i: scores, P.V, dP, dQ over i+1 keys -> 4 contractions of 2*d flops each
        return dt, float(((rows + 1) * 8.0 * d).sum())

    rows = rows_for(threads)
    dt, fl = run(rows)                                   # calibration pass (counts as warm-up)
    n = int(max(threads, min(4096, len(rows) * budget_s / max(dt, 1e-3))))
    rows = rows_for(n)
    dt, fl = run(rows)
    # the dense oracle takes these 4 contractions per visible pair row by row and 4 more column by column
    # for dK and dV (it shares nothing between the two), over all heads
    dense_flop = 8.0 * float(S) * float(S) * d * cfg["H"] * cfg["B"]
    return {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"fp64 oracle forward+dQ of {len(rows)} uniformly spaced query rows of head 0 "
                      f"at S={S}, d={d} ({fl / 1e9:.1f} GFLOP in {dt:.1f} s)",
            "dense_oracle_hours_extrapolated": dense_flop / (fl / dt) / 3600.0}


def parity_check(torch, mb, synth, cfg, q, k, v, g, o, lse, dq, dk, dv, scale, n_rows=12, tail=32):
    """Bounded check of the tensors one step has just produced against the fp64 oracle, before
    anything is timed: O, LSE and dQ of uniformly spaced query rows and dK, dV of the last key
    columns of head 0 (exact oracle rows cost O(i*d) each, so this stays within seconds at 1M)."""
    import numpy as np
    from oracle import memo_oracle
    S = cfg["S"]
    f64 = lambda t: t.detach().to("cpu").double().numpy()
    qh, kh, vh, gh = (f64(t[0, :, 0, :]) for t in (q, k, v, g))
    rows = np.unique(np.concatenate([np.linspace(0, S - 1, n_rows).astype(np.int64), [S // 2 + 77]]))
    ro, rlse, _, rdq = memo_oracle.head_rows(qh, kh, vh, gh, rows, scale)
    rdk, rdv = memo_oracle.head_dkdv_tail(qh, kh, vh, gh, S - tail, scale)
    idx = torch.as_tensor(rows, device=q.device)
    pairs = {"O": (f64(o[0, idx, 0, :]), ro), "dQ": (f64(dq[0, idx, 0, :]), rdq),
             "dK": (f64(dk[0, S - tail:, 0, :]), rdk), "dV": (f64(dv[0, S - tail:, 0, :]), rdv)}
    out = {"rows": len(rows), "tail_columns": tail, "head": 0, "bars": {"max_abs": 2e-2, "rel_l2": 1e-2, "lse_max_abs": 1e-4}}
    ok = True
    for name, (got, ref) in pairs.items():
        err = np.abs(got - ref)
        rel = float(np.linalg.norm(err) / np.linalg.norm(ref))
        out[name] = {"max_abs": float(err.max()), "rel_l2": rel}
        ok = ok and np.isfinite(got).all() and err.max() <= 2e-2 and rel <= 1e-2
    lse_err = float(np.abs(f64(lse[0, 0, idx]) - rlse).max())
    out["LSE"] = {"max_abs": lse_err}
    out["ok"] = bool(ok and lse_err <= 1e-4)
    return out


def run_workload(torch, mb, synth, name, steps, warmup, overlap=True, cpu=True, calibrate_copy=False, parity=True,
                 swap=True):
    """One workload: parity check, timed steps, per-kernel events, overlap section, CPU baseline.
    Returns the JSON object."""
    cfg = synth.CONFIGS[name]
    assert cfg["dtype"] == "bf16", "bench workloads are the bf16 ones (C2..C5)"
    B, S, H, d = cfg["B"], cfg["S"], cfg["H"], cfg["d"]
    row_bytes, alpha = cfg["act_cols"] * cfg["act_elem"], cfg["alpha"]
    scale = synth.default_scale(d)
    seed = synth.config_seed(name)

    q, k, v, g = synth.attn_inputs(B, S, H, d, "bf16", seed, device="cuda")
    o = torch.empty_like(q)
    lse = torch.empty((B, H, S), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
    ws = torch.empty(mb.memo_attn_bwd_workspace_bytes(q, scale), dtype=torch.uint8, device="cuda")
    act = synth.activation(S, row_bytes, seed, device="cuda")
    act_back = torch.empty_like(act)
    plan = mb.memo_swap_plan_make(S, row_bytes, alpha)
    host = torch.empty(max(plan["bytes_swapped"], 1), dtype=torch.uint8, pin_memory=True)

    compute = torch.cuda.current_stream()
    offload, prefetch = torch.cuda.Stream(), torch.cuda.Stream()
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step(rec=None):
        """rec: dict to receive this step's timing events (None during warm-up)."""
        mb.memo_swap_plan_make(S, row_bytes, alpha)
        produced, offloaded, fetched = ev(), ev(), ev()
        f0, f1 = ev(), ev()
        stages = [ev() for _ in range(4)]
        produced.record(compute)
        if swap:
            mb.memo_swap_out(act, alpha, host, offload, wait_event=produced, done_event=offloaded)
        f0.record(compute)
        mb.memo_attn_fwd(q, k, v, scale, o=o, lse=lse)
        f1.record(compute)
        # backward of the layer: prefetch the swapped tokens while attention backward runs (the
        # copy starts once the tokens are on the host AND the forward has ended, as in the
        # schedule of Section 4.1 where a layer's swap-in runs beside a later layer's backward)
        if swap:
            prefetch.wait_event(f1)
            mb.memo_swap_in(act_back, alpha, host, prefetch, wait_event=offloaded, done_event=fetched)
        mb.memo_attn_bwd(q, k, v, o, lse, g, scale, dq=dq, dk=dk, dv=dv, workspace=ws, stage_events=stages)
        if swap:
            compute.wait_event(fetched)                  # the consumer of the activation waits here
        if rec is not None:
            rec.setdefault("fwd", []).append((f0, f1))
            rec.setdefault("stages", []).append(stages)

    parity_res = None
    if parity:
        # one untimed step, checked against the oracle before anything is timed
        step()
        torch.cuda.synchronize()
        parity_res = parity_check(torch, mb, synth, cfg, q, k, v, g, o, lse, dq, dk, dv, scale)
        assert parity_res["ok"], f"parity check failed before timing: {parity_res}"
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    rec = {}
    t0 = time.perf_counter()
    for _ in range(steps):
        step(rec)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / steps

    pairs = float(S) * float(S)                          # 2 * (S^2/2 causal pairs)
    fwd_flop = 2.0 * pairs * d * H * B
    bwd_flop = 5.0 * pairs * d * H * B
    value = (fwd_flop + bwd_flop) / (ms_per_step * 1e-3) / 1e12

    mean = lambda xs: sum(xs) / len(xs)
    fwd_ms = mean([a.elapsed_time(b) for a, b in rec["fwd"]])
    delta_ms = mean([s[0].elapsed_time(s[1]) for s in rec["stages"]])
    dkdv_ms = mean([s[1].elapsed_time(s[2]) for s in rec["stages"]])
    dq_ms = mean([s[2].elapsed_time(s[3]) for s in rec["stages"]])
    # contractions each kernel executes (2*d flops per visible (i,j) pair and contraction):
    # forward 2 (QK^T, PV); dK/dV kernel 4 (QK^T, dO V^T, P^T dO, dS^T Q); dQ kernel 3
    kernels = {
        "attn_fwd_bf16_kernel": (fwd_ms, 2.0 * pairs * d * H * B),
        "attn_bwd_dkdv_bf16_kernel": (dkdv_ms, 4.0 * pairs * d * H * B),
        "attn_bwd_dq_bf16_kernel": (dq_ms, 3.0 * pairs * d * H * B),
    }
    dom = max(kernels, key=lambda n: kernels[n][0])
    dom_ms, dom_flop = kernels[dom]
    achieved = dom_flop / (dom_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": BF16_MFMA_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / BF16_MFMA_PEAK_TFLOPS,
                "traffic": MEASURED_HBM_TRAFFIC_BYTES.get(name, {}).get(dom),
                "traffic_unit": "bytes of HBM traffic per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled)",
                "traffic_source": TRAFFIC_SOURCE if MEASURED_HBM_TRAFFIC_BYTES.get(name, {}).get(dom) else None,
                # tensors each kernel must read or write once: fwd Q,K,V,O; dK/dV Q,K,V,dO,dK,dV;
                # dQ Q,K,V,dO,dQ (the [B,H,S] statistics are 1/64 of a tensor and left out)
                "algorithmic_hbm_bytes": {"attn_fwd_bf16_kernel": 4, "attn_bwd_dkdv_bf16_kernel": 6,
                                          "attn_bwd_dq_bf16_kernel": 5}[dom] * B * S * H * d * 2,
                "avg_launch_ms": dom_ms,
                "all_kernels": {n: {"avg_ms": ms, "TFLOP/s": fl / (ms * 1e-3) / 1e12,
                                    "frac": fl / (ms * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS}
                                for n, (ms, fl) in kernels.items()},
                "delta_kernel_ms": delta_ms}

    # ---- swap/compute overlap, measured outside the timed steps -------------------------
    def timed(fn, stream_sync=True):
        torch.cuda.synchronize()
        t = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3

    def copy_out():
        e0 = ev(); e0.record(compute)
        mb.memo_swap_out(act, alpha, host, offload, wait_event=e0)

    def copy_in():
        e0 = ev(); e0.record(compute)
        mb.memo_swap_in(act_back, alpha, host, prefetch, wait_event=e0)

    def fwd_only():
        mb.memo_attn_fwd(q, k, v, scale, o=o, lse=lse)

    def bwd_only():
        mb.memo_attn_bwd(q, k, v, o, lse, g, scale, dq=dq, dk=dk, dv=dv, workspace=ws)

    if calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)                                   # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    if not overlap:
        swap = None
    else:
        swap = measure_overlap(torch, mb, timed, copy_out, copy_in, fwd_only, bwd_only, plan, alpha)
    alpha_solver = solve_alpha_for(mb, S, H, d, fwd_ms * 1e-3,
                                   swap["d2h_GBps"] * 1e9 if swap and swap["d2h_GBps"] else None)
    out = {
        "metric": METRIC, "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{name}: causal attention fwd+bwd B={B} H={H} S={S} d={d} bf16 "
                               f"N(0,1) q/k/v/dO + token-wise swap of a {S}x{cfg['act_cols']} bf16 "
                               f"activation, alpha={alpha}",
                   "flop_convention": "causal: fwd 2*S^2*d*H, bwd 5*S^2*d*H",
                   "frac_of_bf16_mfma_peak": value / BF16_MFMA_PEAK_TFLOPS,
                   "mfu_convention_TFLOPs": 6.0 * pairs * d * H * B / (ms_per_step * 1e-3) / 1e12},
        "roofline": roofline,
        "parity_before_timing": parity_res,
        "swap": swap,
        "alpha_solver": alpha_solver,
        "device": device_info(torch),
    }
    if cpu:
        ceil = mfma_ceiling(torch, mb)
        out["roofline"]["mfma_only_sustained_TFLOPs"] = {
            "zero_operands": ceil["zeros"], "normal_operands": ceil["normal"],
            "frac_of_normal": achieved / ceil["normal"],
            "note": "MFMA-only probe measured in this run; the attention inputs are N(0,1), so the "
                    "power-limited ceiling for this workload is the second figure, not the published peak"}
        out["cpu_baseline"] = cpu_baseline(cfg, q, k, v, g, scale)
    return out


def device_info(torch):
    """Name, compute-unit count and maximum clock as the runtime reports them, and the dense bf16
    MFMA peak those give (4096 flop per clock and compute unit) beside the published figure the
    roofline divides by."""
    p = torch.cuda.get_device_properties(0)
    cus = int(p.multi_processor_count)
    khz = getattr(p, "clock_rate", None)
    if not khz:                                   # not in this torch's properties: the driver's clock table
        import glob
        import re
        mhz = []
        for path in glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"):
            try:
                mhz += [int(x) for x in re.findall(r"(\d+)\s*Mhz", open(path).read(), re.I)]
            except OSError:
                pass
        khz = max(mhz) * 1000 if mhz else None
    info = {"name": p.name, "compute_units": cus, "max_clock_MHz": khz / 1e3 if khz else None,
            "published_bf16_peak_TFLOPs": BF16_MFMA_PEAK_TFLOPS}
    if khz:
        info["bf16_peak_from_units_and_clock_TFLOPs"] = cus * khz * 1e3 * 4096 / 1e12
    return info


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="C5", help="workload C2..C5 (default: the 1M-token one)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the additional S=256K workload that the default run also times")
    ap.add_argument("--no-overlap", action="store_true",
                    help="skip the separate swap/compute overlap measurement (profiling runs)")
    ap.add_argument("--no-swap", action="store_true",
                    help="attention kernels only, no swap-out/swap-in beside them (counter runs of the kernels alone; "
                         "the line then is not the benchmark's step)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy kernel (reference for HBM counters)")
    ap.add_argument("--schedule", default=None, metavar="S[,S...]",
                    help="instead of the default step: run the two-rounding-buffer schedule over "
                         "--layers stand-in layers at these sequence lengths and report the exposed "
                         "copy time per alpha")
    ap.add_argument("--recompute", default=None, metavar="S",
                    help="instead of the default step: time the token-wise recomputation kernels "
                         "(LayerNorm h=4096 and the 4096 -> 1536 projection) on rows [k,S) per alpha")
    ap.add_argument("--atomic-probe", action="store_true",
                    help="instead of the default step: measure the fp32 atomic-add rate in the access pattern a "
                         "fused backward (dQ through atomics) would produce, and what that costs at C3 and C5")
    ap.add_argument("--layers", type=int, default=6)
    ap.add_argument("--alphas", default="0,0.25,0.5,0.75,1")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one GPU's share of a tensor-parallel layer); "
              "--gpus above 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2407_12117_amd import binding as mb
    from paper_2407_12117_amd import synth

    mb.lib()                                             # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.schedule:
        schedule_bench(torch, mb, synth, args)
        return
    if args.recompute:
        recompute_bench(torch, mb, args)
        return
    if args.atomic_probe:
        atomic_probe(torch)
        return
    out = run_workload(torch, mb, synth, args.config, args.steps, args.warmup, overlap=not args.no_overlap,
                       cpu=not args.no_cpu_baseline, calibrate_copy=args.calibrate_copy, swap=not args.no_swap)
    if args.no_swap:
        out["note"] = "--no-swap: attention kernels only; not the benchmark's step"
        out["swap"] = None
    if args.config == "C5" and not args.no_extra:
        # the metric names S = 256K beside 1M: the 13B-shaped 256K workload and the two shorter ones,
        # timed the same way (no overlap section, no CPU leg), ride along in the same line
        import gc
        out["also_measured"] = {}
        for other, n_steps in (("C4", 3), ("C3", 5), ("C2", 10)):
            gc.collect()
            torch.cuda.empty_cache()
            r = run_workload(torch, mb, synth, other, n_steps, 2, overlap=False, cpu=False)
            m = {k: r[k] for k in ("value", "unit", "ms_per_step", "steps", "warmup")}
            m["workload"] = r["config"]["workload"]
            m["frac_of_bf16_mfma_peak"] = r["config"]["frac_of_bf16_mfma_peak"]
            m["kernels"] = r["roofline"]["all_kernels"]
            m["parity_before_timing"] = r["parity_before_timing"]
            out["also_measured"][other] = m
    print(json.dumps(out), flush=True)


def bench_aids():
    import ctypes
    from paper_2407_12117_amd import build as memo_build
    if not os.path.exists(memo_build.BENCH_AIDS_LIB):
        memo_build.build_bench_aids()
    return ctypes.CDLL(memo_build.BENCH_AIDS_LIB)


def atomic_probe(torch):
    """What a fused five-contraction backward would pay for dQ: a key-stationary workgroup (256 keys) has a
    32 x 128 fp32 partial dQ (16 KB) to add to global memory per query tile step, after a reduction over its
    eight key-block waves through LDS (eight times that without).  Measures the chip's rate for that pattern
    (32 KB blocks, workgroups of one head walking forward a few blocks apart) and prices the atomics alone at
    C3 and C5 against the dQ kernel they would replace."""
    import ctypes
    aids = bench_aids()
    aids.memo_bench_atomic_add.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p]
    heads, nblocks = 4, 1 << 14                          # per head 16384 blocks of 32 KB: S = 1M rows of 128 fp32
    buf = torch.zeros(heads * nblocks * 8192, dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    rows = []
    for scope, sname in ((0, "device-scope atomic add"), (1, "workgroup-scope atomic add"), (2, "plain store")):
        for wgs in (256, 2048):
            for dup in (1, 4):
                iters = 2000
                assert aids.memo_bench_atomic_add(buf.data_ptr(), nblocks, heads, wgs, 10, dup, nblocks, scope, st) == 0
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                assert aids.memo_bench_atomic_add(buf.data_ptr(), nblocks, heads, wgs, iters, dup, nblocks, scope, st) == 0
                e1.record()
                torch.cuda.synchronize()
                byt = wgs * iters * dup * 32768.0
                rows.append({"op": sname, "workgroups": wgs, "partials_per_block": dup,
                             "TB_per_s": byt / (e0.elapsed_time(e1) * 1e-3) / 1e12})
    rate = max(r["TB_per_s"] for r in rows if r["op"] == "device-scope atomic add") * 1e12
    cost = {}
    for name, S, H in (("C3", 131072, 4), ("C5", 1048576, 4)):
        steps = (S / 256.0) * (S / 32.0) / 2.0 * H       # visible (key tile, query tile) pairs
        cost[name] = {"atomic_bytes_after_lds_reduction": steps * 16384.0,
                      "atomics_alone_ms": steps * 16384.0 / rate * 1e3,
                      "atomics_alone_unreduced_ms": steps * 8 * 16384.0 / rate * 1e3}
    print(json.dumps({"metric": "fp32 atomic-add rate in the dQ pattern of a fused backward", "unit": "TB/s of operand bytes",
                      "rows": rows, "fused_backward_dq_cost": cost}), flush=True)


def mfma_ceiling(torch, mb, iters=30000):
    """The MFMA-only rate this chip sustains, measured live: 256 workgroups x 8 waves issue nothing
    but bf16 32x32x16 MFMAs on (a) zeros and (b) N(0,1) operands.  The published peak assumes the
    nominal clock; under the power limit the clock, and with it the attainable rate, depends on the
    operand bits, so the attention kernels (N(0,1) inputs) are bounded by (b), not by the peak."""
    import ctypes
    aids = bench_aids()
    aids.memo_bench_probe_mfma.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                           ctypes.c_void_p]
    aids.memo_bench_probe_mfma.restype = ctypes.c_int
    sink = torch.zeros(512, dtype=torch.float32, device="cuda")

    def probe(ops, n_iters, workgroups=256):
        rc = aids.memo_bench_probe_mfma(ops.data_ptr(), sink.data_ptr(), workgroups, n_iters,
                                        torch.cuda.current_stream().cuda_stream)
        assert rc == 0, f"memo_bench_probe_mfma failed ({rc})"
        return float(workgroups) * 8 * n_iters * 32 * 32768.0

    out = {}
    gen = torch.Generator(device="cuda").manual_seed(5)
    for name in ("zeros", "normal"):
        n = 256 * 512 * 128
        ops = torch.zeros(n, dtype=torch.bfloat16, device="cuda") if name == "zeros" else \
            torch.randn(n, generator=gen, device="cuda").to(torch.bfloat16)
        probe(ops, 200)                                    # warm-up
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flop = probe(ops, iters)
        e1.record()
        torch.cuda.synchronize()
        out[name] = flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
    return out


def solve_alpha_for(mb, S, H, d, t_fwd_s, bandwidth, n_layers=32, m_cpu=2.0 * 2 ** 40 / 8):
    """The alpha problem of Section 4.1 fed with what this run measured: T_layer = the attention
    forward alone (a lower bound of the layer's forward, so alpha is a lower bound too), B = the
    measured device-to-host rate.  Sizes are one GPU's share of a layer: input and attention
    output S*H*d 16-bit elements each, the other saved tensors 14 times that (16 in all);
    n = 32 layers and 2 TiB of host memory shared by 8 GPUs, as in the paper's 7B setting."""
    if bandwidth is None:
        return None
    unit = float(S) * H * d * 2
    res = {"s_in_bytes": unit, "s_attn_bytes": unit, "s_oth_bytes": 14 * unit,
           "bandwidth_GBps": bandwidth / 1e9, "t_layer_s": t_fwd_s, "n_layers": n_layers,
           "m_cpu_bytes": m_cpu}
    try:
        res["alpha"] = mb.memo_solve_alpha(unit, unit, 14 * unit, bandwidth, t_fwd_s, n_layers, m_cpu)
        a_time = (t_fwd_s * bandwidth - 2 * unit) / (14 * unit)
        a_mem = (m_cpu / (n_layers - 2) - 2 * unit) / (14 * unit)
        res["binding"] = "none" if res["alpha"] >= 1.0 else ("time" if a_time <= a_mem else "host memory")
    except mb.MemoError as e:
        res["alpha"], res["binding"] = None, str(e)
    return res


def measure_overlap(torch, mb, timed, copy_out, copy_in, fwd_only, bwd_only, plan, alpha):
    med = lambda fn: sorted(timed(fn) for _ in range(3))[1]     # median of three
    t_out, t_in = med(copy_out), med(copy_in)
    t_f, t_b = med(fwd_only), med(bwd_only)
    t_f_out = med(lambda: (copy_out(), fwd_only()))
    t_b_in = med(lambda: (copy_in(), bwd_only()))
    nbytes = plan["bytes_swapped"]
    hidden = lambda ta, tc, tac: max(0.0, min(1.0, (ta + tc - tac) / tc)) if tc > 0 else 1.0
    swap = {
        "bytes_swapped": nbytes, "alpha": alpha, "k_swapped": plan["k_swapped"],
        "d2h_GBps": nbytes / (t_out * 1e-3) / 1e9 if nbytes else None,
        "h2d_GBps": nbytes / (t_in * 1e-3) / 1e9 if nbytes else None,
        "swap_out_ms": t_out, "swap_in_ms": t_in, "fwd_alone_ms": t_f, "bwd_alone_ms": t_b,
        "fwd_with_swap_out_ms": t_f_out, "bwd_with_swap_in_ms": t_b_in,
        "hidden_fraction_swap_out": hidden(t_f, t_out, t_f_out),
        "hidden_fraction_swap_in": hidden(t_b, t_in, t_b_in),
        "attn_slowdown_fwd": t_f_out / t_f if t_f_out > t_f else 1.0,
        "attn_slowdown_bwd": t_b_in / t_b if t_b_in > t_b else 1.0,
        "repeats": "median of 3 for every timing above",
    }

    return swap


def recompute_bench(torch, mb, args):
    """Token-wise recomputation (Section 4.1) of one GPU's share of a 7B layer: input_norm =
    LayerNorm(x) over h = 4096 and q,k,v = input_norm . W^T (N = 1536) on the dropped rows [k,S).
    LayerNorm is HBM-bound (reads and writes h bf16 per row), the projection MFMA-bound
    (2*K*N flop per row); both are timed with events on the launch stream."""
    S, h, N, eps = int(args.recompute), 4096, 1536, 1e-5
    gen = torch.Generator(device="cuda").manual_seed(77)
    x = torch.randn((S, h), generator=gen, device="cuda").to(torch.bfloat16)
    gamma = torch.ones(h, dtype=torch.bfloat16, device="cuda")
    beta = torch.zeros(h, dtype=torch.bfloat16, device="cuda")
    w = (torch.randn((N, h), generator=gen, device="cuda") / h ** 0.5).to(torch.bfloat16)
    bias = torch.zeros(N, dtype=torch.bfloat16, device="cuda")
    norm = torch.empty_like(x)
    qkv = torch.empty((S, N), dtype=torch.bfloat16, device="cuda")
    ev = lambda: torch.cuda.Event(enable_timing=True)
    rows_out = []
    for alpha in [float(a) for a in args.alphas.split(",")]:
        k = mb.memo_split_tokens(S, alpha)
        n = S - k
        t_ln = t_lin = 0.0
        reps = max(1, args.steps)
        for r in range(args.warmup + reps):
            e = [ev() for _ in range(3)]
            e[0].record()
            mb.memo_layernorm_rows(x, gamma, beta, eps, y=norm, rows=(k, S))
            e[1].record()
            mb.memo_linear_rows(norm, w, bias, out=qkv, rows=(k, S))
            e[2].record()
            torch.cuda.synchronize()
            if r >= args.warmup:
                t_ln += e[0].elapsed_time(e[1]) / reps
                t_lin += e[1].elapsed_time(e[2]) / reps
        ln_bytes, lin_flop = 2.0 * n * h * 2, 2.0 * n * h * N
        rows_out.append({"alpha": alpha, "rows_recomputed": n, "layernorm_ms": t_ln, "linear_ms": t_lin,
                         "layernorm_GBps": ln_bytes / (t_ln * 1e-3) / 1e9 if n else None,
                         "linear_TFLOPs": lin_flop / (t_lin * 1e-3) / 1e12 if n else None})
    full = rows_out[0] if rows_out and rows_out[0]["rows_recomputed"] == S else None
    # context, not part of the path: the vendor library's GEMM of the same shape on the same data
    lib_ms = 0.0
    for r in range(args.warmup + max(1, args.steps)):
        e0, e1 = ev(), ev()
        e0.record()
        torch.matmul(norm, w.t(), out=qkv)
        e1.record()
        torch.cuda.synchronize()
        if r >= args.warmup:
            lib_ms += e0.elapsed_time(e1) / max(1, args.steps)
    out = {"metric": "token-wise recomputation of input_norm and q,k,v", "unit": "ms", "S": S, "h": h, "N": N,
           "rows": rows_out,
           "library_gemm_all_rows": {"what": "torch.matmul (hipBLASLt), no bias, same operands", "ms": lib_ms,
                                     "TFLOPs": 2.0 * S * h * N / (lib_ms * 1e-3) / 1e12},
           "roofline_layernorm": None if not full else {"bound": "hbm", "achieved": full["layernorm_GBps"], "peak": 8000.0,
                                                        "unit": "GB/s", "frac": full["layernorm_GBps"] / 8000.0},
           "roofline_linear": None if not full else {"bound": "mfma", "achieved": full["linear_TFLOPs"],
                                                     "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                                                     "frac": full["linear_TFLOPs"] / BF16_MFMA_PEAK_TFLOPS}}
    print(json.dumps(out), flush=True)


def schedule_bench(torch, mb, synth, args):
    """Exposed copy time of the rounding-buffer schedule (Section 4.1, Figure 5) against alpha:
    one training iteration over n stand-in layers (H = 4 heads of d = 128, 16 saved tensors of
    S x 1 KiB per layer) with swap, minus the same iteration with every layer resident; beside it
    what three queues that never slow each other would leave exposed given the measured per-layer
    times and copy rates (each swapped layer pays the excess of its copy over the pass it hides
    behind, forward and backward), and the alpha the solver picks for them."""
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import layer_stack as ls                     # the harness of stand-in layers lives beside the tests
    H, d, n = 4, 128, args.layers
    scale = synth.default_scale(d)
    alphas = [float(a) for a in args.alphas.split(",")]
    rows = []
    # One set of streams for every stack: HIP maps streams onto 4 hardware queues, and a stack whose
    # copy stream shares a queue with its compute stream would not overlap anything.
    streams = tuple(torch.cuda.Stream() for _ in range(3))

    def run(stack, x0, g, iters):
        """Median wall time of one iteration (forward + backward, synchronised at its ends)."""
        times = []
        for i in range(iters + 1):                         # the first iteration is a warm-up
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            stack.forward(x0)
            stack.backward(g)
            torch.cuda.synchronize()
            if i > 0:
                times.append(time.perf_counter() - t0)
        times.sort()
        return times[len(times) // 2]

    for S in [int(x) for x in args.schedule.split(",")]:
        gen = torch.Generator(device="cuda").manual_seed(4242)
        x0 = torch.randn((S, H * d), generator=gen, device="cuda").to(torch.bfloat16)
        g = torch.randn((S, H * d), generator=gen, device="cuda").to(torch.bfloat16)
        iters = max(3, args.steps)
        res = ls.LayerStack(n, S, H, d, 1.0, scale, swap=False, streams=streams)
        t_res = run(res, x0, g, iters)
        torch.cuda.synchronize()
        t0 = time.perf_counter(); res.forward(x0); torch.cuda.synchronize()
        t_fwd = (time.perf_counter() - t0) / n
        t_bwd = t_res / n - t_fwd
        res.close(); del res
        torch.cuda.empty_cache()
        # copy rates on this machine, both directions, on one layer's worth of bytes
        _, _, layer_host = mb.memo_buffer_plan_make(S, ls.layer_tensors(H, d, 1.0))
        host = torch.empty(max(n - 2, 1) * layer_host, dtype=torch.uint8, pin_memory=True)
        probe = torch.empty(layer_host, dtype=torch.uint8, device="cuda")
        for i in range(max(n - 2, 1)):                     # first touch of every pinned page, untimed
            host[i * layer_host:(i + 1) * layer_host].copy_(probe, non_blocking=True)
        torch.cuda.synchronize()
        side = streams[1]
        rate = {}
        for name, fn in (("d2h", mb.memo_swap_out), ("h2d", mb.memo_swap_in)):
            fn(probe.view(S, -1), 1.0, host, side); torch.cuda.synchronize()
            t0 = time.perf_counter(); fn(probe.view(S, -1), 1.0, host, side); torch.cuda.synchronize()
            rate[name] = layer_host / (time.perf_counter() - t0)
        del probe
        unit = float(S) * H * d * 2
        try:
            a_star = mb.memo_solve_alpha(unit, unit, 14 * unit, rate["d2h"], t_fwd, n, 1e18)
        except mb.MemoError:
            a_star = None
        for alpha in alphas + ([round(a_star, 3)] if a_star is not None and a_star < 1.0 else []):
            st = ls.LayerStack(n, S, H, d, alpha, scale, swap=True, host=host, streams=streams)
            t_swap = run(st, x0, g, iters)
            hb = st.host_bytes
            st.close(); del st
            torch.cuda.empty_cache()
            pred = {"exposed": max(0, n - 2) * (max(0.0, hb / rate["d2h"] - t_fwd) +
                                                max(0.0, hb / rate["h2d"] - t_bwd))}
            rows.append({"S": S, "alpha": alpha, "layer_host_bytes": hb,
                         "iter_resident_ms": t_res * 1e3, "iter_swapped_ms": t_swap * 1e3,
                         "exposed_ms": (t_swap - t_res) * 1e3,
                         "exposed_predicted_ms": pred["exposed"] * 1e3,
                         "t_fwd_layer_ms": t_fwd * 1e3, "t_bwd_layer_ms": t_bwd * 1e3,
                         "t_out_ms": hb / rate["d2h"] * 1e3, "t_in_ms": hb / rate["h2d"] * 1e3,
                         "alpha_solved": a_star})
            print(f"[schedule] S={S} alpha={alpha} resident {t_res * 1e3:.1f} ms swapped "
                  f"{t_swap * 1e3:.1f} ms exposed {(t_swap - t_res) * 1e3:.1f} ms "
                  f"(predicted {pred['exposed'] * 1e3:.1f})", file=sys.stderr, flush=True)
        del host
    print(json.dumps({"metric": "exposed copy time of the two-rounding-buffer schedule",
                      "unit": "ms per iteration", "layers": n, "H": H, "d": d,
                      "saved_tensors_per_layer": ls.N_SAVED, "rows": rows}), flush=True)


if __name__ == "__main__":
    main()
