#!/usr/bin/env python3
"""Benchmark of one training round (selection + masked consensus average + local SGD step,
plus the per-worker gradients where the configuration has a model) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C]

A step is one pass of the whole hot path over one round of synthetic input that is already
resident in HBM.  Prints one JSON line.  The default workload is the consensus-only stress
configuration (128 workers, 8-regular graph, d = 11.2 M), the one the averaging-bandwidth
metric is quoted on; its parameter and gradient matrices are stored tile-major by default
(--layout rows for one row per worker; the line reports the other layout as well).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_FP32_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix

def measured_traffic(kernel: str, cid: int):
    """HBM bytes per launch from hardware counters, as tabulated in profiles/hbm_traffic.md, or None
    when there is no row for (kernel, configuration) or the kernel's source has changed since the
    counters were taken."""
    import hashlib
    try:
        rows = open(os.path.join(ROOT, "profiles", "hbm_traffic.md")).read().splitlines()
    except OSError:
        return None
    for line in rows:
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) != 5 or cells[0] != kernel or cells[1] != str(cid):
            continue
        try:
            digest = hashlib.sha256(open(os.path.join(ROOT, cells[3]), "rb").read()).hexdigest()[:16]
        except OSError:
            return None
        return float(cells[2]) if digest == cells[4] else None
    return None


def cpu_baseline(cid: int, wl_rowptr, wl_colidx, budget_s: float = 15.0):
    """The CPU oracle, as it stands, timed on this host on a bounded sample of the same
    workload; reported as worker-rounds/s.  Not the target, a reference point."""
    import numpy as np
    import oracle
    from paper_2102_06280_amd import inputs

    cfg = inputs.CONFIGS[cid]
    threads = oracle.set_threads(min(16, os.cpu_count() or 1))
    n = cfg.n
    if cfg.model == "none":
        frac = 4
        cols = cfg.d // frac
        x = inputs.flat_params(cfg, n, cols, inputs.P_PARAMS, 1.0)
        g = inputs.flat_params(cfg, n, cols, inputs.P_GRADS, 0.01)
        done, spent, t0 = 0, 0.0, time.perf_counter()
        while True:
            t = inputs.response_times(cfg, done)
            b = inputs.backup_counts(cfg, done, wl_rowptr)
            t1 = time.perf_counter()
            mask, p, _ = oracle.select(wl_rowptr, wl_colidx, t, b)
            x = oracle.round_(wl_rowptr, wl_colidx, mask, p, x, g, cfg.lr, 0)
            spent += time.perf_counter() - t1
            done += 1
            if time.perf_counter() - t0 > budget_s or done >= 8:
                break
        value = n * done / (spent * frac)
        sample = (f"{done} rounds on the first d/{frac} = {cols} columns (columns are independent), mean time per round "
                  f"scaled x{frac}")
        # the same on one thread, on an eighth of those columns
        oracle.set_threads(1)
        c1 = max(cols // 8, 1)
        x1, g1 = np.ascontiguousarray(x[:, :c1]), np.ascontiguousarray(g[:, :c1])
        t1 = time.perf_counter()
        oracle.round_(wl_rowptr, wl_colidx, mask, p, x1, g1, cfg.lr, 0)
        value_1 = n / ((time.perf_counter() - t1) * (cfg.d / c1))
    else:
        desc = inputs.model_dims(cfg.model)
        kind, od = oracle.model_desc(desc)
        ld = inputs.pad_ld(cfg.d)
        workers = list(range(min(n, threads if cid == 3 else n)))
        x = inputs.init_params(desc, n, ld, inputs.rng(cid, inputs.P_PARAMS), zero=cfg.zero_init)
        bx, by = inputs.batch(cfg, 0, workers=workers)
        t1 = time.perf_counter()
        grad, _ = oracle.grad_all(kind, od, cfg.d, x[workers], bx, by)
        t_grad = (time.perf_counter() - t1) * n / len(workers)
        t = inputs.response_times(cfg, 0)
        b = np.zeros(n, np.int32)
        g = np.zeros_like(x)
        t1 = time.perf_counter()
        mask, p, _ = oracle.select(wl_rowptr, wl_colidx, t, b)
        oracle.round_(wl_rowptr, wl_colidx, mask, p, x, g, cfg.lr, 0, d=cfg.d)
        t_mix = time.perf_counter() - t1
        value = n / (t_grad + t_mix)
        sample = (f"1 round: gradients of {len(workers)} of {n} workers (time scaled to {n}) "
                  f"+ selection and averaging of all workers")
        # the same on one thread: one worker's gradient, scaled
        oracle.set_threads(1)
        t1 = time.perf_counter()
        oracle.grad_all(kind, od, cfg.d, x[:1], bx[:1], by[:1])
        t_grad1 = (time.perf_counter() - t1) * n
        t1 = time.perf_counter()
        oracle.round_(wl_rowptr, wl_colidx, mask, p, x, g, cfg.lr, 0, d=cfg.d)
        value_1 = n / (t_grad1 + (time.perf_counter() - t1))
    oracle.set_threads(1)
    return {"value": value, "unit": "worker-rounds/s", "cores": threads, "kind": "oracle", "sample": sample,
            "value_1core": value_1}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4, choices=[1, 2, 3, 4, 5, 6, 7])
    ap.add_argument("--order", choices=["cta", "atc"], default="cta")
    ap.add_argument("--layout", choices=["rows", "tiles"], default=None,
                    help="storage layout of the parameter matrices; default: tile-major for the consensus-only "
                         "stress (config 4), rows elsewhere; the other layout is timed as well and reported")
    ap.add_argument("--ld", type=int, default=0, help="row stride in floats (default: d rounded up to 64)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="after the timed region, run three plain device copies of one N x ld parameter matrix "
                         "(known size) so that hardware byte counters can be scaled against them")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this implementation runs on exactly one GPU (all N workers are simulated on it); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2102_06280_amd import binding as B, inputs
    from paper_2102_06280_amd.workload import Workload

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = inputs.CONFIGS[args.config]
    if args.layout is None:
        args.layout = "tiles" if args.config == 4 else "rows"
    rounds = args.steps + args.warmup
    wl = Workload(args.config, min(rounds, max(cfg.rounds, 8)), order=B.ORDER_ATC if args.order == "atc" else B.ORDER_CTA,
                  ld_override=args.ld or None, layout=B.LAYOUT_TILES if args.layout == "tiles" else B.LAYOUT_ROWS)

    for _ in range(args.warmup):
        wl.step()
    B.dbw_check(wl.h)
    # The timed region: K plain steps, nothing but the library's launches on the stream.
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        wl.step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    B.dbw_check(wl.h)

    # Per-kernel durations: the same K steps once more with HIP events recorded around every
    # kernel on the launch stream.  Kept out of the timed region because two event records per
    # kernel slow a launch-bound round down by up to half; reported next to the timed figure.
    B.dbw_set_timing(wl.h, True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        wl.step()
    torch.cuda.synchronize()
    events_ms = (time.perf_counter() - t0) / args.steps * 1e3
    kern = B.dbw_get_timing(wl.h)
    B.dbw_set_timing(wl.h, False)
    B.dbw_check(wl.h)

    if args.copy_calibration:
        for _ in range(3):
            wl.x[wl.cur ^ 1].copy_(wl.x[wl.cur])
        torch.cuda.synchronize()

    # the same rounds replayed as HIP graphs (one per round): what a launch-bound
    # configuration gains from a single submission per round; reported next to the eager figure
    graph_ms = None
    if cfg.model != "none":
        graphs = wl.capture_steps(args.steps)
        wl.replay(graphs[:2])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        wl.replay(graphs)
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) / args.steps * 1e3
        del graphs

    # r gradient-free rounds (the consensus-only tail) one by one and collapsed into one pass
    # through the product of their consensus matrices; outside the timed region
    tail = None
    if cfg.model == "none" and cfg.n <= 256 and args.layout == "rows":
        r = min(8, wl.rounds)
        src, dst = wl.x[wl.cur], wl.x[wl.cur ^ 1]

        def timed(fn, reps=3):
            fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / reps * 1e3

        def single():
            a, c = src, dst
            for q in range(r):
                B.dbw_select(wl.h, wl.t[q], wl.b[q])
                B.dbw_round(wl.h, a, c, 0.0)
                a, c = c, a

        ms_single = timed(single)
        ms_collapsed = timed(lambda: B.dbw_consensus_rounds(wl.h, src, dst, wl.t[:r], wl.b[:r], r))
        tail = {"rounds": r, "ms_single_rounds": ms_single, "ms_collapsed": ms_collapsed}

    # simulated duration of a round (Section 3.2.2) with the workload's backup counts and with
    # full participation (b = 0) on the same response times; outside the timed region
    T = torch.zeros(2, device="cuda")
    zero_b = torch.zeros(cfg.n, dtype=torch.int32, device="cuda")
    dur = {"dybw": 0.0, "full": 0.0}
    for r in range(wl.rounds):
        for key, b in (("dybw", wl.b[r]), ("full", zero_b)):
            B.dbw_select(wl.h, wl.t[r], b)
            B.dbw_round_time(wl.h, T)
            dur[key] += float(T[1].item()) / wl.rounds      # T(k) over the workers somebody waits for

    ms_per_step = elapsed / args.steps * 1e3
    value = cfg.n * args.steps / elapsed

    mix_path = B.dbw_mix_path(wl.h)
    dominant = max(kern, key=lambda k: kern[k][0])
    dom_ms = kern[dominant][0] / kern[dominant][1]
    if dominant.startswith(("mix_csr", "mix_lds", "mix_tile")):
        work = 3.0 * cfg.n * cfg.d * 4          # read X, read G, write X' once each
        roofline = {"bound": "hbm", "achieved": work / (dom_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "traffic": None}
    elif dominant.startswith("mix_dense"):
        npad = 32
        while npad < cfg.n:
            npad *= 2
        work = 2.0 * cfg.n * cfg.n * cfg.d      # dense P(k) X
        roofline = {"bound": "mfma", "achieved": work / (dom_ms * 1e-3) / 1e12, "peak": MFMA_FP32_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "traffic": None}
    else:
        from paper_2102_06280_amd.flops import kernel_flops
        work = kernel_flops(cfg, dominant)
        roofline = {"bound": "mfma", "achieved": work / (dom_ms * 1e-3) / 1e12, "peak": MFMA_FP32_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "traffic": None}
    roofline["traffic"] = measured_traffic(dominant, cfg.cid)
    roofline["frac"] = roofline["achieved"] / roofline["peak"]
    roofline["kernel"] = dominant
    roofline["kernel_ms"] = dom_ms
    roofline["kernels_ms"] = {k: v[0] / v[1] for k, v in kern.items()}

    out = {
        "metric": "worker-rounds/sec", "value": value, "unit": "worker-rounds/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config {cfg.cid}: {cfg.name}", "workers": cfg.n, "graph": cfg.graph, "d": cfg.d,
                   "ld": wl.ld, "layout": args.layout, "per_worker_network": cfg.model, "per_worker_batch": cfg.batch,
                   "order": args.order,
                   "mix_path": "dense" if mix_path == B.MIX_DENSE else "csr",
                   "gradients": "one fixed supplied matrix, reused every round" if cfg.model == "none" else "computed"},
        "roofline": roofline,
        "ms_per_step_with_kernel_events": events_ms,
        "hip_graph_ms_per_step": graph_ms,
        "consensus_tail": tail,
        "simulated_round_duration": {"dybw": dur["dybw"], "full_participation": dur["full"],
                                     "shorter_by": 1.0 - dur["dybw"] / dur["full"], "rounds": wl.rounds},
    }
    rowptr, colidx = wl.rowptr, wl.colidx
    wl.close()
    del wl
    torch.cuda.empty_cache()
    # the same workload in the other storage layout, same number of steps
    if args.config == 4 and not args.ld:
        other = "rows" if args.layout == "tiles" else "tiles"
        wl2 = Workload(args.config, min(rounds, max(cfg.rounds, 8)), order=B.ORDER_ATC if args.order == "atc" else B.ORDER_CTA,
                       layout=B.LAYOUT_TILES if other == "tiles" else B.LAYOUT_ROWS)
        for _ in range(args.warmup):
            wl2.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            wl2.step()
        torch.cuda.synchronize()
        el2 = time.perf_counter() - t0
        B.dbw_set_timing(wl2.h, True)
        for _ in range(args.steps):
            wl2.step()
        k2 = B.dbw_get_timing(wl2.h)
        dom2 = max(k2, key=lambda k: k2[k][0])
        ms2 = k2[dom2][0] / k2[dom2][1]
        out["other_layout"] = {"layout": other, "value": cfg.n * args.steps / el2, "ms_per_step": el2 / args.steps * 1e3,
                               "kernel": dom2, "kernel_ms": ms2,
                               "frac": 3.0 * cfg.n * cfg.d * 4 / (ms2 * 1e-3) / 1e9 / HBM_PEAK_GBS}
        wl2.close()
        del wl2
        torch.cuda.empty_cache()
    # what plain kernels reach on this device, next to the nominal peak: a streaming triad
    # over three 1 GiB arrays, or register-resident fp32 matrix instructions
    if roofline["bound"] == "hbm":
        roofline["achievable"] = B.dbw_calibrate(B.CAL_HBM_TRIAD, 1 << 30, 10)
    else:
        roofline["achievable"] = B.dbw_calibrate(B.CAL_MFMA_FP32, 4096, 5)
    roofline["frac_of_achievable"] = roofline["achieved"] / roofline["achievable"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config, rowptr, colidx)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
