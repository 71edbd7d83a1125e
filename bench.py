#!/usr/bin/env python3
"""Benchmark of the online-learner hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic workload already resident in
HBM: reset the state, run all T rounds of all R runs (round kernel + meta kernel), export
the final iterates / Hedge weights / combined iterate, and read back the regret.  The
metric is learner-updates per second, R*K*T*d / time.

Prints ONE JSON line.  `roofline` prices the dominant kernel (the round kernel: all its launches
of a step, timed with HIP events on the library's stream inside the timed region) against the
resource that bounds it; `cpu_baseline` times the fp64 reference on the host cores on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_TFLOPS = 157.3     # MI355X vector fp32 (256 CUs x 2.4 GHz x 128 lanes x 2, packed)
PEAK_HBM_GBS = 8000.0

DESCR = {
    "c1": "c1: single projected OGD, linear loss, d=10 T=1000 K=1 R=1",
    "c2": "c2: K=15 OGD + Hedge, squared loss, d=100 T=10000 R=64, per-run streams",
    "c3": "c3: K=17 OGD + Hedge, squared loss, piecewise-stationary comparator, d=1000 T=100000 R=256",
    "c4": "c4: K=16 OGD + Hedge, logistic loss, shared stream, d=4096 T=20000 R=1024",
    "c5": "c5: K=8 OGD + Hedge, sparse squared loss (32 nnz/round), d=2^20 T=100000 R=16",
}


def roofline_model(wl):
    """Algorithmic work of the round kernels of ONE step (all T rounds of all runs; the library
    enqueues a long call as several launches of the same kernel).

    dense: per learner-coordinate-round 7 flops (inner product 2, gradient step 2, norm of the
    stepped vector 2, projection scale 1) plus the comparator's inner product (2 per
    run-coordinate-round).  sparse: per touched learner coordinate 4 B read + 4 B written,
    plus the round stream (8 B per entry), labels (4 B per run-round) and the comparator's
    gathers (4 B per run-entry)."""
    if wl.nnz:
        b = (wl.R * wl.K * wl.T * wl.nnz * 8 + wl.T * wl.nnz * 8 + wl.R * wl.T * 4
             + wl.R * wl.T * wl.nnz * 4)
        return "hbm", float(b), PEAK_HBM_GBS, "GB/s", 1e9
    f = 7.0 * wl.units + 2.0 * wl.R * wl.T * wl.d
    return "alu", f, PEAK_FP32_TFLOPS, "TFLOP/s", 1e12


def run_workload(name, steps, warmup, WL, B, torch, keep=None, optimistic=False):
    wl = WL.make(name, optimistic=optimistic)
    data = WL.generate(wl)
    sim = B.Simulation(wl, data)
    W = torch.empty((wl.R, wl.K, wl.d), dtype=torch.float32, device="cuda")
    p = torch.empty((wl.R, wl.K), dtype=torch.float32, device="cuda")
    wbar = torch.empty((wl.R, wl.d), dtype=torch.float32, device="cuda")
    B.oco_set_timing(sim.h, True)

    def step():
        sim.reset()
        sim.run(0, wl.T)
        B.oco_get_state(sim.h, W, p, wbar)
        return sim.regret()          # synchronises the stream

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    kern_ms = []
    t0 = time.perf_counter()
    for _ in range(steps):
        reg = step()
        kern_ms.append(B.oco_last_timing(sim.h))
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = 1e3 * dt / steps
    out = dict(wl=wl, ms_per_step=ms, value=wl.units / (dt / steps),
               round_kernel_ms=float(sum(k[0] for k in kern_ms) / steps),
               meta_kernel_ms=float(sum(k[1] for k in kern_ms) / steps),
               regret_mean=float(reg.mean()))
    if keep is not None:
        keep.update(data=data, regret=reg, accel=sim.accel_bounds(4, 0.05))
    sim.close()
    del sim, W, p, wbar
    torch.cuda.empty_cache()
    return out


def run_specdec(name, reps, WL, B, torch, with_cpu=False):
    """The verification step of Algorithm 1 (next row of the scope table) on one synthetic batch:
    sd_verify and sd_acceptance timed per launch with events on the launch stream.  Between
    launches a 1 GiB buffer is read through, so that no row of the previous launch is still in
    the 256 MB Infinity Cache (a write pass alone would leave dirty lines whose write-back then
    competes with the timed kernel's reads)."""
    import numpy as np
    shape = WL.SPECDEC[name]
    d = WL.specdec_inputs(seed=1, **shape)
    dev = torch.device("cuda:0")
    p, q = torch.from_numpy(d["p"]).to(dev), torch.from_numpy(d["q"]).to(dev)
    tok, r = torch.from_numpy(d["tok"]).to(dev), torch.from_numpy(d["r"]).to(dev)
    u = torch.from_numpy(d["u"].view(np.int32)).to(dev)
    Bn, k, V = d["q"].shape
    n = torch.empty((Bn,), dtype=torch.int32, device=dev)
    nx = torch.empty_like(n)
    acc = torch.empty((Bn, k), dtype=torch.float64, device=dev)
    flush = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
    tv, ta = [], []
    for rep in range(reps + 1):
        flush.sum()
        e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        e[0].record()
        B.sd_verify(p, q, tok, r, u, n, nx)
        e[1].record()
        flush.sum()
        e2 = torch.cuda.Event(enable_timing=True)
        e2.record()
        B.sd_acceptance(p, q, acc)
        e[2].record()
        torch.cuda.synchronize()
        if rep:                                   # first launch is the warm-up
            tv.append(e[0].elapsed_time(e[1]))
            ta.append(e2.elapsed_time(e[2]))
    nn = n.cpu().numpy()
    rows = float(((nn < k) * 2 + (nn >= k)).sum())
    bytes_v = rows * V * 4 + Bn * k * 20.0        # rows needed + gathered scalars (tok, r, p, q) + outputs
    bytes_a = float(Bn) * k * 2 * V * 4
    mv, ma = sum(tv) / len(tv), sum(ta) / len(ta)
    out = {"shape": shape, "mean_accepted": float(nn.mean()),
           "verify": {"ms": mv, "steps_per_s": Bn / (mv * 1e-3),
                      "roofline": {"bound": "hbm", "achieved": bytes_v / (mv * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                                   "unit": "GB/s", "frac": bytes_v / (mv * 1e-3) / 1e9 / PEAK_HBM_GBS}},
           "acceptance": {"ms": ma,
                          "roofline": {"bound": "hbm", "achieved": bytes_a / (ma * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                                       "unit": "GB/s", "frac": bytes_a / (ma * 1e-3) / 1e9 / PEAK_HBM_GBS}}}
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        tr = json.load(open(tpath))
        out["verify"]["roofline"]["traffic"] = tr.get(name + "_verify")
        out["acceptance"]["roofline"]["traffic"] = tr.get(name + "_acceptance")
    if with_cpu:
        from oracle import specdec_oracle as SO
        m = min(Bn, 256)
        t0 = time.perf_counter()
        rn, rnx = SO.verify(d["p"][:m], d["q"][:m], d["tok"][:m], d["r"][:m], d["u"][:m])
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": m / dt, "unit": "steps/s", "cores": 1, "kind": "oracle",
                               "sample": "%d of %d steps, %.2f s wall" % (m, Bn, dt)}
        out["parity_exact"] = bool((rn == nn[:m]).all() and (rnx == nx.cpu().numpy()[:m]).all())
    del p, q, flush
    torch.cuda.empty_cache()
    return out


def cpu_baseline(wl, data, WL):
    """The fp64 reference as it stands, one run per thread, on a bounded sample."""
    from oracle import oracle as O
    cores = min(16, os.cpu_count() or 1)
    runs = list(range(min(wl.R, cores if wl.name != "c2" else wl.R)))
    T = wl.T if wl.name != "c5" else 5000
    swl, sdat = WL.run_slice(wl, data, runs)
    if T != wl.T:
        from dataclasses import replace
        swl = replace(swl, T=T)
        sdat = dict(sdat)
        for k in ("x", "col", "val"):
            if sdat.get(k) is not None:
                sdat[k] = sdat[k][..., :T, :]
        sdat["y"] = sdat["y"][:, :T].copy()
        sdat["seg_start"] = sdat["seg_start"][sdat["seg_start"] < T]
        sdat["u"] = sdat["u"][:, : len(sdat["seg_start"])].copy()
    t0 = time.perf_counter()
    ref = O.run_workload(swl, sdat, threads=cores)
    dt = time.perf_counter() - t0
    return dict(value=swl.units / dt, unit="learner-updates/s", cores=int(ref["threads"]), kind="oracle",
                sample="%d of %d runs, %d of %d rounds, fp64, one run per thread, %.2f s wall" % (
                    len(runs), wl.R, T, wl.T, dt)), ref, runs, T


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="c4", choices=sorted(DESCR) + ["v2", "v3"])
    ap.add_argument("--no-others", action="store_true", help="skip the short runs of the other workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU baseline")
    ap.add_argument("--copy-probe", action="store_true",
                    help="only run a plain 1 GiB device copy three times (calibrates HBM byte counters)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this path runs on ONE GPU (runs are independent and would shard with no "
              "communication, but nothing here uses a second device); got --gpus %d" % a.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2603_12617_amd import binding as B
    from paper_2603_12617_amd import workloads as WL
    B.lib()                       # raises if the HIP library is not built: no fallback
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3

    if a.copy_probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read": src.numel() * 4, "copy_probe_bytes_written": src.numel() * 4}))
        return 0

    if a.config in ("v2", "v3"):       # the verification kernels alone (used for their rocprofv3 summaries)
        print(json.dumps({"workload": "specdec " + a.config, **run_specdec(a.config, a.steps, WL, B, torch)}))
        return 0

    keep = {}
    main_res = run_workload(a.config, a.steps, a.warmup, WL, B, torch, keep)
    wl = main_res["wl"]
    bound, work, peak, unit, scale = roofline_model(wl)
    achieved = work / (main_res["round_kernel_ms"] * 1e-3) / scale
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(a.config)
    line = {
        "metric": "learner-updates/sec (runs x K x rounds x d / s)",
        "value": main_res["value"], "unit": "learner-updates/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 iterates, f64 losses/weights/regret", "data": "synthetic",
        "config": {"workload": DESCR[a.config], "R": wl.R, "K": wl.K, "d": wl.d, "T": wl.T,
                   "loss": wl.loss, "nnz": wl.nnz, "rounds_per_call": wl.T},
        "kernels_ms": {"round_kernel": main_res["round_kernel_ms"], "meta_kernel": main_res["meta_kernel_ms"]},
        "roofline": {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit,
                     "frac": achieved / peak, "traffic": traffic, "kernel": "round kernel (S0-S2,S4)"},
    }
    # what rocprofv3 counted behind L2 for the round kernels of one step, as a rate, against the
    # nominal peak and against a plain device copy timed here
    if traffic:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        dst.copy_(src)
        ev0.record()
        for _ in range(3):
            dst.copy_(src)
        ev1.record()
        torch.cuda.synchronize()
        copy_gbs = 3 * 2 * src.numel() * 4 / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
        del src, dst
        torch.cuda.empty_cache()
        gbs = traffic / (main_res["round_kernel_ms"] * 1e-3) / 1e9
        line["hbm_counters"] = {"traffic_bytes_per_step": traffic, "rate_GBps": gbs, "frac_of_peak": gbs / PEAK_HBM_GBS,
                                "copy_ceiling_GBps": copy_gbs, "frac_of_copy_ceiling": gbs / copy_gbs,
                                "source": "profiles/hbm_traffic.json (rocprofv3 FETCH_SIZE + WRITE_SIZE)"}
    bpath = os.path.join(ROOT, "profiles", "binding_resource.json")
    if os.path.exists(bpath):
        line["binding_resource"] = json.load(open(bpath)).get(a.config)
    ab = keep["accel"]
    line["accel_bounds_k4_alpha0.05"] = {"gamma_lower_mean": float(ab[:, 2].mean()), "gamma_upper": float(ab[0, 3]),
                                         "note": "Theorem 1 from the regret of each run, mean over runs"}
    if wl.nnz:
        line["algorithmic_value"] = {"value": wl.R * wl.K * wl.T * wl.nnz / (main_res["ms_per_step"] * 1e-3),
                                     "unit": "touched learner-coordinates/s (R*K*T*nnz/s)"}

    if not a.no_cpu:
        cb, ref, runs, Tref = cpu_baseline(wl, keep["data"], WL)
        line["cpu_baseline"] = cb
        if Tref == wl.T:
            got = keep["regret"][runs]
            line["parity_regret_max_rel"] = float(np.max(np.abs(got - ref["regret"]) /
                                                         np.maximum(np.abs(ref["regret"]), 1.0)))
    keep.clear()

    if not a.no_others:
        others = {}
        for name in sorted(DESCR):
            if name == a.config:
                continue
            r = run_workload(name, 2, 1, WL, B, torch)
            others[name] = {"value": r["value"], "ms_per_step": r["ms_per_step"],
                            "round_kernel_ms": r["round_kernel_ms"], "meta_kernel_ms": r["meta_kernel_ms"]}
        for name in ("c3", "c4", "c5"):    # the optimistic two-step update (Eq. (3)) on the same streams
            r = run_workload(name, 2, 1, WL, B, torch, optimistic=True)
            others[name + "_optimistic"] = {"value": r["value"], "ms_per_step": r["ms_per_step"],
                                            "round_kernel_ms": r["round_kernel_ms"],
                                            "meta_kernel_ms": r["meta_kernel_ms"]}
        for name in ("v2", "v3"):          # verification step of Algorithm 1 on synthetic distributions
            others["specdec_" + name] = run_specdec(name, 5, WL, B, torch, with_cpu=not a.no_cpu)
        line["other_workloads"] = others

    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
