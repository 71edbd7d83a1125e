#!/usr/bin/env python3
"""Benchmark of the online-learner hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic workload already resident in
HBM: reset the state, run all T rounds of all R runs (round kernel + meta kernel), export
the final iterates / Hedge weights / combined iterate, and read back the regret.  The
metric is learner-updates per second, R*K*T*d / time.

Prints ONE JSON line.  `roofline` prices the dominant kernel (the kernel that works the rounds;
each of its launches timed with a pair of HIP events on the library's stream inside the timed
region) per launch against the resource that bounds it; `hbm` always says what fraction of the
HBM roofline the step's compulsory bytes amount to; `binding` names the resource that holds the
configuration back; `cpu_baseline` times the fp64 reference on the host cores on a bounded
sample.  Every entry of `other_workloads` carries the same three blocks.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_TFLOPS = 157.3     # MI355X fp32: vector (256 CUs x 2.4 GHz x 128 lanes x 2, packed) and matrix cores alike
NONPACKED_FP32_TFLOPS = 78.65  # what vector code reaches when every instruction works 64 lanes x 1 (this build: packed fp32 off)
PEAK_HBM_GBS = 8000.0
HBM_TARGET_FRAC = 0.60       # the fraction of the HBM roofline asked of the largest configuration

DESCR = {
    "c1": "c1: single projected OGD, linear loss, d=10 T=1000 K=1 R=1",
    "c2": "c2: K=15 OGD + Hedge, squared loss, d=100 T=10000 R=64, per-run streams",
    "c3": "c3: K=17 OGD + Hedge, squared loss, piecewise-stationary comparator, d=1000 T=100000 R=256",
    "c4": "c4: K=16 OGD + Hedge, logistic loss, shared stream, d=4096 T=20000 R=1024",
    "c5": "c5: K=8 OGD + Hedge, sparse squared loss (32 nnz/round), d=2^20 T=100000 R=16",
}
STAMPS = {}                  # profiles/*.json, read once


def profile_json(name):
    if name not in STAMPS:
        path = os.path.join(ROOT, "profiles", name)
        STAMPS[name] = json.load(open(path)) if os.path.exists(path) else {}
    return STAMPS[name]


def window_iterates_in_registers(wl, options):
    """Whether the windowed dense kernel keeps the iterates in registers for a whole launch: the
    launcher's rule (include/oco.h, OCO_OPT_WINDOW_RESIDENT), restated for the byte count."""
    ro = (options or {}).get("window_resident", -1)
    if ro == 1:
        return wl.d <= 4096 and not wl.optimistic
    if ro == 4:
        return wl.d <= 1024
    if ro >= 0:
        return False
    if wl.R * wl.K >= 16384 and wl.d >= 2048:        # four tiles per workgroup, loading wavefronts
        return False
    return (wl.d + 15) // 16 >= 32 and wl.d <= 1024


def algorithmic_hbm_bytes(wl, kernel, launches, in_registers=False):
    """Compulsory HBM bytes of the round kernels of one step.  Dense: the round stream once, the
    labels, the predictions out, the state in and out per launch; the windowed kernel also
    reads the two re-tiled copies of the stream that its pre-pass wrote and, unless it keeps
    them in registers, moves every iterate in and out once per window of 64 rounds.  Sparse: per
    touched learner coordinate 4 B read + 4 B written, the round stream (8 B per entry), labels
    and the comparator's gathers."""
    if wl.nnz:
        return float(wl.R * wl.K * wl.T * wl.nnz * 8 + wl.T * wl.nnz * 8 + wl.R * wl.T * 4 + wl.R * wl.T * wl.nnz * 4)
    x = 4.0 * wl.T * wl.d * (1 if wl.x_shared else wl.R)
    b = x + 4.0 * wl.R * wl.T + 4.0 * wl.R * (wl.K + 1) * wl.T + 8.0 * wl.R * wl.K * wl.d * max(launches, 1)
    if kernel.startswith("dense_window"):
        b += 4.0 * x
        if not in_registers:
            b += 8.0 * wl.R * wl.K * wl.d * ((wl.T + 63) // 64)
    return b


def roofline_block(wl, kt, config_key):
    """Roofline of the dominant kernel, per launch: algorithmic work of a launch / its average duration.

    Dense work per unit (one coordinate of one learner for one round): 5 + 2/K flops -- inner
    product 2, gradient step 2, projection scale 1, the comparator's inner product 2 per run.
    Executed: the projection is one scalar per learner (lazy scale), so the register kernel
    issues 4 + 2/K and the windowed kernel 4 (two contractions; the comparator's inner products
    run in a kernel of their own)."""
    launches = max(kt["launches"], 1)
    avg_ms = kt["ms_sum"] / max(kt["timed"], 1)
    kernel = kt["kernel"]
    hbm_bytes = algorithmic_hbm_bytes(wl, kernel, launches, kt.get("iterates") == "registers")
    entry = profile_json("hbm_traffic.json").get(config_key)
    entry = entry if isinstance(entry, dict) and entry.get("kernel") == kernel else None
    traffic = entry["bytes_per_launch"] if entry else None
    rl = {"kernel": kernel, "launches_per_step": launches, "avg_launch_ms": avg_ms}
    if kernel.startswith("dense_window"):
        rl["iterates"] = kt.get("iterates", "hbm")
    if wl.nnz:
        ach = hbm_bytes / launches / (avg_ms * 1e-3) / 1e9
        rl.update(bound="hbm", achieved=ach, peak=PEAK_HBM_GBS, unit="GB/s", frac=ach / PEAK_HBM_GBS)
    else:
        per_unit = 5.0 + 2.0 / wl.K
        executed = 4.0 if kernel.startswith("dense_window") else 4.0 + 2.0 / wl.K
        ach = per_unit * wl.units / launches / (avg_ms * 1e-3) / 1e12
        rl.update(bound="mfma" if kernel.startswith("dense_window") else "alu", achieved=ach, peak=PEAK_FP32_TFLOPS,
                  unit="TFLOP/s", frac=ach / PEAK_FP32_TFLOPS, flops_per_unit=per_unit,
                  executed_flops_per_unit=executed, executed_flops_frac=ach * executed / per_unit / PEAK_FP32_TFLOPS)
        if not kernel.startswith("dense_window"):
            rl["non_packed_ceiling"] = {"peak": NONPACKED_FP32_TFLOPS, "unit": "TFLOP/s",
                                        "executed_flops_frac": ach * executed / per_unit / NONPACKED_FP32_TFLOPS,
                                        "note": "vector fp32 with packed instructions off, as this build is compiled"}
    rl["traffic"] = traffic
    if entry and traffic is not None:
        rl["traffic_stamp"] = {"commit": entry.get("commit"), "plan": entry.get("plan"),
                               "source": "profiles/hbm_traffic.json (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a device copy)"}
        rl["traffic_over_algorithmic_bytes"] = traffic * launches / hbm_bytes
    gbs = hbm_bytes / launches / (avg_ms * 1e-3) / 1e9
    hbm = {"algorithmic_bytes_per_step": hbm_bytes, "GBps": gbs, "frac_of_peak": gbs / PEAK_HBM_GBS,
           "target_frac": HBM_TARGET_FRAC, "target_met": bool(gbs / PEAK_HBM_GBS >= HBM_TARGET_FRAC)}
    if traffic is not None:
        hbm["counter_GBps"] = traffic / (avg_ms * 1e-3) / 1e9
        hbm["counter_frac_of_peak"] = hbm["counter_GBps"] / PEAK_HBM_GBS
    return rl, hbm


def binding_block(wl, res, config_key, floor=None):
    """The resource that bounds the configuration, with its own utilisation."""
    us_round = res["round_kernel_ms"] * 1e3 / wl.T
    kernel = res["kernel_timing"]["kernel"]
    b = {"us_per_round": us_round}
    if floor is not None:
        b.update(resource="dependent chain of a round (latency): one wavefront reduction and the scalars behind it",
                 floor_us_per_round=floor["us_per_round"], floor=floor["what"],
                 over_floor=us_round / floor["us_per_round"])
    elif wl.nnz:
        b.update(profile_json("binding_resource.json").get(config_key) or {})
        b["us_per_round"] = us_round
    elif kernel.startswith("dense_window"):
        kt = res["kernel_timing"]
        step_ms = kt["ms_sum"] / max(kt["timed"], 1) * max(kt["launches"], 1)      # all launches of a step
        floor_ms = 4.0 * wl.units / (PEAK_FP32_TFLOPS * 1e12) * 1e3
        where = ("matrix cores, fed from L2 (round rows), the iterates in registers"
                 if kt.get("iterates") == "registers" else "matrix cores, fed from L2 (round rows) and HBM (iterates)")
        b.update(resource=where + "; the dependent rounds of a window "
                          "(64 rounds on float64 scalars, one wavefront per tile of 16 learners) run beside the sweep",
                 tiles=(wl.R * wl.K + 15) // 16, windows=(wl.T + 63) // 64,
                 matrix_core_floor_ms=floor_ms, utilisation=floor_ms / step_ms,
                 dependent_rounds_us_per_round=step_ms * 1e3 / wl.T)
    else:
        b.update(resource="vector ALU issue (fused multiply-adds of the inner product and the step)")
        b.update(profile_json("binding_resource.json").get(config_key.split(" ")[0]) or {})
    return b


def run_workload(name, steps, warmup, WL, B, torch, keep=None, optimistic=False, options=None, over=None):
    wl = WL.make(name, optimistic=optimistic, **(over or {}))
    data = WL.generate(wl)
    sim = B.Simulation(wl, data, options=options)
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
    kern_ms, ktim = [], []
    t0 = time.perf_counter()
    for _ in range(steps):
        reg = step()
        kern_ms.append(B.oco_last_timing(sim.h))
        ktim.append(B.oco_last_kernel_timing(sim.h))
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = 1e3 * dt / steps
    kt = dict(kernel=ktim[0]["kernel"], launches=ktim[0]["launches"], timed=sum(k["timed"] for k in ktim),
              ms_sum=sum(k["ms_sum"] for k in ktim))
    if kt["kernel"].startswith("dense_window"):
        kt["iterates"] = "registers" if window_iterates_in_registers(wl, options) else "hbm"
    out = dict(wl=wl, ms_per_step=ms, value=wl.units / (dt / steps),
               round_kernel_ms=float(sum(k[0] for k in kern_ms) / steps),
               meta_kernel_ms=float(sum(k[1] for k in kern_ms) / steps),
               kernel_timing=kt, regret_mean=float(reg.mean()))
    if keep is not None:
        keep.update(data=data, regret=reg, accel=sim.accel_bounds(4, 0.05))
    sim.close()
    del sim, W, p, wbar
    torch.cuda.empty_cache()
    return out


def empty_round_floor(name, WL, B, torch):
    """us per round of the same kernel on one learner of d = 4: a round is then only its
    dependent chain (inner product reduction, slope, step scalars) and the hand-over to the next."""
    r = run_workload(name, 2, 1, WL, B, torch, over=dict(d=4, K=1, R=1))
    return {"us_per_round": r["round_kernel_ms"] * 1e3 / r["wl"].T,
            "what": "same kernel, one learner of d=4, same T and loss (measured in this run)"}


def summary_entry(res, config_key, floor=None):
    wl = res["wl"]
    rl, hbm = roofline_block(wl, res["kernel_timing"], config_key)
    e = {"value": res["value"], "ms_per_step": res["ms_per_step"], "round_kernel_ms": res["round_kernel_ms"],
         "meta_kernel_ms": res["meta_kernel_ms"], "roofline": rl, "hbm": hbm,
         "binding": binding_block(wl, res, config_key, floor)}
    if wl.nnz:
        e["algorithmic_value"] = {"value": wl.R * wl.K * wl.T * wl.nnz / (res["ms_per_step"] * 1e-3),
                                  "unit": "touched learner-coordinates/s (R*K*T*nnz/s)"}
    return e


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
    for part in ("verify", "acceptance"):
        entry = profile_json("hbm_traffic.json").get(name + "_" + part)
        entry = entry if isinstance(entry, dict) else None
        out[part]["roofline"]["traffic"] = entry["bytes_per_launch"] if entry else None
        if entry:
            out[part]["roofline"]["traffic_stamp"] = {"commit": entry.get("commit"), "plan": entry.get("plan")}
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
    per_thread = {"c4": 4, "c3": 2}.get(wl.name, 1)          # sized for 10-30 s of CPU work
    runs = list(range(min(wl.R, cores * per_thread if wl.name != "c2" else wl.R)))
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
    floor = empty_round_floor(a.config, WL, B, torch) if a.config in ("c1", "c2") else None
    rl, hbm = roofline_block(wl, main_res["kernel_timing"], a.config)
    line = {
        "metric": "learner-updates/sec (runs x K x rounds x d / s)",
        "value": main_res["value"], "unit": "learner-updates/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 iterates, f64 losses/weights/regret", "data": "synthetic",
        "config": {"workload": DESCR[a.config], "R": wl.R, "K": wl.K, "d": wl.d, "T": wl.T,
                   "loss": wl.loss, "nnz": wl.nnz, "rounds_per_call": wl.T},
        "kernels_ms": {"round_kernel": main_res["round_kernel_ms"], "meta_kernel": main_res["meta_kernel_ms"]},
        "roofline": rl, "hbm": hbm, "binding": binding_block(wl, main_res, a.config, floor),
    }
    # a plain device copy timed here: what the HBM counters' rate can be held against besides the nominal peak
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    dst.copy_(src)
    ev0.record()
    for _ in range(3):
        dst.copy_(src)
    ev1.record()
    torch.cuda.synchronize()
    line["hbm"]["copy_ceiling_GBps"] = 3 * 2 * src.numel() * 4 / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    del src, dst
    torch.cuda.empty_cache()
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
            fl = empty_round_floor(name, WL, B, torch) if name in ("c1", "c2") else None
            others[name] = summary_entry(run_workload(name, 2, 1, WL, B, torch), name, fl)
        # the same workload on the other dense kernels (labelled: never the headline)
        if a.config == "c4":
            for label, opts in (("c4_register_kernel (one wavefront per learner, iterate in registers)", dict(dense_path=1)),
                                ("c4_window_kernel_iterates_in_registers", dict(dense_path=2, window_resident=1))):
                others[label] = summary_entry(run_workload("c4", 2, 1, WL, B, torch, options=opts), label)
        # c5 without the workgroups that fetch the rows of coming windows into L2 ahead of the working ones
        label = "c5_without_fetching_workgroups"
        others[label] = summary_entry(run_workload("c5", 2, 1, WL, B, torch, options=dict(sparse_fetch=0)), label)
        for name in ("c3", "c4", "c5"):    # the optimistic two-step update (Eq. (3)) on the same streams
            key = name + "_optimistic"
            others[key] = summary_entry(run_workload(name, 2, 1, WL, B, torch, optimistic=True), key)
        # optimism at both levels of the ensemble (the meta learner on cumulative plus last observed losses)
        others["c3_optimistic_both_levels"] = summary_entry(run_workload("c3", 2, 1, WL, B, torch, optimistic=2),
                                                            "c3_optimistic_both_levels")
        for name in ("v2", "v3"):          # verification step of Algorithm 1 on synthetic distributions
            others["specdec_" + name] = run_specdec(name, 5, WL, B, torch, with_cpu=not a.no_cpu)
        line["other_workloads"] = others

    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
