#!/usr/bin/env python3
"""Throughput of the local-update SGD hot path on one MI355X.

A "step" is one local iteration of all m replicas (mini-batch gather, forward,
softmax cross-entropy, backward with fused momentum update), with the replica
averaging every tau steps and, for the adaptive workloads, the loss evaluation
and AdaComm decision every `interval` steps -- i.e. the whole schedule driver
(lc_run) over K iterations.  Inputs are synthetic and resident in HBM before
the timed region starts.

The default workload is the largest configuration that has a model (cfg4: MLP
3072-2048-2048-2048-10, m = 64 replicas, batch 32, bf16 operands, AdaComm with
tau_0 = 10).  The K-step schedule is repeated until at least half a second has
been timed; the line reports the median repeat.

Prints ONE JSON line: replica-steps/s for the workload, the roofline figures of
the dominant kernel (measured with HIP events around each of its launches in
further passes over the same steps), the other workloads and the paper's
runtime model in `extra`, the averaging step at the two stress sizes, and the
oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_FP32_PEAK_TFLOPS = 157.3
MFMA_BF16_PEAK_TFLOPS = 2500.0

# (cfg3, cfg4: twice the configuration's loss-evaluation interval, so that the timed steps hold the
# evaluations and decisions of the schedule at their own spacing)
DEFAULT_STEPS = {"cfg1": 2000, "cfg2": 2000, "cfg3": 1000, "cfg4": 400, "cfg5a": 50, "cfg5b": 20}
DEFAULT_WARMUP = {"cfg1": 100, "cfg2": 100, "cfg3": 20, "cfg4": 10, "cfg5a": 5, "cfg5b": 3}
FLAT = {"cfg5a": (16, 25_600_000), "cfg5b": (8, 138_000_000)}
MIN_TIMED_S = 0.5          # the K-step schedule is repeated until this much has been timed
KERNEL_NAMES = {1: "backward_kernel", 2: "first_layer_kernel", 3: "sync_first_layer_kernel", 4: "head_kernel",
                5: "resident_kernel"}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="cfg4", choices=sorted(DEFAULT_STEPS))
    ap.add_argument("--tau", type=int, default=None, help="fixed communication period (overrides the workload's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the other workloads, the runtime model and the averaging-stress figures")
    ap.add_argument("--eager", action="store_true", help="write the average to every row at once (no deferred broadcast)")
    ap.add_argument("--layer-kernels", action="store_true",
                    help="launch-per-layer kernels also where the resident step kernel applies")
    ap.add_argument("--agent-scope-exchange", action="store_true",
                    help="resident kernel: exchange through device scope (see lc_set_xcd_local_exchange)")
    ap.add_argument("--no-deferred-update", action="store_true",
                    help="at tau = 1 write every replica's weights in the step (lc_set_deferred_update(0))")
    ap.add_argument("--fused-averaging", type=int, default=None, choices=[0, 1, 2],
                    help="lc_set_fused_averaging: 0 off, 1 first layer, 2 large hidden layers too (library default)")
    ap.add_argument("--no-implicit-momentum", action="store_true",
                    help="momentum rows read and written in every step (lc_set_implicit_momentum(0))")
    ap.add_argument("--no-first-layer-fusion", action="store_true",
                    help="separate first-layer forward launch in every step (see lc_set_first_layer_fusion)")
    return ap.parse_args()


def sync():
    import torch
    torch.cuda.synchronize()


def timed_repeats(fn, min_s=MIN_TIMED_S, min_repeats=3, max_repeats=200):
    """Calls fn() (which must leave its work queued or done) with a synchronise on both sides until
    min_s seconds have been timed; returns the list of durations."""
    out = []
    while len(out) < max_repeats and (len(out) < min_repeats or sum(out) < min_s):
        sync()
        t0 = time.perf_counter()
        fn()
        sync()
        out.append(time.perf_counter() - t0)
    return out


def read_pmc(workload, tag):
    """Counter-derived figures of one kernel of one workload, from the rocprofv3 --pmc summary kept
    under profiles/ (lines `@bench <tag> key=value ...`, written with the summary)."""
    path = os.path.join(ROOT, "profiles", f"pmc_traffic_mfma_{workload}.txt")
    if not os.path.exists(path):
        return None, None
    for line in open(path):
        if line.startswith("@bench ") and line.split()[1] == tag:
            kv = dict(f.split("=", 1) for f in line.split()[2:])
            return {k: float(v) for k, v in kv.items()}, os.path.relpath(path, ROOT)
    return None, os.path.relpath(path, ROOT)


def make_run(args, pkg, synth, name, cache):
    if name not in cache:
        cache[name] = synth.make_workload(name)
    w = cache[name]
    md = pkg.make_model(pkg.KIND_MLP, w.dims, B=w.B, N=w.N, E=w.E, lr=w.lr, beta=w.beta, wd=w.wd, bf16=w.bf16)
    run = pkg.LocalSGD(w.m, md, w.seed, w.x1, w.data, w.labels)
    run.set_lazy_broadcast(not args.eager)   # bit-identical results; see lc_set_lazy_broadcast
    run.set_resident(not args.layer_kernels)
    run.set_first_layer_fusion(not args.no_first_layer_fusion)
    run.set_deferred_update(not args.no_deferred_update)
    run.set_implicit_momentum(0 if args.no_implicit_momentum else 1)
    if args.fused_averaging is not None:
        run.set_fused_averaging(args.fused_averaging)
    run.set_xcd_local_exchange(not args.agent_scope_exchange)
    return w, run


def schedule_of(w, args, K):
    tau0 = args.tau if args.tau is not None else w.tau0
    adaptive = w.adaptive and args.tau is None
    interval = 0
    if adaptive:
        # the configuration's interval when the run is long enough to reach it twice, else one
        # that lets the K timed steps contain a loss evaluation and a decision
        interval = w.interval if K >= 2 * w.interval else max(tau0, K // 2)
    return tau0, adaptive, interval


def dominant_kernel(run, w, K2, tau0):
    """HIP events around every launch of the backward class, one pass per (layer, kernel): the
    (layer, kernel) that takes the most time, and all of them."""
    from paper_1810_08313_amd.binding import TIME_BWD, TIME_NONE
    L = len(w.dims) - 1
    found = []
    run.timing_begin(TIME_BWD)
    run.run(K2, tau0, adaptive=False)
    n_all, ms_all = run.timing_read()
    for layer in ([0] if run.resident_active() else range(1, L + 1)):
        for kernel in ([5] if layer == 0 else [1, 2, 3, 4]):
            run.timing_begin(TIME_BWD)
            run.timing_select(layer, kernel)
            run.run(K2, tau0, adaptive=False)
            n, ms = run.timing_read()
            if n:
                found.append({"layer": layer, "kernel": KERNEL_NAMES[kernel], "kernel_id": kernel, "launches": n,
                              "total_ms": ms, "avg_us": ms / n * 1e3})
    run.timing_begin(TIME_NONE)
    found.sort(key=lambda r: -r["total_ms"])
    return found, n_all, ms_all


def layer_bytes(w, rec, tau0, args, implicit_tau=0):
    """Algorithmic HBM bytes of one launch of a backward-class kernel on one layer: W and V of
    every replica read and written once (16 B per parameter); the tile-owner kernel of tau = 1
    reads and writes V only and the one averaged model once (8 m + 8 B per weight).
    implicit_tau > 0: the run keeps the momentum implicit inside periods of that length -- a step
    that is not the last of its period reads two consecutive models and writes one (12 B per
    parameter), the last one writes model and momentum (16 B).  The first-layer kernel runs only
    on steps that have a successor in their period (12 B); the row-owner kernel on layer 1 takes
    the others (priced at 16 B)."""
    l = rec["layer"]
    n = w.dims[l - 1] * w.dims[l] + w.dims[l]
    if rec["kernel_id"] == 3 and tau0 != 1:
        # last step of a longer period, the layer's averaging in the same launch: every replica's
        # weights and momentum (or older model) read, its momentum written, one averaged tile written
        return (12.0 * w.m + 4.0) * w.dims[l - 1] * w.dims[l]
    if rec["kernel_id"] == 3:
        return (8.0 * w.m + 8.0) * w.dims[l - 1] * w.dims[l]
    if tau0 == 1 and not args.eager:
        return ((8.0 if not args.no_deferred_update else 12.0) * w.m + 4.0) * n
    if implicit_tau > 1 and l < len(w.dims) - 1 and 4.0 * w.dims[l - 1] * w.dims[l] >= 2**20:
        if rec["kernel_id"] == 2:
            return 12.0 * w.m * n
        if rec["kernel_id"] == 1 and l > 1:
            return (12.0 * (implicit_tau - 1) + 16.0) / implicit_tau * w.m * n
    return 16.0 * w.m * n


def bench_mlp(args, pkg, synth, name, cache, headline=True):
    w, run = make_run(args, pkg, synth, name, cache)
    K = args.steps if (args.steps is not None and headline) else DEFAULT_STEPS[name]
    W = args.warmup if (args.warmup is not None and headline) else DEFAULT_WARMUP[name]
    tau0, adaptive, interval = schedule_of(w, args, K)
    resident = run.resident_active()

    if W > 0:
        run.run(W, tau0, adaptive=False)
    last = {}

    def one():
        last["sched"], last["rounds"] = run.run(K, tau0, adaptive=adaptive, interval=interval)

    times = timed_repeats(one)
    sec = statistics.median(times)
    out = dict(value=w.m * K / sec, sec=sec, K=K, W=W, repeats=len(times), timed_s=sum(times),
               dtype="bf16" if w.bf16 else "f32", workload=w, tau0=tau0, run=run)
    cfg = {"workload": f"{name}: MLP {'-'.join(map(str, w.dims))}, m={w.m}, B={w.B}, "
                       f"{'AdaComm tau0=' if adaptive else 'tau='}{tau0}"
                       f"{', interval=%d' % interval if adaptive else ''}, lr={w.lr}, momentum={w.beta}",
           "m": w.m, "P": w.P, "batch_per_replica": w.B, "tau0": tau0, "adaptive": adaptive,
           "averaging_rounds": last["rounds"], "tau_schedule": last["sched"][:16],
           "deferred_broadcast": not args.eager, "resident_step_kernel": resident,
           "first_layer_fusion": not args.no_first_layer_fusion,
           "deferred_update_at_tau_1": not args.no_deferred_update and not args.eager,
           "implicit_momentum_inside_periods": run.implicit_momentum_layers() > 0,
           "fused_averaging_mode": 2 if args.fused_averaging is None else args.fused_averaging}
    if name == "cfg3":
        cfg["note"] = ("at this configuration's own learning rate and momentum the averaged model stays near ln 10 "
                       "with periods of 20, so the rule keeps tau near tau0: an adapting tau is not exercised here")
    out["config"] = cfg
    if not headline:
        return out

    # roofline of the dominant kernel: further passes over K2 steps with HIP events around its launches
    K2 = min(K, 100)
    kernels, n_all, ms_all = dominant_kernel(run, w, K2, tau0)
    dom = kernels[0]
    if resident:
        # small model, weights on chip: the launch is priced against the matrix cores.  Algorithmic
        # flops of one replica-step: forward 2 B (d0 d1 + d1 d2), weight gradients the same again,
        # hidden-layer delta 2 B d1 d2 (copies that workgroups compute redundantly are not counted).
        if len(w.dims) == 3:
            d0, d1, d2 = w.dims
            flops_step = 2.0 * w.B * (2 * d0 * d1 + 3 * d1 * d2)
            workgroups = w.m * ((d1 + 63) // 64 * 64 // 16)
        else:   # softmax regression: forward and weight gradient only, one workgroup per replica
            d0, d1 = w.dims
            flops_step = 2.0 * w.B * 2 * d0 * d1
            workgroups = w.m
        per_launch = flops_step * w.m * K2 / dom["launches"]
        achieved = per_launch / (dom["avg_us"] * 1e-6) / 1e12
        peak = MFMA_BF16_PEAK_TFLOPS if w.bf16 else MFMA_FP32_PEAK_TFLOPS
        pmc, src = read_pmc(name, "resident") if (args.tau is None and not args.agent_scope_exchange) else (None, None)
        roof = {"bound": "mfma", "kernel": "%s (all layers of %d local steps per launch, weights in LDS%s)"
                % ("resident_kernel" if len(w.dims) == 3 else "resident1_kernel", round(K2 / dom["launches"]),
                   ", averaging steps inside" if K2 / dom["launches"] > tau0 else ""),
                "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                "traffic": pmc["traffic_bytes"] if pmc else None,
                "launches": dom["launches"], "avg_launch_us": round(dom["avg_us"], 2),
                "algorithmic_flops_per_launch": per_launch,
                "mfma_busy_pct": pmc["mfma_busy_pct"] if pmc else None, "counters_from": src,
                "workgroups": workgroups, "compute_units": 256}
    else:
        imp_tau = tau0 if cfg["implicit_momentum_inside_periods"] else 0
        tau_arg = tau0 if not adaptive else 0
        per_launch = layer_bytes(w, dom, tau_arg, args, imp_tau)
        achieved = per_launch / (dom["avg_us"] * 1e-6) / 1e9
        tag = f"layer{dom['layer']}:{dom['kernel']}"
        pmc, src = read_pmc(name if (args.tau is None) else f"{name}_tau{args.tau}", tag)
        what = {1: "dA + dW + momentum update of one layer, weights walked by row blocks",
                2: "dW + momentum update of layer 1 and the next step's first-layer forward",
                3: "dW, momentum update and the layer's averaging at tau = 1, weights owned by tile",
                4: "last layer: forward, softmax and backward"}[dom["kernel_id"]]
        roof = {"bound": "hbm", "kernel": f"{dom['kernel']} on layer {dom['layer']} "
                                          f"({w.dims[dom['layer'] - 1]}x{w.dims[dom['layer']]}; {what})",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": pmc["traffic_bytes"] if pmc else None,
                "launches": dom["launches"], "avg_launch_us": round(dom["avg_us"], 2),
                "algorithmic_bytes_per_launch": per_launch,
                "mfma_busy_pct": pmc["mfma_busy_pct"] if pmc else None, "counters_from": src}
        if imp_tau > 1:
            at16 = layer_bytes(w, dom, tau_arg, args) / (dom["avg_us"] * 1e-6) / 1e9
            roof["note"] = ("implicit momentum: a step that is not the last of its period reads two consecutive models and "
                            "writes one, 12 B per parameter, which is what `achieved` prices; against the 16 B per "
                            "parameter of a step that reads and writes W and V the same launch is `at_16_bytes_per_parameter`")
            roof["at_16_bytes_per_parameter"] = {"achieved": round(at16, 1), "frac": round(at16 / HBM_PEAK_GBS, 4)}
        # every kernel of the backward class, and the class as a whole
        roof["backward_class"] = {
            "launches": n_all, "avg_launch_us": round(ms_all / n_all * 1e3, 2),
            "GBps": round(sum(layer_bytes(w, r, tau_arg, args, imp_tau) * r["launches"] for r in kernels)
                          / (ms_all * 1e-3) / 1e9, 1),
            "kernels": [{"layer": r["layer"], "kernel": r["kernel"], "launches": r["launches"],
                         "avg_us": round(r["avg_us"], 2),
                         "GBps": round(layer_bytes(w, r, tau_arg, args, imp_tau) / (r["avg_us"] * 1e-6) / 1e9, 1)}
                        for r in kernels]}
    out["roofline"] = roof
    cfg["final_loss"] = round(run.loss(), 6)
    return out


def runtime_model(run, w, taus, K):
    """The paper's runtime model (Sec. 3.1, constant delays): an iteration takes Y + D / tau, so
    periods of tau are (1 + alpha) / (1 + alpha / tau) times faster than tau = 1, alpha = D / Y.
    Here Y = one local step of all replicas (lc_local_steps alone), D = one averaging step (HIP
    events around its kernels during a run at the first tau > 1), both measured; set against the
    measured ms per iteration at every tau."""
    from paper_1810_08313_amd.binding import TIME_AVG, TIME_NONE
    n = max(K, 2 * max(taus))
    run.run(n, max(taus), adaptive=False)
    Y = statistics.median(timed_repeats(lambda: run.local_steps(n), min_s=0.2)) / n
    run.average()
    tref = next((t for t in taus if t > 1), 1)
    run.timing_begin(TIME_AVG)
    run.run(n // tref * tref, tref, adaptive=False)
    launches, ms = run.timing_read()
    run.timing_begin(TIME_NONE)
    D = ms * 1e-3 / max(launches, 1)
    T = {}
    for tau in taus:
        k = n // tau * tau
        run.run(k, tau, adaptive=False)
        T[tau] = statistics.median(timed_repeats(lambda: run.run(k, tau, adaptive=False), min_s=0.2)) / k
    alpha = D / Y
    out = {"Y_ms": round(Y * 1e3, 5), "D_ms": round(D * 1e3, 5), "alpha": round(alpha, 4),
           "ms_per_iteration": {str(t): round(v * 1e3, 5) for t, v in T.items()}}
    if 1 in T:
        out["speedup_over_tau_1"] = {str(t): {"predicted": round((1 + alpha) / (1 + alpha / t), 3),
                                              "measured": round(T[1] / T[t], 3)} for t in taus if t != 1}
    return out


def flat_measure(pkg, m, P, K, W):
    import ctypes as C
    import torch
    from paper_1810_08313_amd.binding import TIME_AVG, TIME_UPD, TIME_UPDAVG, TIME_NONE
    L = pkg.lib()
    md = pkg.make_model(pkg.KIND_QUAD, [P], lr=0.05, beta=0.9)
    h = C.c_void_p()
    assert L.lc_init(m, P, C.byref(md), 0, C.byref(h)) == 0
    Ps = pkg.lc_row_stride(P)
    gen = torch.Generator(device="cuda:0").manual_seed(20181008)
    X = torch.zeros((m, Ps), device="cuda:0")
    X[:, :P] = torch.randn((m, P), generator=gen, device="cuda:0") * 0.1
    V = torch.zeros((m, Ps), device="cuda:0")
    G = torch.zeros((m, Ps), device="cuda:0")
    G[:, :P] = torch.randn((m, P), generator=gen, device="cuda:0") * 1e-3
    ws = int(L.lc_workspace_bytes(h))
    S = torch.empty(ws, dtype=torch.uint8, device="cuda:0")
    assert L.lc_attach(h, X.data_ptr(), V.data_ptr(), S.data_ptr(), ws, None, None,
                       torch.cuda.current_stream().cuda_stream) == 0
    assert L.lc_set_grad(h, G.data_ptr()) == 0

    def step():
        assert L.lc_update_from_grad(h) == 0
        assert L.lc_average(h) == 0

    for _ in range(W):
        step()
    sync()
    t0 = time.perf_counter()
    for _ in range(K):
        step()
    sync()
    sec = time.perf_counter() - t0

    out = {"sec": sec}
    n, ms = C.c_int64(0), C.c_double(0.0)
    for which, key, nbytes in ((TIME_AVG, "avg", 8.0 * m * P), (TIME_UPD, "upd", 20.0 * m * P)):
        L.lc_timing_begin(h, which)
        for _ in range(K):
            step()
        assert L.lc_timing_read(h, C.byref(n), C.byref(ms)) == 0
        out[key + "_gbs"] = nbytes / (ms.value / n.value * 1e-3) / 1e9
        out[key + "_us"] = ms.value / n.value * 1e3
        if key == "avg":
            out["launches"] = n.value
    L.lc_timing_begin(h, TIME_UPDAVG)
    for _ in range(K):
        assert L.lc_update_from_grad_and_average(h) == 0
    assert L.lc_timing_read(h, C.byref(n), C.byref(ms)) == 0
    out["fused_gbs"] = 20.0 * m * P / (ms.value / n.value * 1e-3) / 1e9
    out["fused_us"] = ms.value / n.value * 1e3
    L.lc_timing_begin(h, TIME_NONE)
    sync()
    L.lc_destroy(h)
    del X, V, G, S
    torch.cuda.empty_cache()
    return out


def bench_flat(args, pkg, name):
    """Averaging stress: {update from explicit gradients; average} per step."""
    m, P = FLAT[name]
    K = args.steps if args.steps is not None else DEFAULT_STEPS[name]
    W = args.warmup if args.warmup is not None else DEFAULT_WARMUP[name]
    res = flat_measure(pkg, m, P, K, W)
    pmc, src = read_pmc(name, "averaging")
    roof = {"bound": "hbm", "kernel": "averaging step (one launch sequence over all column chunks: reduce + broadcast)",
            "achieved": round(res["avg_gbs"], 1), "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": round(res["avg_gbs"] / HBM_PEAK_GBS, 4),
            "traffic": pmc["traffic_bytes"] if pmc else None, "counters_from": src,
            "launches": res["launches"], "avg_launch_us": round(res["avg_us"], 2),
            "algorithmic_bytes_per_launch": 8.0 * m * P}
    cfg = {"workload": f"{name}: flat fp32 vectors m={m}, P={P}, step = momentum-SGD update from explicit "
                       f"gradients + replica averaging", "m": m, "P": P,
           "update_GBps": round(res["upd_gbs"], 1), "fused_update_average_GBps": round(res["fused_gbs"], 1)}
    return dict(value=m * K / res["sec"], sec=res["sec"], K=K, W=W, repeats=1, timed_s=res["sec"], roofline=roof,
                config=cfg, dtype="f32", workload=None, tau0=1)


def cpu_baseline(res):
    """The oracle as it stands on the host cores, on a bounded sample of the same workload: local
    steps of as many replicas as there are host threads (workers do not interact inside a period),
    one step at a time until about 10 s have passed."""
    import oracle
    w = res["workload"]
    if w is None:
        return None
    cores = min(w.m, len(os.sched_getaffinity(0)))
    threads = oracle.set_threads(cores)
    md = oracle.make_model(oracle.KIND_MLP, w.dims, B=w.B, N=w.N, E=w.E, lr=w.lr, beta=w.beta, wd=w.wd, bf16=w.bf16)
    ref = oracle.Run(w.m, md, w.seed, w.x1, w.data, w.labels)
    ids = list(range(threads))
    t0 = time.perf_counter()
    steps = 0
    while True:
        ref.local_steps(1, ids=ids)
        steps += 1
        el = time.perf_counter() - t0
        if el > 10.0 or steps >= 2000:
            break
    oracle.set_threads(1)
    return {"value": round(len(ids) * steps / el, 2), "unit": "replica-steps/s", "cores": threads, "kind": "oracle",
            "sample": f"{steps} local steps of {len(ids)} of the {w.m} replicas ({el:.1f} s), one replica per host "
                      f"thread; the averaging step (under 3 % of the oracle's time) is not in the sample"}


def release(res):
    import torch
    run = res.pop("run", None)
    if run is not None:
        run.close()
        del run
    torch.cuda.empty_cache()


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (no collectives, no sharding); --gpus {args.gpus} is not "
              f"supported. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU path", file=sys.stderr)
        sys.exit(2)
    import paper_1810_08313_amd as pkg
    import synth
    pkg.lib()
    torch.cuda.set_device(0)
    cache = {}

    if args.workload in FLAT:
        res = bench_flat(args, pkg, args.workload)
    else:
        res = bench_mlp(args, pkg, synth, args.workload, cache)

    line = {
        "metric": "replica-steps/sec (all m replicas); averaging HBM GB/s as fraction of peak",
        "value": round(res["value"], 2),
        "unit": "replica-steps/s",
        "n_gpus": 1,
        "steps": res["K"],
        "warmup": res["W"],
        "ms_per_step": round(res["sec"] / res["K"] * 1e3, 5),
        "repeats": res["repeats"],
        "timed_region_s": round(res["timed_s"], 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": res["dtype"],
        "data": "synthetic",
        "config": res["config"],
        "roofline": res["roofline"],
    }
    if not args.no_extra and args.workload not in FLAT:
        extra = {}
        # the paper's runtime model against measurement, on the headline workload ...
        taus_model = {"cfg4": [1, 10], "cfg3": [1, 20], "cfg2": [1, 5, 20], "cfg1": [1, 4]}
        extra["runtime_model"] = {args.workload: runtime_model(res["run"], res["workload"], taus_model[args.workload],
                                                               res["K"])}
        release(res)
        # ... the other workloads (median of repeats that add up to half a second each), and the
        # headline workload at tau = 1
        others = {}
        saved = (args.steps, args.warmup, args.tau)
        for name in ("cfg1", "cfg2", "cfg3", "cfg4"):
            for tau in ([None] if name != args.workload else []) + ([1] if name in ("cfg3", "cfg4") else []):
                args.tau = tau
                r = bench_mlp(args, pkg, synth, name, cache, headline=False)
                key = name if tau is None else f"{name}_tau{tau}"
                others[key] = {"workload": r["config"]["workload"], "replica_steps_per_s": round(r["value"], 1),
                               "ms_per_step": round(r["sec"] / r["K"] * 1e3, 5), "steps": r["K"], "repeats": r["repeats"]}
                if name == "cfg2" and tau is None and args.workload != "cfg2":
                    extra["runtime_model"]["cfg2"] = runtime_model(r["run"], r["workload"], taus_model["cfg2"], r["K"])
                release(r)
            if name != "cfg4":
                cache.pop(name, None)
        args.steps, args.warmup, args.tau = saved
        extra["workloads"] = others
        line["extra"] = extra
        cache.clear()
        # the second half of the metric: averaging kernel at the stress sizes
        avg = {}
        for name, (m, P) in FLAT.items():
            r = flat_measure(pkg, m, P, DEFAULT_STEPS[name], DEFAULT_WARMUP[name])
            avg[name] = {"m": m, "P": P, "average_GBps": round(r["avg_gbs"], 1),
                         "average_frac_of_peak": round(r["avg_gbs"] / HBM_PEAK_GBS, 4),
                         "average_us": round(r["avg_us"], 1),
                         "update_GBps": round(r["upd_gbs"], 1),
                         "fused_update_average_GBps": round(r["fused_gbs"], 1)}
        line["averaging"] = avg
    else:
        release(res)
    line["cpu_baseline"] = None if args.no_cpu_baseline else cpu_baseline(res)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
