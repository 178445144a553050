#!/usr/bin/env python3
"""Throughput of the local-update SGD hot path on one MI355X.

A "step" is one local iteration of all m replicas (mini-batch gather, forward,
softmax cross-entropy, backward with fused momentum update), with the replica
averaging every tau steps and, for the adaptive workloads, the loss evaluation
and AdaComm decision every `interval` steps -- i.e. the whole schedule driver
(lc_run) over K iterations.  Inputs are synthetic and resident in HBM before
the timed region starts.

Prints ONE JSON line: replica-steps/s for the workload, the roofline figures of
the dominant kernel (measured with HIP events around each of its launches in a
second pass over the same steps), and the oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_FP32_PEAK_TFLOPS = 157.3
MFMA_BF16_PEAK_TFLOPS = 2500.0

DEFAULT_STEPS = {"cfg1": 2000, "cfg2": 2000, "cfg3": 200, "cfg4": 40, "cfg5a": 50, "cfg5b": 20}
DEFAULT_WARMUP = {"cfg1": 100, "cfg2": 100, "cfg3": 20, "cfg4": 5, "cfg5a": 5, "cfg5b": 3}
FLAT = {"cfg5a": (16, 25_600_000), "cfg5b": (8, 138_000_000)}

# HBM bytes per launch of the dominant kernel and its MFMA busy share, from rocprofv3 --pmc runs of
# this script: FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 (calibration on the plain streaming update
# kernel) and SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE / 8 XCDs x 1024 SIMDs).  For the
# launch-per-layer path the dominant kernel is the backward kernel (figures averaged over the
# layers' launches of one iteration, the busy share weighted by launch duration); for the resident
# path it is the one kernel.  Summaries with the commands are in profiles/pmc_traffic_mfma_<workload>.txt.
PMC = {
    "cfg2": {"traffic": (28.115e6 + 2.389e6) / 2, "mfma_busy_pct": (8.19 * 8.6 + 1.21 * 8.9) / 17.5},
    # layer 1: first_layer_kernel where the next step's input is at hand (18 of 20 steps at tau=20,
    # 9 of 10 at tau=10; 16 steps are gathered per launch), backward_kernel otherwise
    "cfg3": {"traffic": ((0.9 * 841.605e6 + 0.1 * 822.536e6) + 288.527e6 + 15.974e6) / 3,
             "mfma_busy_pct": (0.9 * 7.58 * 199.0 + 0.1 * 3.20 * 162.0 + 4.88 * 64.3 + 1.17 * 9.7) /
                              (0.9 * 199.0 + 0.1 * 162.0 + 64.3 + 9.7)},
    "cfg4": {"traffic": ((0.9 * 6422.756e6 + 0.1 * 6466.302e6) + 2 * 4342.029e6 + 46.472e6) / 4,
             "mfma_busy_pct": (0.9 * 2.39 * 1278 + 0.1 * 0.86 * 1184 + 1.67 * 1669 + 1.21 * 28) /
                              (0.9 * 1278 + 0.1 * 1184 + 1669 + 28)},
}
# the same two workloads with --no-first-layer-fusion (backward_kernel for every layer)
PMC_UNFUSED = {
    "cfg3": {"traffic": (822.536e6 + 288.527e6 + 15.974e6) / 3,
             "mfma_busy_pct": (3.20 * 162.0 + 4.88 * 64.3 + 1.17 * 9.7) / 236.0},
    "cfg4": {"traffic": (6466.302e6 + 2 * 4342.029e6 + 46.472e6) / 4,
             "mfma_busy_pct": (0.86 * 1184 + 1.67 * 1669 + 1.21 * 28) / 2881},
}
PMC_RESIDENT = {
    "cfg1": {"traffic": 0.982e6, "mfma_busy_pct": 0.08},     # per launch of 32 local steps and 8 averaging steps
    "cfg2": {"traffic": 44.759e6, "mfma_busy_pct": 12.05},   # per launch of 5 local steps
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="cfg2", choices=sorted(DEFAULT_STEPS))
    ap.add_argument("--tau", type=int, default=None, help="fixed communication period (overrides the workload's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the averaging-stress figures")
    ap.add_argument("--eager", action="store_true", help="write the average to every row at once (no deferred broadcast)")
    ap.add_argument("--layer-kernels", action="store_true",
                    help="launch-per-layer kernels also where the resident step kernel applies")
    ap.add_argument("--agent-scope-exchange", action="store_true",
                    help="resident kernel: exchange through device scope (see lc_set_xcd_local_exchange)")
    ap.add_argument("--no-deferred-update", action="store_true",
                    help="at tau = 1 write every replica's weights in the step (lc_set_deferred_update(0))")
    ap.add_argument("--no-first-layer-fusion", action="store_true",
                    help="separate first-layer forward launch in every step (see lc_set_first_layer_fusion)")
    return ap.parse_args()


def sync():
    import torch
    torch.cuda.synchronize()


def bench_mlp(args, pkg, synth):
    import torch
    name = args.workload
    w = synth.make_workload(name)
    tau0 = args.tau if args.tau is not None else w.tau0
    adaptive = w.adaptive and args.tau is None
    K = args.steps if args.steps is not None else DEFAULT_STEPS[name]
    W = args.warmup if args.warmup is not None else DEFAULT_WARMUP[name]
    md = pkg.make_model(pkg.KIND_MLP, w.dims, B=w.B, N=w.N, E=w.E, lr=w.lr, beta=w.beta, wd=w.wd, bf16=w.bf16)
    run = pkg.LocalSGD(w.m, md, w.seed, w.x1, w.data, w.labels)
    run.set_lazy_broadcast(not args.eager)   # bit-identical results; see lc_set_lazy_broadcast
    run.set_resident(not args.layer_kernels)
    run.set_first_layer_fusion(not args.no_first_layer_fusion)
    run.set_deferred_update(not args.no_deferred_update)
    run.set_xcd_local_exchange(not args.agent_scope_exchange)
    resident = run.resident_active()
    interval = w.interval if adaptive else 0

    run.run(W, tau0, adaptive=False) if W > 0 else None
    sync()
    t0 = time.perf_counter()
    sched, rounds = run.run(K, tau0, adaptive=adaptive, interval=interval)
    sync()
    sec = time.perf_counter() - t0

    # second pass over the same number of steps with HIP events around every
    # launch of the dominant kernel (backward + fused update)
    from paper_1810_08313_amd.binding import TIME_BWD, TIME_NONE
    K2 = min(K, 200)
    run.timing_begin(TIME_BWD)
    run.run(K2, tau0, adaptive=False)
    launches, total_ms = run.timing_read()
    run.timing_begin(TIME_NONE)
    avg_launch_ms = total_ms / launches
    if resident:
        # small two-layer model, weights on chip: the launch is priced against the matrix cores.
        # Algorithmic flops of one replica-step: forward 2 B (d0 d1 + d1 d2), weight gradients the
        # same again, hidden-layer delta 2 B d1 d2 (copies that workgroups compute redundantly
        # are not counted).
        if len(w.dims) == 3:
            d0, d1, d2 = w.dims
            flops_step = 2.0 * w.B * (2 * d0 * d1 + 3 * d1 * d2)
            workgroups = w.m * ((d1 + 63) // 64 * 64 // 16)
        else:   # softmax regression: forward and weight gradient only, one workgroup per replica
            d0, d1 = w.dims
            flops_step = 2.0 * w.B * 2 * d0 * d1
            workgroups = w.m
        per_launch_flops = flops_step * w.m * K2 / launches
        achieved = per_launch_flops / (avg_launch_ms * 1e-3) / 1e12
        peak = MFMA_BF16_PEAK_TFLOPS if w.bf16 else MFMA_FP32_PEAK_TFLOPS
        roof = {"bound": "mfma", "kernel": "%s (all layers of %d local steps per launch, weights in LDS%s)"
                % ("resident_kernel" if len(w.dims) == 3 else "resident1_kernel", round(K2 / launches),
                   ", averaging steps inside" if K2 / launches > tau0 else ""),
                "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                "traffic": PMC_RESIDENT[name]["traffic"]
                if name in PMC_RESIDENT and args.tau is None and not args.agent_scope_exchange else None,
                "launches": launches, "avg_launch_us": round(avg_launch_ms * 1e3, 2),
                "algorithmic_flops_per_launch": per_launch_flops,
                "mfma_busy_pct": PMC_RESIDENT[name]["mfma_busy_pct"] if name in PMC_RESIDENT else None,
                "workgroups": workgroups, "compute_units": 256}
    else:
        bytes_per_iter = 16.0 * w.m * w.P                    # read W,V + write W,V of every replica, fp32
        if tau0 == 1 and not adaptive and not args.eager:
            # every iteration starts from the one averaged model (read once), and with the deferred
            # update the weights of the replicas are never written
            bytes_per_iter = (8.0 if not args.no_deferred_update else 12.0) * w.m * w.P + 4.0 * w.P
        per_launch_bytes = bytes_per_iter * K2 / launches
        achieved = per_launch_bytes / (avg_launch_ms * 1e-3) / 1e9
        pmc = (PMC_UNFUSED if args.no_first_layer_fusion and name in PMC_UNFUSED else PMC).get(name) \
            if args.tau is None else None
        roof = {"bound": "hbm", "kernel": "backward_kernel (dA + dW + momentum update, all layers; where "
                                          "first_layer_kernel serves layer 1 its launch also holds the next "
                                          "step's first-layer forward)",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": pmc["traffic"] if pmc else None,
                "launches": launches, "avg_launch_us": round(avg_launch_ms * 1e3, 2),
                "algorithmic_bytes_per_launch": per_launch_bytes,
                "mfma_busy_pct": round(pmc["mfma_busy_pct"], 2) if pmc else None}
    final_loss = run.loss()
    run.close()
    cfg = {"workload": f"{name}: MLP {'-'.join(map(str, w.dims))}, m={w.m}, B={w.B}, "
                       f"{'AdaComm tau0=' if adaptive else 'tau='}{tau0}"
                       f"{', interval=%d' % interval if adaptive else ''}, lr={w.lr}, momentum={w.beta}",
           "m": w.m, "P": w.P, "batch_per_replica": w.B, "tau0": tau0, "adaptive": adaptive,
           "averaging_rounds": rounds, "tau_schedule": sched[:16], "final_loss": round(final_loss, 6),
           "deferred_broadcast": not args.eager, "resident_step_kernel": resident,
           "first_layer_fusion": not args.no_first_layer_fusion,
           "deferred_update_at_tau_1": not args.no_deferred_update and not args.eager}
    return dict(value=w.m * K / sec, sec=sec, K=K, W=W, roofline=roof, config=cfg,
                dtype="bf16" if w.bf16 else "f32", workload=w, tau0=tau0)


def bench_flat(args, pkg, name):
    """Averaging stress: {update from explicit gradients; average} per step."""
    import ctypes as C
    import torch
    from paper_1810_08313_amd.binding import TIME_AVG, TIME_NONE
    m, P = FLAT[name]
    K = args.steps if args.steps is not None else DEFAULT_STEPS[name]
    W = args.warmup if args.warmup is not None else DEFAULT_WARMUP[name]
    res = flat_measure(pkg, m, P, K, W)
    roof = {"bound": "hbm", "kernel": "averaging step (reduce_chunk_kernel + broadcast_chunk_kernel over all chunks)", "achieved": round(res["avg_gbs"], 1), "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": round(res["avg_gbs"] / HBM_PEAK_GBS, 4), "traffic": None,
            "launches": res["launches"], "avg_launch_us": round(res["avg_us"], 2),
            "algorithmic_bytes_per_launch": 8.0 * m * P}
    cfg = {"workload": f"{name}: flat fp32 vectors m={m}, P={P}, step = momentum-SGD update from explicit "
                       f"gradients + replica averaging", "m": m, "P": P,
           "update_GBps": round(res["upd_gbs"], 1), "fused_update_average_GBps": round(res["fused_gbs"], 1)}
    return dict(value=m * K / res["sec"], sec=res["sec"], K=K, W=W, roofline=roof, config=cfg, dtype="f32",
                workload=None, tau0=1)


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


def cpu_baseline(res):
    """The oracle as it stands on the host cores, on a bounded sample of the
    same workload: whole periods (tau local steps + averaging) until about 10 s
    have passed."""
    import oracle
    w = res["workload"]
    if w is None:
        return None
    cores = min(w.m, len(os.sched_getaffinity(0)))
    threads = oracle.set_threads(cores)
    md = oracle.make_model(oracle.KIND_MLP, w.dims, B=w.B, N=w.N, E=w.E, lr=w.lr, beta=w.beta, wd=w.wd, bf16=w.bf16)
    ref = oracle.Run(w.m, md, w.seed, w.x1, w.data, w.labels)
    tau = max(1, min(res["tau0"], 5))
    t0 = time.perf_counter()
    steps = 0
    while True:
        ref.local_steps(tau)
        ref.average()
        steps += tau
        el = time.perf_counter() - t0
        if el > 10.0 or steps >= 2000:
            break
    oracle.set_threads(1)
    return {"value": round(w.m * steps / el, 2), "unit": "replica-steps/s", "cores": threads, "kind": "oracle",
            "sample": f"{steps} iterations of all {w.m} replicas in periods of {tau} local steps + averaging "
                      f"({el:.1f} s), OpenMP over replicas"}


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

    if args.workload in FLAT:
        res = bench_flat(args, pkg, args.workload)
    else:
        res = bench_mlp(args, pkg, synth)

    line = {
        "metric": "replica-steps/sec (all m replicas); averaging HBM GB/s as fraction of peak",
        "value": round(res["value"], 2),
        "unit": "replica-steps/s",
        "n_gpus": 1,
        "steps": res["K"],
        "warmup": res["W"],
        "ms_per_step": round(res["sec"] / res["K"] * 1e3, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": res["dtype"],
        "data": "synthetic",
        "config": res["config"],
        "roofline": res["roofline"],
    }
    if not args.no_extra and args.workload not in FLAT:
        # the second half of the metric: averaging kernel at the stress sizes
        extra = {}
        for name, (m, P) in FLAT.items():
            r = flat_measure(pkg, m, P, DEFAULT_STEPS[name], DEFAULT_WARMUP[name])
            extra[name] = {"m": m, "P": P, "average_GBps": round(r["avg_gbs"], 1),
                           "average_frac_of_peak": round(r["avg_gbs"] / HBM_PEAK_GBS, 4),
                           "average_us": round(r["avg_us"], 1),
                           "update_GBps": round(r["upd_gbs"], 1),
                           "fused_update_average_GBps": round(r["fused_gbs"], 1)}
        line["averaging"] = extra
    line["cpu_baseline"] = None if args.no_cpu_baseline else cpu_baseline(res)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
