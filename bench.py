#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input: the local
step of all M replicas (gather, forward, backward, batch gradient, test statistics, optimizer
update), the batch-size test and rule on the host, and, every H steps, the replica average.
Inputs (dataset, parameters, index batches) are resident in HBM before the timed region.

Default workload: the MLP 3072-2048-2048-2048-100 / GELU / heavy-ball / inner-product-test
configuration with M=16 replicas, timed in steady state at the batch cap b=8192 (the shapes
the matrix-core target is stated on).  `--workload` selects another configuration, `--adaptive`
times the run from b0 with the batch size growing under the test.

Prints ONE JSON line: throughput in samples/s (all replicas), the roofline record of the
dominant kernel (per-launch HIP-event timing collected inside the timed region), and the CPU
oracle's throughput on a bounded sample of the same workload.
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

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PROF_EVERY = 4                 # per-kernel events on every 4th timed step
COPY_GBS = 6700.0              # fastest plain copy measured on this machine (non-temporal, 16 B per thread)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=16)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="config3", choices=["config1", "config2", "config3", "config4", "config5"])
    ap.add_argument("--adaptive", action="store_true", help="start at b0 and let the test grow b")
    ap.add_argument("--batch", type=int, default=0, help="fixed local batch size (default: the cap)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="also run the library's plain copy kernel once on 2 x 1 GiB (the known-traffic "
                         "reference for scaling rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--cpu-sample-batch", type=int, default=0)
    ap.add_argument("--graphs", action="store_true",
                    help="replay captured HIP graphs on the steps that are not bracketed by events (fixed batch size)")
    ap.add_argument("--plain-update", action="store_true",
                    help="store the fp32 gradient and run the optimizer as a kernel of its own "
                         "(abs_set_fused_update(0)) instead of the library's default for bf16, the step inside the "
                         "weight-gradient epilogue")
    ap.add_argument("--fused-update", action="store_true", help="the default; accepted for older command lines")
    ap.add_argument("--gram-ip-max-batch", type=int, default=-1,
                    help="largest local batch whose inner products come from Gram matrices "
                         "(abs_set_gram_ip_max_batch; default: the library's, 256; 0: never)")
    ap.add_argument("--sustain-seconds", type=float, default=-1.0,
                    help="after the timed steps keep stepping for at least this long and report the step time of that "
                         "period as ms_per_step_sustained (the chip settles at its power limit within seconds; "
                         "default: 10 s for the default run, 0 with --batch / --adaptive / --no-cpu-baseline / other workloads)")
    ap.add_argument("--no-also", action="store_true", help="skip the reference measurement of config 2 (profiling runs)")
    ap.add_argument("--beyond", action="store_true",
                    help="time the entry points beyond the base path on config-3 / config-2 shapes instead: the "
                         "cross-worker estimator, ragged per-worker batch sizes, accumulated steps")
    return ap.parse_args()


def cpu_baseline(w, X, y, x0, sample_bs):
    """The oracle as it stands, timed on this machine's host cores: one local step of all M replicas (statistics,
    test and rule included) at each local batch size of sample_bs (the configuration's first size b0 and
    min(cap, 512)); `value` is the rate at the last (largest) one."""
    import numpy as np
    from oracle import abs_oracle as O
    from paper_2406_13936_amd import workloads as W
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    net = O.Net(w.dims, w.act, w.has_bias)
    runs = []
    for sb in sample_bs:
        orc = O.Replicas(net, x0, X, y, w.M, opt=w.opt, momentum=w.momentum, beta1=w.beta1, beta2=w.beta2,
                         eps=w.eps, weight_decay=w.weight_decay, mixed=(w.prec == W.PREC_BF16),
                         want_ip=(w.test != W.TEST_NORM))
        idx = W.step_indices(w, 0, 0, sb)
        t0 = time.perf_counter()
        orc.local_step(idx, w.lr)
        res = orc.test(w.test, eta=w.eta, theta=w.theta, nu=w.nu)
        O.next_batch_size([r["T"] for r in res], [sb] * w.M, w.b_cap, True)
        dt = time.perf_counter() - t0
        runs.append({"local_batch": sb, "seconds": dt, "samples_per_s": w.M * sb / dt})
    last = runs[-1]
    return {"value": last["samples_per_s"], "unit": "samples/s", "cores": int(threads), "kind": "oracle",
            "host_cpus": os.cpu_count(),
            "sample": "one local step of all M=%d replicas incl. statistics, test and rule at b=%s (%s s); value is the "
                      "rate at b=%d; fp64 numpy (its BLAS threads = cores), bf16 rounding points emulated"
                      % (w.M, "/".join(str(r["local_batch"]) for r in runs),
                         "/".join("%.1f" % r["seconds"] for r in runs), last["local_batch"]),
            "runs": runs}


def stats_stress(a, np, torch, A, W):
    """Statistics and averaging alone (no model run): M = 32 replicas of 4 stacked 4096x4096
    layers in bf16 at b = 8192; per-sample squared gradient norms, ||gbar||^2, <g_i, gbar> for every
    replica, then the 32-way average of the bf16 parameters (4.3 GB)."""
    from concurrent.futures import ThreadPoolExecutor
    M, L, b, d = 32, 4, a.batch or 8192, 4096
    dev = torch.device("cuda")
    a_list = [torch.empty((M, b, d), dtype=torch.bfloat16, device=dev) for _ in range(L)]
    d_list = [torch.empty((M, b, d), dtype=torch.bfloat16, device=dev) for _ in range(L)]

    def gen(ml):
        m, l = ml
        return ml, W.stats_stress_layer(0, m, l, b, d, d)

    with ThreadPoolExecutor(16) as ex:
        for (m, l), (av, dv) in ex.map(gen, [(m, l) for m in range(M) for l in range(L)]):
            a_list[l][m].copy_(torch.from_numpy(av).to(dev))
            d_list[l][m].copy_(torch.from_numpy(dv).to(dev))
    params = torch.empty((M, L * d * d), dtype=torch.bfloat16, device=dev)
    rng = np.random.default_rng(5)
    for m in range(M):
        params[m].copy_(torch.from_numpy(rng.standard_normal(L * d * d, dtype=np.float32) / 64).to(dev))
    torch.cuda.synchronize()
    for _ in range(max(1, a.warmup)):
        A.layer_stats(a_list, d_list)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        res, _, _, _ = A.layer_stats(a_list, d_list)
    torch.cuda.synchronize()
    dt_stats = (time.perf_counter() - t0) / a.steps
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    scratch = torch.empty(L * d * d, device=dev, dtype=torch.bfloat16)
    A.average_bf16(params, scratch)
    e0.record()
    for _ in range(a.steps):
        A.average_bf16(params, scratch)
    e1.record()
    torch.cuda.synchronize()
    ms_avg = e0.elapsed_time(e1) / a.steps
    avg_bytes = 2.0 * M * L * d * d * 2
    flops = 2.0 * 2 * M * L * b * d * d                 # weight-gradient + inner-product contractions
    return {
        "metric": "statistics-only samples/sec (all replicas) + replica-average GB/s",
        "value": M * b / dt_stats, "unit": "samples/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": dt_stats * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "cfg5_stats_stress", "M": M, "layers": L, "width": d, "local_batch": b},
        "roofline": {"bound": "hbm", "kernel": "average_bf16_reduce_kernel + average_bf16_spread_kernel", "achieved": avg_bytes / (ms_avg * 1e-3) / 1e9,
                     "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": avg_bytes / (ms_avg * 1e-3) / 1e9 / PEAK_HBM_GBS,
                     "traffic": None, "avg_launch_ms": ms_avg},
        "stats_gemm_tflops": flops / dt_stats / 1e12,
        "check": {"S1_replica0": res[0].sum_sq, "S2_replica0": res[0].gbar_sq},
    }


def measure(a, wname, np, torch, A, W, with_cpu):
    """Time a.steps steps of workload `wname` (inputs resident in HBM) and return the result line as a dict."""
    w = getattr(W, wname)()
    X, y = W.make_dataset(w)
    x0 = W.make_x0(w)
    if a.graphs:
        torch.cuda.set_stream(torch.cuda.Stream())     # stream capture needs a created stream (default priority)
    rep = A.Replicas.from_workload(w, X, y, x0)
    if a.plain_update and w.prec == W.PREC_BF16:
        rep.set_fused_update(False)
    if a.gram_ip_max_batch >= 0:
        rep.set_gram_ip_max_batch(a.gram_ip_max_batch)
    b_fixed = a.batch or w.b_cap

    def test_and_rule(b):
        # abs_norm_test / abs_inner_product_test, then abs_next_batch_size (max over the workers)
        if w.test == W.TEST_NORM:
            return rep.test_and_next_batch_size(b, w.b_cap, eta=w.eta)[0]
        return rep.test_and_next_batch_size(b, w.b_cap, theta=w.theta, nu=w.nu if w.test == W.TEST_AUG_IP else 0.0)[0]

    # pre-stage every index batch in HBM
    total = a.warmup + a.steps
    sizes, idx_dev = [], []
    if not a.adaptive:
        for s in range(total):
            k, h = divmod(s, w.H)
            t, b = rep.upload_indices(W.step_indices(w, k, h, b_fixed))
            idx_dev.append(t)
            sizes.append(b)
    else:
        # indices for the largest size, resident in HBM; row m of step s uses its first b entries per replica
        # (index j of a batch does not depend on b), cut out on the device
        for s in range(total):
            k, h = divmod(s, w.H)
            idx_dev.append(rep.upload_indices(W.step_indices(w, k, h, w.b_cap))[0])
    torch.cuda.synchronize()

    def run(s, b):
        if a.adaptive:
            t = idx_dev[s][:, :b].contiguous()
        else:
            t = idx_dev[s]
        if a.graphs:
            rep.local_step_graphed_dev(t, b, w.lr)
        else:
            rep.local_step_dev(t, b, w.lr)
        nb = test_and_rule(b)
        if (s + 1) % w.H == 0:
            rep.average_replicas()
        return nb

    if a.pmc_probe and with_cpu is not None:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        src.zero_()
        A.copy_probe(src, dst)
        torch.cuda.synchronize()
        del src, dst

    if a.adaptive:
        # one untimed run of the whole schedule first (every kernel variant and batch size on the growth path is
        # loaded), on a context of its own; the timed run starts again from x0
        b = w.b0
        for s in range(total):
            b = run(s, b)
        torch.cuda.synchronize()
        rep.close()
        rep = A.Replicas.from_workload(w, X, y, x0)
        if a.plain_update and w.prec == W.PREC_BF16:
            rep.set_fused_update(False)
        if a.gram_ip_max_batch >= 0:
            rep.set_gram_ip_max_batch(a.gram_ip_max_batch)
    b = w.b0 if a.adaptive else b_fixed
    for s in range(a.warmup):
        nb = run(s, b)
        b = nb if a.adaptive else b
    torch.cuda.synchronize()
    rep.profile_enable(True)
    samples = 0
    sched = []
    t0 = time.perf_counter()
    sampled = 0
    for s in range(a.warmup, total):
        samples += w.M * b
        sched.append(b)
        # per-kernel HIP events on every PROF_EVERY-th step of the timed region only: two events per launch cost
        # a few microseconds each, which would distort steps that take a few hundred
        on = (s - a.warmup) % PROF_EVERY == 0
        rep.profile_pause(not on)
        sampled += on
        nb = run(s, b)
        b = nb if a.adaptive else b
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = rep.profile_read()
    rep.profile_enable(False)
    scale = a.steps / max(sampled, 1)                  # sampled steps -> all timed steps (for the shares)
    # sustained rate: the same steps (staged index batches reused in turn) for at least sustain_s seconds
    sustained = None
    sustain_s = a.sustain_seconds
    if sustain_s < 0:
        sustain_s = 10.0 if (with_cpu and not a.adaptive and not a.batch and wname == "config3") else 0.0
    if sustain_s > 0 and not a.adaptive:
        n_s, t1 = 0, time.perf_counter()
        while True:
            for s in range(total):
                run(s, b)
            n_s += total
            torch.cuda.synchronize()
            if time.perf_counter() - t1 >= sustain_s:
                break
        dts = time.perf_counter() - t1
        sustained = {"ms_per_step_sustained": dts * 1e3 / n_s, "sustained_steps": n_s, "sustained_seconds": dts,
                     "value_sustained": w.M * b * n_s / dts}

    # dominant kernel = the matrix-core GEMM class with the largest total time
    gemms = {k: v for k, v in prof.items() if k.startswith("gemm_")}
    kernels = {}
    for k, v in prof.items():
        e = {"calls": v["calls"], "avg_ms": v["total_ms"] / v["calls"],
             "share": v["total_ms"] * scale / (dt * 1e3)}
        if v["flops"] > 0:
            e["tflops"] = v["flops"] / (v["total_ms"] * 1e-3) / 1e12
            e["frac_of_mfma_peak"] = e["tflops"] / PEAK_BF16_TFLOPS
        if v["bytes"] > 0:
            e["gbs"] = v["bytes"] / (v["total_ms"] * 1e-3) / 1e9
            e["frac_of_hbm_peak"] = e["gbs"] / PEAK_HBM_GBS
            e["frac_of_copy"] = e["gbs"] / COPY_GBS        # against the fastest plain copy measured here
        kernels[k] = e
    roof = None
    if prof and w.prec == W.PREC_BF16:       # (the fp32 configuration is launch- and latency-bound: no roof is meaningful)
        # Launch classes as a kernel trace sees them: one kernel symbol per (epilogue, tile shape) whatever the layer,
        # one per streaming kernel.  The dominant class is the one with the largest total time; its average launch
        # duration is what `rocprofv3 --kernel-trace --stats` reports for that symbol.  Which roof bounds it follows
        # from its algorithmic intensity: above the ridge of the machine (2.5 PFLOP/s over 8 TB/s = 312 flop/byte)
        # the matrix cores, below it (short batches: weight streaming and the per-parameter streams) HBM.
        classes = {}
        for k, v in prof.items():
            cname = k.rsplit("_L", 1)[0] if k.startswith("gemm_") else k
            ce = classes.setdefault(cname, {"total_ms": 0.0, "flops": 0.0, "bytes": 0.0, "calls": 0, "layers": []})
            ce["total_ms"] += v["total_ms"]; ce["flops"] += v["flops"]; ce["bytes"] += v["bytes"]
            ce["calls"] += v["calls"]; ce["layers"].append(k)
        name = max(classes, key=lambda k: classes[k]["total_ms"])
        v = classes[name]
        ridge = PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
        if w.prec == W.PREC_BF16 and v["flops"] > 0 and v["flops"] / max(v["bytes"], 1.0) >= ridge:
            ach = v["flops"] / (v["total_ms"] * 1e-3) / 1e12
            roof = {"bound": "mfma", "kernel": name, "achieved": ach, "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS, "traffic": None,
                    "avg_launch_ms": v["total_ms"] / v["calls"], "launches": v["calls"],
                    "flops_per_launch": v["flops"] / v["calls"], "layers": sorted(v["layers"])}
        elif v["bytes"] > 0:
            ach = v["bytes"] / (v["total_ms"] * 1e-3) / 1e9
            roof = {"bound": "hbm", "kernel": name, "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": ach / PEAK_HBM_GBS, "traffic": None, "avg_launch_ms": v["total_ms"] / v["calls"],
                    "launches": v["calls"], "bytes_per_launch": v["bytes"] / v["calls"],
                    "flops_per_byte": v["flops"] / v["bytes"], "layers": sorted(v["layers"])}
        if roof is not None:
            # HBM bytes per launch (mean over the class's layers) as read by rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
            # (scaled by the copy kernel) in the committed summary of this same command: a stored profile, not a
            # reading of this run; null when no summary covers the class
            tpath = os.path.join(ROOT, "profiles", "pmc_traffic_%s.json" % wname)
            if os.path.exists(tpath) and not a.adaptive and not a.batch and not a.plain_update:
                try:
                    tj = json.load(open(tpath)).get("kernels", {})
                    if all(k in tj for k in v["layers"]):
                        roof["traffic"] = sum(tj[k]["hbm_bytes_per_launch"] for k in v["layers"]) / len(v["layers"])
                        roof["traffic_source"] = "stored profile: profiles/" + os.path.basename(tpath)
                except Exception:
                    pass
        if gemms and w.prec == W.PREC_BF16 and roof is not None:
            allf = sum(v["flops"] for v in gemms.values())
            allt = sum(v["total_ms"] for v in gemms.values())
            roof["all_gemms_tflops"] = allf / (allt * 1e-3) / 1e12
            roof["all_gemms_frac"] = roof["all_gemms_tflops"] / PEAK_BF16_TFLOPS
    n_graphs = rep.graph_count()
    rep.close()
    if a.graphs:
        torch.cuda.set_stream(torch.cuda.default_stream())

    out = {
        "metric": "local-step samples/sec (all replicas, incl. batch test)",
        "value": samples / dt, "unit": "samples/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": dt * 1e3 / a.steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if w.prec == W.PREC_BF16 else "f32", "data": "synthetic",
        "config": {"workload": w.name, "dims": list(w.dims), "M": w.M, "H": w.H,
                   "local_batch": "adaptive from b0=%d" % w.b0 if a.adaptive else b_fixed,
                   "schedule": sched if a.adaptive else None,
                   "optimizer": ["sgd", "shb", "adamw", "adagrad"][w.opt],
                   "test": ["norm", "inner_product", "augmented_inner_product"][w.test]},
        "roofline": roof, "kernels": kernels,
    }
    if sustained:
        out.update(sustained)
    if w.prec == W.PREC_BF16:
        out["config"]["update"] = "separate kernel" if a.plain_update else "in the weight-gradient epilogue"
    if a.graphs:
        out["config"]["hip_graphs"] = n_graphs
    if with_cpu:
        # the configuration's first size and min(cap, 512) (config 2, cheap enough: its cap as well)
        sbs = [w.b0, min(w.b_cap, 512)] + ([w.b_cap] if wname == "config2" else [])
        if a.cpu_sample_batch:
            sbs = [min(a.cpu_sample_batch, w.b_cap)]
        out["cpu_baseline"] = cpu_baseline(w, X, y, x0, sorted(set(sbs)))
    return out


def beyond_base_path(np, torch, A, W):
    """Step times of the entry points beyond the base path (cross-worker estimator, ragged sizes, accumulation)
    on config-3 shapes at the cap and one accumulated case on config 2; inputs resident in HBM, test included."""
    def timeit(f, n):
        f()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            f()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    cases = []
    w = W.config3()
    X, y = W.make_dataset(w)
    rep = A.Replicas.from_workload(w, X, y, W.make_x0(w))
    b = w.b_cap
    t_idx, _ = rep.upload_indices(W.step_indices(w, 0, 0, b))
    dt = timeit(lambda: (rep.local_step_dev(t_idx, b, w.lr), rep.inner_product_test(w.theta)), 6)
    cases.append({"case": "config 3 uniform step, b = %d" % b, "ms": dt * 1e3, "samples_per_s": w.M * b / dt})
    dt = timeit(lambda: rep.cross_worker_test(0.5), 10)
    cases.append({"case": "cross-worker estimator on the gradients of the last step", "ms": dt * 1e3,
                  "gbs": w.M * rep.n_params * 4 / dt / 1e9})
    for name, bs in (("ragged: 8 workers at 8192, 8 at 4096", [8192] * 8 + [4096] * 8),
                     ("ragged: sizes spread from 1024 to 8192", [1024 + (8192 - 1024) * m // 15 for m in range(16)])):
        rows = [W.batch_indices(w.seed, 0, 0, m, bs[m], w.N) for m in range(w.M)]
        dt = timeit(lambda: (rep.local_step_ragged(rows, w.lr), rep.inner_product_test(w.theta)), 4)
        cases.append({"case": name, "ms": dt * 1e3, "samples_per_s": sum(bs) / dt,
                      "note": "indices uploaded from the host in every call"})
    idx2 = W.step_indices(w, 0, 1, 2 * b)
    dt = timeit(lambda: (rep.local_step_accumulated(idx2, b, w.lr), rep.inner_product_test(w.theta)), 3)
    cases.append({"case": "accumulated: b = %d in two micro-batches, inner-product statistics" % (2 * b), "ms": dt * 1e3,
                  "samples_per_s": w.M * 2 * b / dt, "note": "indices uploaded from the host in every call"})
    rep.close()
    w2 = W.config2()
    X, y = W.make_dataset(w2)
    rep = A.Replicas.from_workload(w2, X, y, W.make_x0(w2))
    idx2 = W.step_indices(w2, 0, 1, 4 * w2.b_cap)
    dt = timeit(lambda: (rep.local_step_accumulated(idx2, w2.b_cap, w2.lr), rep.norm_test(w2.eta)), 10)
    cases.append({"case": "config 2 accumulated: b = %d in four micro-batches, norm statistics" % (4 * w2.b_cap),
                  "ms": dt * 1e3, "samples_per_s": w2.M * 4 * w2.b_cap / dt,
                  "note": "indices uploaded from the host in every call"})
    rep.close()
    return {"metric": "step time of the entry points beyond the base path", "unit": "ms", "n_gpus": 1,
            "dtype": "bf16", "data": "synthetic", "config": {"workload": "cfg3 / cfg2 shapes at the cap"}, "cases": cases}


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build measures one GPU; all M worker replicas are batched on it and the "
              "replica average is an in-device mean (no collective). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import paper_2406_13936_amd as A
    from paper_2406_13936_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(3)
    if a.beyond:
        print(json.dumps(beyond_base_path(np, torch, A, W)))
        return
    if a.workload == "config5":
        print(json.dumps(stats_stress(a, np, torch, A, W)))
        return
    out = measure(a, a.workload, np, torch, A, W, not a.no_cpu_baseline)
    if a.workload == "config3" and not a.adaptive and not a.batch and not a.no_also:
        # the medium configuration (MLP 784-512-512-10, M = 8) at its cap, same contract, for reference
        o2 = measure(a, "config2", np, torch, A, W, False)
        out["also"] = {o2["config"]["workload"]: {
            "value": o2["value"], "unit": o2["unit"], "ms_per_step": o2["ms_per_step"],
            "local_batch": o2["config"]["local_batch"], "M": o2["config"]["M"],
            "all_gemms_tflops": (o2.get("roofline") or {}).get("all_gemms_tflops")}}
        # the same configuration in its short-batch regime (its first size, where the adaptive run stays): bound by
        # HBM; and both sizes with the optimizer as a kernel of its own (abs_set_fused_update(0))
        import copy
        for key, batch, plain in (("cfg3_b64", 64, False), ("cfg3_b64_plain_update", 64, True),
                                  ("cfg3_cap_plain_update", 0, True)):
            if plain and a.plain_update:
                continue
            a2 = copy.copy(a)
            a2.batch, a2.plain_update, a2.steps, a2.warmup = batch, plain or a.plain_update, 40 if batch else a.steps, 5
            o3 = measure(a2, "config3", np, torch, A, W, False)
            r3 = o3.get("roofline") or {}
            out["also"][key] = {"value": o3["value"], "unit": o3["unit"], "ms_per_step": o3["ms_per_step"],
                                "local_batch": o3["config"]["local_batch"],
                                "roofline": {k: r3.get(k) for k in ("bound", "kernel", "achieved", "peak", "unit", "frac")}}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
