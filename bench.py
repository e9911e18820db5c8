"""Benchmark of one HADFL aggregation cycle on one MI355X.

A step is one whole cycle -- every replica's local SGD steps, the probabilistic selection, the partial aggregate
and the global synchronisation -- over seeded synthetic inputs already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1|2|3|4|5] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E
MFMA_PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}
PAPER_CONTEXT = {"speedup_vs_decentralized_fedavg": 3.15, "speedup_vs_pytorch_distributed": 4.68,
                 "hardware": "4x V100, PCIe 3.0 x8, CIFAR-10, time-to-max-accuracy (Table 1, Sec. 4.2)"}
# HBM bytes per launch from rocprofv3 FETCH_SIZE / WRITE_SIZE (scaled by a plain copy of known size; see profiles/),
# valid only while the kernel's source files are unchanged: (kernel, workload) -> (source files, sha256 of their
# concatenation at measurement, bytes)
TRAFFIC = {
    ("aggregate", "agg-stress-n64"): (("paper_2111_08274_amd/csrc/aggregate.hip",),
                                      "6b6bc47f1584798896ab4395b0a3a8cedd8eec64ecd27d1eed8fa062f3c54da8",
                                      402287976.8),
    # all launches of the class in a cycle, averaged
    ("conv_dgrad", "vgg16-bf16-n32"): (("paper_2111_08274_amd/csrc/conv_bf16_fast.hip",
                                        "paper_2111_08274_amd/csrc/conv_stats.h"),
                                       "cc0afcd2862a6484e800f471bc016390d19f86eb04bffca742fcb93523bb020d",
                                       468965566.6),
    ("conv_fwd", "vgg16-bf16-n32"): (("paper_2111_08274_amd/csrc/conv_bf16_fast.hip",
                                      "paper_2111_08274_amd/csrc/conv_first_bf16.hip",
                                      "paper_2111_08274_amd/csrc/conv_stats.h"),
                                     "6d0b5b6f326de0b4d04d62e23f359ecac5d4aeece24567464504b1531826c890",
                                     324417802.8),
    # (the figure includes the fused update's parameter and momentum traffic)
    ("conv_wgrad", "vgg16-bf16-n32"): (("paper_2111_08274_amd/csrc/conv_bf16_fast.hip",
                                        "paper_2111_08274_amd/csrc/conv_first_bf16.hip"),
                                       "3a34545bbf20a11296692c6e63155e1cb74b497520169af88177b48f30ff7ecd",
                                       552115616.3),
}


def source_digest(files):
    import hashlib
    h = hashlib.sha256()
    for f in files:
        h.update(open(os.path.join(ROOT, f), "rb").read())
    return h.hexdigest()


def measured_traffic(kernel, workload):
    ent = TRAFFIC.get((kernel, workload))
    if not ent:
        return None
    try:
        digest = source_digest(ent[0])
    except OSError:
        return None
    return ent[2] if digest == ent[1] else None


GEMM_KERNELS = ("conv_fwd", "conv_dgrad", "conv_wgrad", "dense_fwd", "dense_dgrad", "dense_wgrad")


def build_training(c):
    import torch
    from paper_2111_08274_amd import hadfl, synth
    cfg, x, y = synth.config_inputs(c)
    hc = hadfl.make_config(cfg["n_replicas"], cfg["n_select"], net=cfg["net"], bf16=cfg["bf16"], batch=cfg["batch"],
                           n_samples=cfg["n_samples"], in_shape=cfg["in_shape"], lr=cfg["lr"],
                           momentum=cfg["momentum"], seed=synth.SELECT_SEED)
    w0 = synth.he_normal_init(hadfl.param_layout(hc), seed=0)
    ctx = hadfl.Context(hc, cfg["ratio"], w0=w0, x=torch.as_tensor(x), y=torch.as_tensor(y))
    return cfg, ctx, (w0, x, y)


def build_aggregation():
    import torch
    from paper_2111_08274_amd import hadfl, synth
    cfg = dict(synth.CONFIGS[4])
    N, m = cfg["n_replicas"], cfg["m"]
    hc = hadfl.make_config(N, cfg["n_select"], net="none", m_none=m, seed=synth.SELECT_SEED)
    _, _, stride = hadfl.param_count(hc)
    rep = torch.zeros(N * stride, dtype=torch.float32, device="cuda")
    g = torch.Generator(device="cuda"); g.manual_seed(404)
    rep.view(N, stride)[:, :m].normal_(0.0, cfg["std"], generator=g)
    versions = torch.as_tensor(synth.versions_uniform(N, *cfg["version_range"], seed=304)).cuda()
    ctx = hadfl.Context(hc, np.ones(N, dtype=np.int32), replicas=rep)
    return cfg, ctx, versions


def time_cycles(fn, steps, warmup):
    import torch
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        fn(warmup + i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def cpu_baseline_training(c, data, budget_s=20.0):
    """The oracle as it stands, timed on the same workload's inputs.  Workloads 1-2: whole cycles until about
    budget_s.  Workloads 3 and 5 (170 / 690 TFLOP of fp64 loops for the full run): a bounded sample -- ONE local step at
    the workload's own batch size on as many replicas as the oracle has threads (it parallelises over replicas only),
    i.e. that many replica-steps of the cycle's sum(E_k); the cycle figure is the extrapolation stated in `sample`."""
    import oracle
    from oracle import nets
    from paper_2111_08274_amd import synth
    cfg = dict(synth.CONFIGS[c])
    w0, x, y = data
    fn, shape = nets.NETS[cfg["net"]]
    net = oracle.Net(fn(), shape, bf16=bool(cfg["bf16"]))
    N = cfg["n_replicas"]
    threads = oracle.lib().hadfl_oracle_num_threads()
    if c in (3, 5):
        n_rep = min(threads, N)
        B = cfg["batch"]
        xs = np.ascontiguousarray(x[:n_rep, :B]).reshape(n_rep, B, -1)
        ys = np.ascontiguousarray(y[:n_rep, :B])
        cyc = oracle.Cycle(net, n_rep, 1, w0, xs, ys, B, cfg["lr"], cfg["momentum"], np.ones(n_rep, dtype=np.int32),
                           seed=synth.SELECT_SEED)
        t0 = time.perf_counter()
        cyc.local_steps()
        el = time.perf_counter() - t0
        ratio = synth.compute_ratios(N, *cfg["ratio_range"], seed=200 + c)
        steps_per_cycle = int(oracle.step_counts(ratio).sum())
        return {"value": n_rep * B / el, "unit": "samples/s", "cores": n_rep, "kind": "oracle",
                "sample": "one local step at the workload's batch %d on %d replicas of workload %d (%d of the cycle's %d "
                          "replica-steps) in %.1f s; a whole cycle at this rate: %.0f s"
                          % (B, n_rep, c, n_rep, steps_per_cycle, el, steps_per_cycle * el / n_rep)}
    ratio = cfg["ratio"]
    cyc = oracle.Cycle(net, N, cfg["n_select"], w0, x.reshape(N, x.shape[1], -1), y, cfg["batch"], cfg["lr"],
                       cfg["momentum"], ratio, seed=synth.SELECT_SEED)
    per_cycle = int(cfg["batch"] * cyc.steps.sum())
    done, t0 = 0, time.perf_counter()
    while True:
        cyc.run_cycle(done)
        done += 1
        el = time.perf_counter() - t0
        if el >= budget_s or done >= cfg["cycles"] or el * (done + 1) / done > 1.5 * budget_s:
            break
    return {"value": per_cycle * done / el, "unit": "samples/s", "cores": min(threads, N), "kind": "oracle",
            "sample": "%d whole cycle(s) of workload %d (%d samples each) in %.1f s" % (done, c, per_cycle, el)}


def cpu_baseline_aggregation(cfg, budget_s=15.0):
    import oracle
    from paper_2111_08274_amd import synth
    N, m, n_select = 8, cfg["m"], cfg["n_select"]      # only the selected rows are ever read: 8 rows suffice
    rows = synth.replica_rows_gaussian(N, m, cfg["std"], seed=404)
    a = np.full(N, 1.0 / n_select)
    done, t0 = 0, time.perf_counter()
    while True:
        oracle.aggregate_f32(rows, a)
        done += 1
        el = time.perf_counter() - t0
        if el >= budget_s or done >= 20:
            break
    gb = (n_select + 1) * 4.0 * m * done / 1e9
    return {"value": gb / el, "unit": "GB/s", "cores": oracle.lib().hadfl_oracle_num_threads(), "kind": "oracle",
            "sample": "%d aggregate(s) of 8 x %d fp32 rows in %.1f s" % (done, m, el)}


def measure_training(c, steps, warmup, overlap=True):
    """Times whole cycles of training workload c and, in a separate pass, every kernel class with HIP events on the
    stream it is launched on.  -> (result dict, data for the CPU baseline)."""
    from paper_2111_08274_amd import hadfl
    cfg, ctx, data = build_training(c)
    if not overlap:
        ctx.set_option(hadfl.OPT_SIDE_STREAM, 0)
    samples_per_cycle = int(cfg["batch"] * ctx.steps().sum())
    def cycle(i):
        ctx.local_steps()
        ctx.select(i)
        ctx.aggregate(resync=True)
    t_cycle = time_cycles(cycle, steps, warmup)
    t_local = time_cycles(lambda i: ctx.local_steps(), max(2, steps // 2), 1)
    ctx.profile(True)
    n_prof = max(2, min(steps, 10))
    for i in range(n_prof):
        cycle(10000 + i)
    prof = ctx.profile_read()
    ctx.profile(False)
    total_ms = sum(v["ms"] for v in prof.values())
    dom = max(prof, key=lambda n: prof[n]["ms"])
    kd = prof[dom]
    avg_ms = kd["ms"] / kd["launches"]
    dtype = "bf16" if cfg["bf16"] else "f32"
    if dom in GEMM_KERNELS:
        ach = kd["flops"] / kd["launches"] / (avg_ms * 1e-3) / 1e12
        roof = {"kernel": dom, "bound": "mfma", "achieved": ach, "peak": MFMA_PEAK_TFLOPS[dtype], "unit": "TFLOP/s",
                "frac": ach / MFMA_PEAK_TFLOPS[dtype], "traffic": measured_traffic(dom, cfg["name"])}
    else:
        ach = kd["bytes"] / kd["launches"] / (avg_ms * 1e-3) / 1e9
        roof = {"kernel": dom, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": ach / HBM_PEAK_GBS, "traffic": measured_traffic(dom, cfg["name"])}
    roof["avg_launch_ms"] = avg_ms
    roof["overlap"] = ("weight-gradient launches share the chip with the input-gradient and normalisation kernels of "
                       "the main stream; --no-overlap times each kernel alone") if overlap else "none"
    roof["share_of_kernel_time"] = kd["ms"] / total_ms
    gemm_flops = sum(v["flops"] for n, v in prof.items() if n in GEMM_KERNELS) / n_prof
    res = {"metric": "local-SGD samples/s over all replicas, whole aggregation cycles", "value": samples_per_cycle / t_cycle,
           "unit": "samples/s", "steps": steps, "warmup": warmup, "ms_per_step": t_cycle * 1e3, "dtype": dtype,
           "config": {"workload": cfg["name"], "net": cfg["net"], "n_replicas": cfg["n_replicas"],
                      "n_select": cfg["n_select"], "batch": cfg["batch"], "steps_per_replica": ctx.steps().tolist(),
                      "samples_per_cycle": samples_per_cycle},
           "roofline": roof,
           "local_steps": {"ms_per_cycle": t_local * 1e3, "samples/s": samples_per_cycle / t_local,
                           "algorithmic_TFLOP_per_cycle": gemm_flops / 1e12,
                           "mfma_utilisation": gemm_flops / t_local / 1e12 / MFMA_PEAK_TFLOPS[dtype]},
           "kernels": {n: {"launches_per_cycle": v["launches"] / n_prof, "ms_per_cycle": v["ms"] / n_prof}
                       for n, v in sorted(prof.items(), key=lambda kv: -kv[1]["ms"])}}
    ctx.close()
    return res, data


DEFAULT_STEPS = {1: (200, 20), 2: (100, 10), 3: (10, 2), 5: (10, 2)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", type=int, default=5, choices=[1, 2, 3, 4, 5],
                    help="5 (default): the largest training workload, where the utilisation targets apply")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true",
                    help="skip the short measurements of the other training workloads reported under `workloads`")
    ap.add_argument("--no-overlap", action="store_true",
                    help="launch the weight-gradient kernels on the caller's stream instead of the library's second "
                         "stream: per-kernel durations are then those of each kernel alone on the chip")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy 5 times (known traffic, to scale rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: every replica lives in one MI355X's HBM and no collective is built; "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2111_08274_amd import hadfl, synth
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    hadfl.lib()                      # fails loudly if the HIP library is not built
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    c = args.workload
    out = {"n_gpus": 1, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "data": "synthetic",
           "paper_context": PAPER_CONTEXT}

    # ---- aggregation on the 64 x 11.2M stress rows: always measured (the aggregation half of the metric) ----
    acfg, actx, versions = build_aggregation()
    a_steps = args.steps if (c == 4 and args.steps) else 200
    a_warm = args.warmup if (c == 4 and args.warmup is not None) else 20
    def agg_cycle(i):
        actx.select(i, versions=versions)
        actx.aggregate(resync=False)
    t_agg = time_cycles(agg_cycle, a_steps, a_warm)
    actx.profile(True)
    for i in range(50):
        agg_cycle(1000 + i)
    prof = actx.profile_read()
    actx.profile(False)
    k = prof["aggregate"]
    agg_ms = k["ms"] / k["launches"]
    agg_gbs = k["bytes"] / k["launches"] / (agg_ms * 1e-3) / 1e9
    cycle_gbs = (k["bytes"] / k["launches"]) / t_agg / 1e9
    aggregation = {"workload": acfg["name"], "ms_per_cycle": t_agg * 1e3, "kernel_ms": agg_ms,
                   "select_kernel_ms": prof["select"]["ms"] / prof["select"]["launches"],
                   "algorithmic_bytes": k["bytes"] / k["launches"], "GB/s": agg_gbs, "frac_of_hbm_peak": agg_gbs / HBM_PEAK_GBS,
                   "cycle_GB/s": cycle_gbs, "cycle_frac_of_hbm_peak": cycle_gbs / HBM_PEAK_GBS,
                   "mode": "no broadcast: (n_select+1)*4*M bytes; cycle = select + aggregate, timed end to end"}
    # the same rows with the global synchronisation fused into the aggregate's store (Algorithm 1: every replica's
    # parameters <- the aggregate): N more rows written per cycle.  Measured last: it makes the rows equal.
    def agg_cycle_bcast(i):
        actx.select(i, versions=versions)
        actx.aggregate(resync=True)
    t_b = time_cycles(agg_cycle_bcast, 40, 5)
    actx.profile(True)
    for i in range(20):
        agg_cycle_bcast(2000 + i)
    prof_b = actx.profile_read()
    actx.profile(False)
    kb = prof_b["aggregate_bcast"]
    b_ms = kb["ms"] / kb["launches"]
    b_bytes = kb["bytes"] / kb["launches"]
    aggregation["with_broadcast"] = {"ms_per_cycle": t_b * 1e3, "kernel_ms": b_ms, "algorithmic_bytes": b_bytes,
                                     "GB/s": b_bytes / (b_ms * 1e-3) / 1e9,
                                     "frac_of_hbm_peak": b_bytes / (b_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                     "cycle_GB/s": b_bytes / t_b / 1e9,
                                     "mode": "aggregate + global synchronisation in one kernel: (n_select+1+n_replicas)*4*M bytes"}
    if c == 4:
        out.update(metric="aggregation HBM GB/s over one select+aggregate cycle", value=cycle_gbs,
                   unit="GB/s", steps=a_steps, warmup=a_warm, ms_per_step=t_agg * 1e3, dtype="f32",
                   config={"workload": acfg["name"], "n_replicas": acfg["n_replicas"], "n_select": acfg["n_select"], "m": acfg["m"]})
        out["roofline"] = {"kernel": "aggregate", "bound": "hbm", "achieved": agg_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": agg_gbs / HBM_PEAK_GBS, "traffic": measured_traffic("aggregate", acfg["name"]),
                           "avg_launch_ms": agg_ms}
        out["aggregation"] = aggregation
        if not args.no_cpu_baseline:
            out["cpu_baseline"] = cpu_baseline_aggregation(acfg)
        actx.close()
        print(json.dumps(out))
        return
    actx.close()
    del actx, versions
    torch.cuda.empty_cache()

    # ---- the training workload: whole cycles ----
    steps = args.steps if args.steps else DEFAULT_STEPS[c][0]
    warmup = args.warmup if args.warmup is not None else DEFAULT_STEPS[c][1]
    res, data = measure_training(c, steps, warmup, overlap=not args.no_overlap)
    out.update(res)
    out["aggregation"] = aggregation
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_training(c, data)
    del data
    # ---- the other training workloads, shortly: every configuration has a measured line ----
    if not args.no_others:
        others = {}
        for oc in (1, 2, 3, 5):
            if oc == c:
                continue
            torch.cuda.empty_cache()
            k_steps, k_warm = {1: (50, 5), 2: (30, 5), 3: (5, 2), 5: (5, 2)}[oc]
            r, _ = measure_training(oc, k_steps, k_warm, overlap=not args.no_overlap)
            others[r["config"]["workload"]] = {"ms_per_cycle": r["ms_per_step"], "samples/s": r["value"], "dtype": r["dtype"],
                                               "steps": k_steps, "warmup": k_warm,
                                               "mfma_utilisation": r["local_steps"]["mfma_utilisation"],
                                               "roofline": r["roofline"]}
        out["workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
