"""Shape of the paper's Table 1 on synthetic data: simulated time for HADFL, decentralized FedAvg and synchronous SGD
to bring the training loss under a target, all three run through the same library calls (see modes.py).

    python -m paper_2111_08274_amd.table1_shape [--workload 2] [--target 1.0] [--max-cycles 400]

The clock is simulated (modes.cycle_time): the GPU executes the arithmetic of every device, the heterogeneity is the
ratio array.  The loss is the mean over devices of the last local step's mini-batch loss, smoothed over 5 cycles.
Output: one JSON line with the time, cycles and local steps each mode needed and HADFL's speedup over the other two
(the paper reports 3.15x and 4.68x on its own hardware and data; only the ordering is comparable).
"""
import argparse
import json

import numpy as np


def run(workload, target, max_cycles, local_steps, t_comm, lr=None):
    from . import hadfl, modes, synth
    cfg, x, y = synth.config_inputs(workload)
    out = {}
    for mode in modes.MODES:
        a = modes.mode_arguments(mode, cfg["ratio"], cfg["n_select"], local_steps=local_steps)
        hc = hadfl.make_config(cfg["n_replicas"], a["n_select"], net=cfg["net"], batch=cfg["batch"],
                               n_samples=cfg["n_samples"], in_shape=cfg["in_shape"], n_classes=10,
                               lr=cfg["lr"] if lr is None else lr,
                               momentum=cfg["momentum"], t_sync=a["t_sync"], seed=synth.SELECT_SEED, bf16=0)
        w0 = synth.he_normal_init(hadfl.param_layout(hc), seed=0)
        ctx = hadfl.Context(hc, a["ratio"], w0=w0, x=x, y=y)
        clock = modes.Clock(mode, cfg["ratio"], local_steps=local_steps, t_comm=t_comm)
        hist, reached = [], None
        for cycle in range(max_cycles):
            ctx.local_steps()
            ctx.select(cycle)
            ctx.aggregate(resync=True)
            clock.tick()
            hist.append(float(np.mean(ctx.losses())))
            if len(hist) >= 5 and np.mean(hist[-5:]) <= target:
                reached = cycle + 1
                break
        out[mode] = {"time": clock.t if reached else None, "cycles": reached, "local_steps": clock.steps,
                     "final_loss": float(np.mean(hist[-5:]))}
        ctx.close()
    times = {m: (v["time"] if v["time"] is not None else float("inf")) for m, v in out.items()}
    out["hadfl_speedup_over"] = modes.speedup_table(times)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", type=int, default=2)
    ap.add_argument("--target", type=float, default=1.0)
    ap.add_argument("--max-cycles", type=int, default=400)
    ap.add_argument("--local-steps", type=int, default=4, help="E of the FedAvg comparator")
    ap.add_argument("--t-comm", type=float, default=0.25,
                    help="one model exchange, in the clock's units (one local step of a device with ratio 1 = 1)")
    ap.add_argument("--lr", type=float, default=0.01, help="learning rate (the paper's 0.01 by default)")
    args = ap.parse_args()
    res = run(args.workload, args.target, args.max_cycles, args.local_steps, args.t_comm, args.lr)
    res["config"] = vars(args)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
