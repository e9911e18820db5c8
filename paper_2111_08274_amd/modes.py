"""The paper's comparison systems as configurations of the same cycle, and a simulated clock.

Sec. 2.2 (local update and FedAvg aggregation equations) and Sec. 4 (Table 1) compare HADFL with decentralized FedAvg
and with synchronous data-parallel SGD.  On the replica-in-HBM path all three are the same four calls with different
step counts and selection sizes; nothing here computes anything, it only chooses arguments and keeps time.

  hadfl     every device trains for the same wall time: E_k = t_sync * r_k / gcd(r) local steps, N_p of N selected
  fedavg    every device takes the same number E of local steps and all N are averaged (FedAvg equations of Sec. 2.2)
  sync_sgd  one step each, all N averaged: averaging the models after one step from a common model is averaging the
            gradients (the distributed-SGD equation of Sec. 2.1), with or without momentum

Simulated clock (Sec. 2.3: the fast devices wait for the slow ones at every synchronisation).  A device with
computing-power ratio r_k needs 1 / r_k time units for a local step.  A cycle takes as long as its slowest member's
local work plus the exchange: max_k E_k / r_k + t_comm.  For hadfl that is t_sync / gcd(r) for every k (nobody waits);
for the two comparators it is E / min(r).  t_comm is the caller's estimate of one model exchange in the same units
(ring over the averaged devices, then the broadcast); the paper's communication volumes are in Sec. 3.3.
"""
import math

import numpy as np

MODES = ("hadfl", "fedavg", "sync_sgd")


def mode_arguments(mode, ratio, n_select, t_sync=1, local_steps=1):
    """-> dict(ratio=int32[N], n_select, t_sync) to build a context / oracle cycle for `mode`.

    ratio: the devices' computing-power ratios (larger = faster), used as they are by hadfl.
    local_steps: E of the fedavg comparator (local steps per device per round)."""
    ratio = np.asarray(ratio, dtype=np.int32)
    n = ratio.size
    if mode == "hadfl":
        return dict(ratio=ratio.copy(), n_select=int(n_select), t_sync=int(t_sync))
    if mode == "fedavg":
        return dict(ratio=np.ones(n, dtype=np.int32), n_select=n, t_sync=int(local_steps))
    if mode == "sync_sgd":
        return dict(ratio=np.ones(n, dtype=np.int32), n_select=n, t_sync=1)
    raise ValueError("mode must be one of %s" % (MODES,))


def steps_per_cycle(mode, ratio, t_sync=1, local_steps=1):
    """Local steps of every device in one cycle (the step-count rule of Sec. 3.3 for hadfl)."""
    ratio = np.asarray(ratio, dtype=np.int64)
    if mode == "hadfl":
        from . import hadfl                    # the rule itself lives in the library (hadfl_step_counts)
        return hadfl.step_counts(ratio, t_sync).astype(np.int64)
    if mode == "fedavg":
        return np.full(ratio.size, int(local_steps), dtype=np.int64)
    if mode == "sync_sgd":
        return np.ones(ratio.size, dtype=np.int64)
    raise ValueError("mode must be one of %s" % (MODES,))


def cycle_time(mode, ratio, t_sync=1, local_steps=1, t_comm=0.0):
    """Simulated duration of one cycle: the slowest member's local work plus one exchange."""
    ratio = np.asarray(ratio, dtype=np.float64)
    steps = steps_per_cycle(mode, ratio.astype(np.int64), t_sync, local_steps).astype(np.float64)
    return float(np.max(steps / ratio)) + float(t_comm)


def exchange_time(n_devices, model_bytes, bytes_per_unit_time):
    """One ring all-reduce over n_devices of a model of model_bytes (2 (n-1)/n of the model crosses each link)
    followed by nothing else: the broadcast to unselected devices overlaps with the next round's computation
    (Sec. 3.3).  n_devices = N_p for hadfl, N for the comparators."""
    if n_devices <= 1:
        return 0.0
    return 2.0 * (n_devices - 1) / n_devices * model_bytes / bytes_per_unit_time


class Clock:
    """Accumulates simulated time over cycles of one mode."""

    def __init__(self, mode, ratio, t_sync=1, local_steps=1, t_comm=0.0):
        self.dt = cycle_time(mode, ratio, t_sync, local_steps, t_comm)
        self.samples_steps = int(steps_per_cycle(mode, ratio, t_sync, local_steps).sum())
        self.t = 0.0
        self.steps = 0

    def tick(self):
        self.t += self.dt
        self.steps += self.samples_steps
        return self.t


def speedup_table(times):
    """times: dict mode -> simulated time to the target; -> dict of hadfl's speedup over the others (Table 1's last
    columns), nan where a run did not reach the target."""
    out = {}
    for m in ("fedavg", "sync_sgd"):
        a, b = times.get(m), times.get("hadfl")
        out[m] = (a / b) if (a is not None and b is not None and b > 0 and math.isfinite(a)) else float("nan")
    return out
