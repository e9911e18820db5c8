"""Runtime version forecast (paper Sec. 3.2) feeding real-valued versions into the selection (Sec. 3.1 step 2,
Sec. 3.3), with per-round step counts that differ from the plan: HIP path against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from oracle import nets
from paper_2111_08274_amd import hadfl, synth
from tests.pair import Pair

pytestmark = pytest.mark.gpu


def test_forecast_and_selection_follow_perturbed_step_counts():
    cfg, x, y = synth.config_inputs(1, n_samples=128)
    fn, shape = nets.NETS["mlp"]
    N = cfg["n_replicas"]
    p = Pair(fn(), shape, N, cfg["n_select"], x, y, cfg["batch"], cfg["lr"], 0.9, [2, 4, 6, 8], net_name="mlp")
    planned = p.cpu.steps.copy()
    assert planned.tolist() == [1, 2, 3, 4]
    rng = np.random.default_rng(17)
    alpha = 0.5
    pred = [oracle.Predictor(alpha) for _ in range(N)]
    for cycle in range(6):
        # a device may finish fewer steps than planned, one sits a round out now and then
        steps = np.maximum(planned - rng.integers(0, 3, size=N), 0).astype(np.int32)
        p.gpu.set_steps(steps)
        assert p.gpu.steps().tolist() == steps.tolist()
        p.gpu.local_steps()
        p.cpu.local_steps(steps=steps)
        v, _ = p.gpu.versions()
        assert v.tolist() == steps.tolist() == p.cpu.versions.tolist()
        p.gpu.predict_versions(alpha, horizon=1)
        want = np.array([pred[k].update(float(v[k]), 1) for k in range(N)])
        got = p.gpu.predicted()
        assert got.tolist() == want.tolist(), (cycle, got, want)            # bit for bit
        p.gpu.select_real(cycle)
        p.cpu.select(cycle, versions=want)
        sel, flag, w = p.gpu.selected()
        assert sel.tolist() == p.cpu.selected.tolist() and flag.tolist() == p.cpu.flag.tolist()
        p.gpu.aggregate(True)
        p.cpu.aggregate(True)
        d = p.max_param_diff()
        print("cycle", cycle, "steps", steps.tolist(), "forecast", got.tolist(), "selected", sel.tolist(), "diff", d, flush=True)
        assert d <= 1e-4
    p.close()


def test_selection_from_real_versions_is_bit_exact():
    N, n_select = 64, 8
    hc = hadfl.make_config(N, n_select, net="none", m_none=256, seed=synth.SELECT_SEED)
    _, _, stride = hadfl.param_count(hc)
    rep = torch.from_numpy(synth.replica_rows_gaussian(N, 256, 0.02, seed=5, row_stride=stride)).cuda()
    ctx = hadfl.Context(hc, np.ones(N, dtype=np.int32), replicas=rep)
    rng = np.random.default_rng(23)
    for cycle in range(200):
        v = rng.uniform(0.0, 12.0, size=N)
        if cycle % 3 == 0:
            v = np.round(v * 4) / 4                    # ties and exact quartiles as well
        avail = (rng.random(N) < 0.8).astype(np.uint8) if cycle % 5 == 4 else None
        if avail is not None and avail.sum() < n_select:
            avail[:n_select] = 1
        ctx.select_real(cycle, versions=torch.from_numpy(v).cuda(), avail=avail)
        sel, flag, w = ctx.selected()
        want_sel, want_flag, want_f, _ = oracle.select(v, n_select, synth.SELECT_SEED, cycle, avail)
        assert sel.tolist() == want_sel.tolist() and flag.tolist() == want_flag.tolist(), cycle
    ctx.close()


def test_error_paths_of_the_forecast_calls():
    N = 4
    hc = hadfl.make_config(N, 2, net="none", m_none=64)
    _, _, stride = hadfl.param_count(hc)
    ctx = hadfl.Context(hc, np.ones(N, dtype=np.int32), replicas=torch.zeros(N * stride, dtype=torch.float32, device="cuda"))
    with pytest.raises(hadfl.HadflError) as e:
        ctx.select_real(0)
    assert e.value.status == hadfl.STATUS_NAMES.index("HADFL_ESTATE")
    with pytest.raises(hadfl.HadflError):
        ctx.predicted()
    for bad in (0.0, 1.0, -0.5):
        with pytest.raises(hadfl.HadflError) as e:
            ctx.predict_versions(bad)
        assert e.value.status == hadfl.STATUS_NAMES.index("HADFL_EINVAL")
    with pytest.raises(hadfl.HadflError) as e:
        ctx.set_steps([1, -1, 2, 3])
    assert e.value.status == hadfl.STATUS_NAMES.index("HADFL_EINVAL")
    ctx.set_steps([0, 0, 5, 1])
    assert ctx.steps().tolist() == [0, 0, 5, 1]
    ctx.predict_versions(0.3, horizon=2, versions=torch.tensor([3, 1, 4, 1], dtype=torch.int32).cuda())
    assert ctx.predicted().tolist() == [3.0, 1.0, 4.0, 1.0]      # first observation: both states equal it, no trend
    ctx.close()


def test_warm_up_round_then_step_counts_from_its_times():
    """Mutual-negotiation phase of Sec. 3.2: every device trains the same few steps with a small learning rate and
    reports its time; the step counts of the following rounds come from those times (Sec. 3.3)."""
    cfg, x, y = synth.config_inputs(1, n_samples=128)
    fn, shape = nets.NETS["mlp"]
    N = cfg["n_replicas"]
    power = np.array([4, 2, 2, 1])                         # Fig. 1's heterogeneity
    p = Pair(fn(), shape, N, cfg["n_select"], x, y, cfg["batch"], cfg["lr"], 0.9, [1, 1, 1, 1], net_name="mlp")
    e_warmup, low_lr = 2, cfg["lr"] / 10
    p.gpu.set_lr(low_lr); p.cpu.lr = low_lr
    warm = np.full(N, e_warmup, dtype=np.int32)
    p.gpu.set_steps(warm)
    p.gpu.local_steps(); p.cpu.local_steps(steps=warm)
    assert p.max_param_diff() <= 1e-4
    # simulated clocks: time = steps / power, read with 1 % noise
    times = e_warmup / power * (1.0 + np.random.default_rng(3).uniform(-0.01, 0.01, size=N))
    steps = hadfl.steps_from_times(times, e_warmup, 0.25)
    assert steps.tolist() == oracle.steps_from_times(times, e_warmup, 0.25).tolist() == [4, 2, 2, 1]
    p.gpu.set_lr(cfg["lr"]); p.cpu.lr = cfg["lr"]
    p.gpu.set_steps(steps); p.cpu.steps = steps
    for cycle in range(2):
        p.local_steps()
        p.select_aggregate(cycle)
        assert p.max_param_diff() <= 1e-4
    v, c = p.gpu.versions()
    assert v.tolist() == [4, 2, 2, 1] and c.tolist() == [10, 6, 6, 4]       # 2 warm-up steps + 2 rounds
    p.close()
