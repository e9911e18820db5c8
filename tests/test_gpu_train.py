"""GPU parity of the local-training path (forward, backward, update) and of whole aggregation cycles against the
fp64 oracle, through the C-ABI.  fp32 tolerance: max-abs 1e-4 on parameters after the configured cycles."""
import numpy as np
import pytest

import oracle
from oracle import nets
from paper_2111_08274_amd import hadfl, synth
from tests.pair import Pair

pytestmark = pytest.mark.gpu
TOL = 1e-4


def _data(N, n, shape, n_classes, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, n) + shape).astype(np.float32)
    y = rng.integers(0, n_classes, size=(N, n)).astype(np.int32)
    return x, y


def _layer_cases():
    c = {}
    b = nets._Builder(); b.dense(b.relu(b.dense(0, 20)), 7)                       # K = 37: ragged K and N
    c["dense_ragged"] = (b.array(), (1, 1, 37), 24)
    b = nets._Builder(); b.dense(b.relu(b.dense(0, 128)), 10)                     # K = 784 = 49 slabs
    c["dense_mlp_shape"] = (b.array(), (1, 1, 784), 32)
    b = nets._Builder(); b.dense(b.relu(b.conv(0, 8)), 5)                         # Cin = 3: scalar loader
    c["conv_cin3"] = (b.array(), (6, 6, 3), 8)
    b = nets._Builder(); b.dense(b.relu(b.conv(b.relu(b.conv(0, 16)), 32)), 5)    # Cin = 16: vector loaders + dgrad
    c["conv_cin16"] = (b.array(), (8, 8, 3), 8)
    b = nets._Builder(); b.dense(b.relu(b.conv(b.relu(b.conv(0, 16)), 32, stride=2)), 5)
    c["conv_stride2"] = (b.array(), (8, 8, 3), 6)
    b = nets._Builder(); b.dense(b.conv(b.relu(b.conv(0, 16)), 32, k=1, stride=2, pad=0, bias=False), 5)
    c["conv_1x1_s2"] = (b.array(), (8, 8, 3), 6)
    b = nets._Builder(); b.dense(b.maxpool(b.relu(b.conv(b.maxpool(b.relu(b.conv(0, 16))), 16))), 5)
    c["maxpool"] = (b.array(), (8, 12, 3), 6)
    b = nets._Builder(); b.dense(b.relu(b.bn(b.conv(0, 16, bias=False))), 5)
    c["bn"] = (b.array(), (8, 8, 3), 16)
    b = nets._Builder()
    t = b.relu(b.bn(b.conv(0, 16, bias=False)))
    u = b.bn(b.conv(b.relu(b.bn(b.conv(t, 16, bias=False))), 16, bias=False))
    b.dense(b.gap(b.relu(b.add(u, t))), 5)
    c["residual_identity"] = (b.array(), (8, 8, 3), 8)
    b = nets._Builder()
    t = b.relu(b.bn(b.conv(0, 16, bias=False)))
    u = b.bn(b.conv(b.relu(b.bn(b.conv(t, 32, stride=2, bias=False))), 32, bias=False))
    sc = b.bn(b.conv(t, 32, k=1, stride=2, pad=0, bias=False))
    b.dense(b.gap(b.relu(b.add(u, sc))), 5)
    c["residual_projection"] = (b.array(), (8, 8, 3), 8)
    b = nets._Builder(); b.dense(b.relu(b.conv(b.relu(b.conv(0, 160)), 144)), 5)  # several N tiles, ragged tiles
    c["conv_wide"] = (b.array(), (5, 7, 3), 5)
    return c


CASES = _layer_cases()


@pytest.mark.parametrize("name", sorted(CASES))
def test_layer_kinds_match_oracle_over_ragged_steps(name):
    ops, shape, batch = CASES[name]
    N, n = 3, batch * 3
    net = oracle.Net(ops, shape)
    x, y = _data(N, n, shape, net.n_out, seed=len(name))
    p = Pair(ops, shape, N, 2, x, y, batch, 0.05, 0.9, [1, 3, 2])
    print(name, "m_total", net.m_total, flush=True)
    p.local_steps()                       # replica 0: 1 step, replica 1: 3 steps, replica 2: 2 steps
    d = p.max_param_diff()
    assert d <= TOL, (name, d)
    losses = p.gpu.losses()
    assert np.abs(losses - p.cpu.loss).max() <= 1e-4
    agg_d = p.select_aggregate(0)
    assert agg_d <= TOL
    p.local_steps()
    assert p.max_param_diff() <= TOL
    p.close()


def test_plain_sgd_without_momentum_is_the_papers_update():
    ops, shape, batch = CASES["conv_cin16"]
    x, y = _data(2, 24, shape, 5, seed=1)
    p = Pair(ops, shape, 2, 1, x, y, batch, 0.1, 0.0, [1, 2])
    p.local_steps()
    assert p.max_param_diff() <= TOL
    p.close()


@pytest.mark.parametrize("c", [1, 2])
def test_workload_runs_all_cycles_within_tolerance(c):
    cfg, x, y = synth.config_inputs(c)
    fn, shape = nets.NETS[cfg["net"]]
    p = Pair(fn(), shape, cfg["n_replicas"], cfg["n_select"], x, y, cfg["batch"], cfg["lr"], cfg["momentum"],
             cfg["ratio"], net_name=cfg["net"])
    assert p.gpu.steps().tolist() == p.cpu.steps.tolist() == list(cfg["ratio"])
    worst = 0.0
    for cycle in range(cfg["cycles"]):
        p.local_steps()
        d_local = p.max_param_diff()
        d_agg = p.select_aggregate(cycle)
        worst = max(worst, d_local, d_agg)
        print("workload", c, "cycle", cycle, "max|dw| local", d_local, "agg", d_agg, flush=True)
        assert d_local <= TOL and d_agg <= TOL, (c, cycle)
    assert p.max_param_diff() <= TOL
    p.close()
