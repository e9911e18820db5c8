"""GPU parity of the local-training path (forward, backward, update) and of whole aggregation cycles against the
fp64 oracle, through the C-ABI.  fp32 tolerance: max-abs 1e-4 on parameters after the configured cycles."""
import numpy as np
import pytest

import oracle
from oracle import nets
from paper_2111_08274_amd import hadfl, synth
from tests import parity_metrics as pm
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
    # BN -> ReLU -> pool and BN -> pool (no ReLU): the pool is folded into the BN kernels; ragged chunks of windows
    b = nets._Builder(); b.dense(b.maxpool(b.bn(b.conv(b.maxpool(b.relu(b.bn(b.conv(0, 16, bias=False)))), 8, bias=False))), 5)
    c["bn_pool"] = (b.array(), (12, 8, 3), 6)
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
    # replica 0: 1 step, replica 1: 3 steps, replica 2: 2 steps.  First cycle step by step from a common state ...
    worst = p.forced_steps()
    d = p.max_param_diff()
    print(name, "m_total", net.m_total, "updates:", pm.show(worst), "max|dw|", d, flush=True)
    assert worst["max"] <= pm.UPDATE_REL_F32       # one or two layers, a few thousand units: element-wise, no twin needed
    assert d <= TOL, (name, d)
    losses = p.gpu.losses()
    assert np.abs(losses - p.cpu.loss).max() <= 1e-4
    agg_d = p.select_aggregate(0)
    assert agg_d <= TOL
    # ... second cycle as one free-running call
    w2 = p.local_steps(check_updates=True)
    print(name, "free-running updates:", pm.show(w2), flush=True)
    assert p.max_param_diff() <= TOL
    p.close()


def test_plain_sgd_without_momentum_is_the_papers_update():
    ops, shape, batch = CASES["conv_cin16"]
    x, y = _data(2, 24, shape, 5, seed=1)
    p = Pair(ops, shape, 2, 1, x, y, batch, 0.1, 0.0, [1, 2])
    p.forced_steps()
    assert p.max_param_diff() <= TOL
    p.local_steps(check_updates=True)
    assert p.max_param_diff() <= TOL
    with pytest.raises(hadfl.HadflError) as e:          # no momentum buffers without momentum
        p.gpu.momentum(0)
    assert e.value.status == hadfl.ESTATE
    p.close()


def _workload_pair(c, lr=None):
    cfg, x, y = synth.config_inputs(c)
    fn, shape = nets.NETS[cfg["net"]]
    p = Pair(fn(), shape, cfg["n_replicas"], cfg["n_select"], x, y, cfg["batch"], cfg["lr"] if lr is None else lr,
             cfg["momentum"], cfg["ratio"], net_name=cfg["net"])
    assert p.gpu.steps().tolist() == p.cpu.steps.tolist() == list(cfg["ratio"])
    return cfg, p


@pytest.mark.parametrize("c,lr", [(1, None), (2, 0.001)])
def test_workload_runs_all_cycles_within_tolerance(c, lr):
    """Free-running: all configured cycles, each side on its own, the fp32 bar after every cycle.  Workload 2 names no
    learning rate; at the paper's 0.01 the oracle itself amplifies one rounding past the bar within the 10 cycles
    (tests/test_oracle_sensitivity.py), so the free-running run uses 0.001 and the run at 0.01 is compared step by
    step below."""
    cfg, p = _workload_pair(c, lr)
    for cycle in range(cfg["cycles"]):
        w = p.local_steps(check_updates=True)
        d_local = p.max_param_diff()
        d_agg = p.select_aggregate(cycle)
        print("workload", c, "cycle", cycle, "max|dw| local", d_local, "agg", d_agg, "updates:", pm.show(w), flush=True)
        assert d_local <= TOL and d_agg <= TOL, (c, cycle)
    assert p.max_param_diff() <= TOL
    p.close()


@pytest.mark.parametrize("c", [1, 2])
def test_workload_every_step_of_every_cycle_from_a_common_state(c):
    """All configured cycles at the workload's learning rate (workload 2: the paper's 0.01), every sub-step compared
    with the oracle from a common state: each tensor's update to 1e-3 of its size, parameters to the fp32 bar."""
    cfg, p = _workload_pair(c)
    for cycle in range(cfg["cycles"]):
        w = p.forced_steps()
        d_local = p.max_param_diff()
        d_agg = p.select_aggregate(cycle)
        print("workload", c, "cycle", cycle, "forced updates:", pm.show(w), "max|dw|", d_local, "agg", d_agg, flush=True)
        assert d_local <= TOL and d_agg <= TOL, (c, cycle)
    p.close()


def test_cnn_workload_free_running_at_the_papers_learning_rate():
    """Workload 2 at lr 0.01, free-running, for the cycles in which the oracle's own sensitivity to one rounding is still
    an order of magnitude below the bar (2.6e-6 after three cycles)."""
    cfg, p = _workload_pair(2)
    assert cfg["lr"] == pytest.approx(0.01)
    for cycle in range(3):
        p.local_steps(check_updates=True)
        d_local = p.max_param_diff()
        d_agg = p.select_aggregate(cycle)
        print("workload 2 lr 0.01 cycle", cycle, "max|dw| local", d_local, "agg", d_agg, flush=True)
        assert d_local <= TOL and d_agg <= TOL
    p.close()


def _narrow_resnet():
    """ResNet-18's structure (stem, basic blocks with identity and projection shortcuts, BN everywhere, average
    pool, classifier) at widths 16/32/64 so that the fp64 oracle finishes in seconds."""
    b = nets._Builder()
    t = b.relu(b.bn(b.conv(0, 16, bias=False)))
    cin = 16
    for cout, stride in ((16, 1), (32, 2), (64, 2)):
        for blk in range(2):
            s = stride if blk == 0 else 1
            u = b.relu(b.bn(b.conv(t, cout, stride=s, bias=False)))
            u = b.bn(b.conv(u, cout, bias=False))
            sc = b.bn(b.conv(t, cout, k=1, stride=s, pad=0, bias=False)) if (s != 1 or cin != cout) else t
            t = b.relu(b.add(u, sc)); cin = cout
    b.dense(b.gap(t), 10)
    return b.array()


def test_resnet_structure_three_cycles():
    # lr 0.001.  Two effects make several-cycle parity at the workload's lr 0.1 meaningless for ANY fp32 code:
    # (1) the trajectory is chaotic there (the fp64 oracle against a copy of itself perturbed by one fp32 rounding
    # diverges past 1e-3 within four cycles, tests/test_oracle_sensitivity.py); (2) a ReLU unit whose pre-activation
    # lies within fp32 rounding of zero takes a different branch in fp32 than in fp64 -- both valid -- and moves the
    # weights by about lr * 1e-2 (measured: 9e-5 at lr 0.01, about one such unit per two cycles at this size).
    # So several cycles are compared where one such event stays below the bar ...
    ops, shape = _narrow_resnet(), (16, 16, 3)
    N, batch, n = 4, 16, 64
    x, y = synth.class_shift_images(N, n, shape, 10, seed=103, dirichlet=0.5)
    p = Pair(ops, shape, N, 2, x, y, batch, 0.001, 0.9, [1, 3, 2, 4])
    for cycle in range(3):
        p.local_steps(check_updates=True)
        d = p.max_param_diff()
        da = p.select_aggregate(cycle)
        print("narrow resnet cycle", cycle, "max|dw|", d, "agg", da, flush=True)
        assert d <= TOL and da <= TOL
    p.close()


def test_resnet_structure_every_step_at_the_workload_lr_from_a_common_state():
    # ... at the workload's lr 0.1, five cycles, every sub-step from a common state: what stays checkable when the
    # free-running trajectories are chaotic
    ops, shape = _narrow_resnet(), (16, 16, 3)
    N, batch, n = 4, 16, 64
    x, y = synth.class_shift_images(N, n, shape, 10, seed=103, dirichlet=0.5)
    p = Pair(ops, shape, N, 2, x, y, batch, 0.1, 0.9, [1, 3, 2, 4])
    for cycle in range(5):
        w = p.forced_steps()
        d = p.max_param_diff()
        da = p.select_aggregate(cycle)
        print("narrow resnet lr 0.1 forced cycle", cycle, "updates:", pm.show(w), "max|dw|", d, "agg", da, flush=True)
        assert d <= TOL and da <= TOL
    p.close()


def test_resnet_structure_first_step_at_the_workload_lr():
    # ... and at lr 0.1 the first step of every replica (nothing has been amplified yet) and its aggregate
    ops, shape = _narrow_resnet(), (16, 16, 3)
    N, batch, n = 4, 16, 64
    x, y = synth.class_shift_images(N, n, shape, 10, seed=103, dirichlet=0.5)
    p = Pair(ops, shape, N, 2, x, y, batch, 0.1, 0.9, [1, 1, 1, 1])
    p.local_steps(check_updates=True)
    d = p.max_param_diff()
    da = p.select_aggregate(0)
    print("narrow resnet lr 0.1 first step max|dw|", d, "agg", da, flush=True)
    assert d <= TOL and da <= TOL
    p.close()


def test_resnet18_full_width_against_oracle():
    """The real ResNet-18 layer shapes (11.2M parameters), two replicas, batch 8, one step each, compared with the
    oracle on every parameter.  lr 0.01: with 20M ReLU units per step one or two pre-activations fall within fp32
    rounding of zero, and at batch 8 one such unit moves its filter by about lr * 1e-3 (measured 1.2e-4 at lr 0.1)."""
    fn, shape = nets.NETS["resnet18"]
    N, batch, n = 2, 8, 16
    x, y = synth.class_shift_images(N, n, shape, 10, seed=103)
    p = Pair(fn(), shape, N, 1, x, y, batch, 0.01, 0.9, [1, 1], net_name="resnet18")
    p.local_steps(check_updates=True)
    d = p.max_param_diff()
    da = p.select_aggregate(0)
    print("resnet18 max|dw|", d, "agg", da, flush=True)
    assert d <= TOL and da <= TOL
    p.close()


@pytest.mark.parametrize("hint", [0, 1])
def test_lean_fp32_kernels_position_sorted_rows(hint):
    """fp32 configuration, layers with 64 / 128 channels on 8x8, 4x4 and 2x2 images at batch 32: forward and data gradient
    run in the lean fp32 kernels with rows ordered by pixel position and out-of-range taps skipped (hint 1: 256-row
    tiles); bias + ReLU, BN and pooling around them; the weight gradient stays in the generic kernel."""
    b = nets._Builder()
    t = b.relu(b.conv(0, 64))
    t = b.maxpool(b.relu(b.bn(b.conv(t, 64, bias=False))))
    t = b.maxpool(b.relu(b.conv(t, 128)))
    t = b.relu(b.conv(t, 128))
    b.dense(b.gap(t), 5)
    ops, shape, batch = b.array(), (8, 8, 3), 32
    N = 3
    x, y = _data(N, 2 * batch, shape, 5, seed=92)
    p = Pair(ops, shape, N, 2, x, y, batch, 0.01, 0.9, [2, 1, 1], options={hadfl.OPT_TILE_HINT: hint})
    w = p.forced_steps()
    d = p.max_param_diff()
    print("lean fp32 kernels max|dw|", d, "updates:", pm.show(w), "loss", p.gpu.losses(), p.cpu.loss, flush=True)
    assert d <= TOL
    assert np.abs(p.gpu.losses() - p.cpu.loss).max() <= 1e-4
    p.close()


@pytest.mark.parametrize("bf16,bias", [(False, 200.0), (True, 8.0)])
def test_batch_norm_statistics_from_a_convolution_with_a_large_bias(bf16, bias):
    """A convolution whose bias is large beside the spread of its outputs, followed by a batch norm that takes its
    statistics from that convolution's epilogue (64 channels: the lean kernels).  Sums of x and x^2 taken about zero
    would lose the variance to cancellation in fp32 (mean^2 / var = 4e4 here: an error of 1e-2 in the variance); the
    epilogue centres them on the bias.  (In the workloads a bias in front of a batch norm has zero gradient and
    stays where the initialisation put it.)"""
    b = nets._Builder()
    t = b.relu(b.conv(0, 64))
    t = b.relu(b.bn(b.conv(t, 64)))
    b.dense(b.gap(t), 5)
    ops, shape, batch = b.array(), (8, 8, 3), 32
    N = 2
    x, y = _data(N, 2 * batch, shape, 5, seed=93)
    p = Pair(ops, shape, N, 1, x, y, batch, 0.01, 0.9, [2, 1], bf16=bf16)
    second_bias = [(o, c) for o, c, k, _ in p.layout if k == "bias"][1]
    p.cpu.params[:, second_bias[0]:second_bias[0] + second_bias[1]] = bias
    w = p.forced_steps()
    print("large bias before BN, bf16 %d: updates %s" % (bf16, pm.show(w)), flush=True)
    assert w["compared"] > 0 and w["ill"] == 0
    p.close()
