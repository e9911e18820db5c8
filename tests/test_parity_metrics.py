"""The update-relative parity metric must be able to fail: mistakes planted in an oracle result (CPU only) -- a deep
layer's update dropped, doubled or sign-flipped -- pass the coarse whole-vector bars and are caught by the per-tensor
metric that the GPU parity tests assert."""
import numpy as np
import pytest

import oracle
from oracle import nets
from paper_2111_08274_amd import synth
from tests import parity_metrics as pm


def _small_vgg_like():
    b = nets._Builder()
    t = b.relu(b.bn(b.conv(0, 8)))
    t = b.maxpool(b.relu(b.bn(b.conv(t, 16))))
    t = b.relu(b.bn(b.conv(t, 16)))
    b.dense(t, 10)
    return b.array(), (8, 8, 3)


def _one_step(bf16):
    ops, shape = _small_vgg_like()
    net = oracle.Net(ops, shape, bf16=bf16)
    N, n, B = 1, 16, 16
    x, y = synth.class_shift_images(N, n, shape, 10, seed=5)
    w0 = synth.he_normal_init(net.layout())
    cyc = oracle.Cycle(net, N, 1, w0, x.reshape(N, n, -1), y, B, 0.01, 0.9, [1], seed=1)
    cyc.local_steps()
    return net.layout(), w0.astype(np.float64), cyc.params[0].copy(), net.m_train


@pytest.mark.parametrize("bf16", [False, True])
def test_planted_update_mistakes_pass_the_coarse_bars_and_fail_the_update_metric(bf16):
    layout, w0, w1, m_train = _one_step(bf16)
    bound = pm.UPDATE_REL_BF16 if bf16 else pm.UPDATE_REL_F32
    # the honest result, stored as the GPU stores it (fp32), passes
    assert pm.assert_updates_match(layout, w0, w1.astype(np.float32), w1, bound) < bound
    deep = [(o, c) for o, c, k, _ in layout if k == "weight"][2]          # third convolution's filters
    o, c = deep
    for name, factor in (("dropped", 0.0), ("doubled", 2.0), ("sign-flipped", -1.0)):
        bad = w1.copy()
        bad[o:o + c] = w0[o:o + c] + factor * (w1[o:o + c] - w0[o:o + c])
        # the bf16 workload's own bar (2e-2 of max|w| over the whole vector) does not see it ...
        if bf16:
            assert np.abs(bad - w1)[:m_train].max() / np.abs(w1[:m_train]).max() <= 2e-2, name
        # ... the per-tensor update metric does
        err, off, kind = pm.worst_update_error(layout, w0, bad, w1)
        assert off == o and kind == "weight" and err >= 0.999, (name, err)
        assert pm.worst_update_error(layout, w0, bad, w1, norm="l2")[0] >= 0.999
        with pytest.raises(AssertionError):
            pm.assert_updates_match(layout, w0, bad, w1, bound, name)


def test_a_tensor_with_no_update_of_its_own_is_measured_against_the_floor():
    # a convolution bias in front of a batch norm has an exactly zero gradient: rounding noise there must not fail the
    # metric, a real update of that size elsewhere must
    layout = [(0, 4, "weight", 4), (4, 4, "bias", 4)]
    w0 = np.zeros(8)
    ref = np.array([1e-3, -2e-3, 5e-4, 1e-3, 1e-19, 0, 0, 0])
    got = ref.copy(); got[4:] = [3e-10, -2e-10, 1e-10, 0]                   # fp32 noise where the oracle has ~0
    assert pm.worst_update_error(layout, w0, got, ref)[0] < 1e-3
    got2 = ref.copy(); got2[0] += 1e-5                                       # 0.5 % of the weight tensor's update
    assert pm.worst_update_error(layout, w0, got2, ref)[0] == pytest.approx(5e-3)


def test_the_twin_widens_the_bound_only_where_the_step_is_ill_conditioned():
    """Two tensors; the twin moves the first by 1 % (ill conditioned) and the second by 1e-6.  A library result that is
    5 % off on the first passes (10 x the twin), 20 % off fails; on the second tensor the fixed bounds apply; where the
    twin itself is 10 % off the allowance stops at the cap, which a dropped update still exceeds."""
    layout = [(0, 100, "weight", 10), (100, 100, "weight", 10)]
    rng = np.random.default_rng(4)
    w0 = np.zeros(200)
    ref = rng.standard_normal(200) * 1e-3
    twin = ref.copy(); twin[:100] *= 1.01; twin[100:] *= 1 + 1e-6
    ok = ref.copy(); ok[:100] *= 1.05
    r = pm.assert_updates_within_twin(layout, w0, ok, ref, w0, twin, pm.BOUNDS_F32)
    assert 0.4 < r["ratio"] < 0.6 and r["max"] == pytest.approx(0.05, rel=1e-3)
    bad = ref.copy(); bad[:100] *= 1.2
    with pytest.raises(AssertionError):
        pm.assert_updates_within_twin(layout, w0, bad, ref, w0, twin, pm.BOUNDS_F32)
    bad2 = ref.copy(); bad2[100:] *= 1.005                  # a systematic 5e-3: above the median bound of 1e-3
    with pytest.raises(AssertionError, match="median"):
        pm.assert_updates_within_twin(layout, w0, bad2, ref, w0, twin, pm.BOUNDS_F32)
    one = ref.copy(); one[150] += 0.02 * np.abs(ref[100:]).max()      # one element 2 % off: a branch event, tolerated
    pm.assert_updates_within_twin(layout, w0, one, ref, w0, twin, pm.BOUNDS_F32)
    twin2 = ref.copy(); twin2[:100] *= 1.10
    r = pm.assert_updates_within_twin(layout, w0, bad, ref, w0, twin2, pm.BOUNDS_F32)
    assert r["ill"] == 2 and r["compared"] == 4             # first tensor: Euclidean and element-wise not compared; second: all


def test_planted_mistakes_fail_the_three_measures():
    layout, w0, w1, _ = _one_step(True)
    o, c = [(o, c) for o, c, k, _ in layout if k == "weight"][2]
    twin = w0 + (w1 - w0) * (1 + 1e-4)
    for factor in (0.0, 2.0, -1.0):
        bad = w1.copy(); bad[o:o + c] = w0[o:o + c] + factor * (w1[o:o + c] - w0[o:o + c])
        with pytest.raises(AssertionError):
            pm.assert_updates_within_twin(layout, w0, bad, w1, w0, twin, pm.BOUNDS_BF16)
    pm.assert_updates_within_twin(layout, w0, w1.astype(np.float32), w1, w0, twin, pm.BOUNDS_BF16)
