"""Pins for the oracle's partial aggregation and the whole cycle (paper Sec. 2.2-2.3, Algorithm 1)."""
import numpy as np

import oracle
from oracle import nets


def test_identical_replicas_return_that_replica():
    rng = np.random.default_rng(0)
    w = rng.standard_normal(1000)
    P = np.tile(w, (6, 1))
    for flag in ([1, 0, 0, 0, 0, 0], [1, 1, 0, 0, 0, 0], [0, 1, 0, 1, 1, 1]):
        a = oracle.aggregation_weights(np.array(flag))
        agg = oracle.aggregate(P, a)
        assert np.abs(agg - w).max() <= 4 * np.finfo(np.float64).eps * np.abs(w).max()
    assert np.array_equal(oracle.aggregate(P, oracle.aggregation_weights(np.array([0, 0, 1, 0, 0, 0]))), w)


def test_all_selected_is_fedavg_mean_and_sum_is_linear():
    rng = np.random.default_rng(1)
    P = rng.standard_normal((5, 777))
    a = oracle.aggregation_weights(np.ones(5))
    assert np.allclose(oracle.aggregate(P, a), P.mean(axis=0), rtol=0, atol=1e-15)
    flag = np.array([1, 0, 1, 1, 0])
    a = oracle.aggregation_weights(flag)
    agg = oracle.aggregate(P, a)
    assert np.allclose(agg, P[[0, 2, 3]].mean(axis=0), atol=1e-15)
    assert np.allclose(oracle.aggregate(3.0 * P, a), 3.0 * agg, atol=1e-14)
    # unselected rows do not matter
    Q = P.copy(); Q[[1, 4]] = 1e9
    assert np.array_equal(oracle.aggregate(Q, a), agg)
    # fp32-stored rows: same sums
    P32 = P.astype(np.float32)
    assert np.allclose(oracle.aggregate_f32(P32, a), P32.astype(np.float64)[[0, 2, 3]].mean(axis=0), atol=1e-15)


def _toy(N, ratio, n_select, mom=0.0, seed=0):
    b = nets._Builder(); b.dense(b.relu(b.dense(0, 6)), 3)
    net = oracle.Net(b.array(), (1, 1, 5))
    rng = np.random.default_rng(seed)
    w0 = rng.standard_normal(net.m_total) * 0.4
    x = rng.standard_normal((N, 16, 5)).astype(np.float32)
    y = rng.integers(0, 3, size=(N, 16)).astype(np.int32)
    return net, w0, x, y, oracle.Cycle(net, N, n_select, w0, x, y, 4, 0.1, mom, ratio, seed=3)


def test_one_replica_cycle_is_plain_sgd():
    net, w0, x, y, _ = _toy(1, [1], 1)
    cyc = oracle.Cycle(net, 1, 1, w0, x, y, 4, 0.1, 0.0, [1], seed=3, t_sync=3)
    assert cyc.steps.tolist() == [3]
    cyc.run_cycle(0); cyc.run_cycle(1)
    ref = oracle.Cycle(net, 1, 1, w0, x, y, 4, 0.1, 0.0, [1], seed=3, t_sync=6)
    ref.local_steps()
    assert np.abs(cyc.params[0] - ref.params[0]).max() < 1e-15


def test_equal_ratios_all_selected_is_fedavg():
    # Sec. 2.2: E equal local steps on every device, then the plain mean over all K devices
    net, w0, x, y, cyc = _toy(4, [2, 2, 2, 2], 4)
    assert cyc.steps.tolist() == [1, 1, 1, 1]
    agg = cyc.run_cycle(0)
    singles = []
    for k in range(4):
        one = oracle.Cycle(net, 1, 1, w0, x[k:k + 1], y[k:k + 1], 4, 0.1, 0.0, [1], seed=3)
        one.local_steps(); singles.append(one.params[0].copy())
    assert np.abs(agg - np.mean(singles, axis=0)).max() < 1e-15
    assert all(np.array_equal(cyc.params[k], agg) for k in range(4))      # global synchronisation


def test_cycle_bookkeeping_and_momentum_survive_synchronisation():
    net, w0, x, y, cyc = _toy(4, [1, 2, 3, 4], 2, mom=0.9)
    cyc.run_cycle(0)
    assert cyc.versions.tolist() == [1, 2, 3, 4] and cyc.cursor.tolist() == [1, 2, 3, 4]
    assert cyc.flag.sum() == 2 and abs(cyc.weights.sum() - 1) < 1e-15
    buf_before = cyc.buf.copy()
    assert np.abs(buf_before).max() > 0           # optimiser state is local: not aggregated, not reset
    cyc.select(1); cyc.aggregate(resync=True)
    assert np.array_equal(cyc.buf, buf_before)
    cyc.run_cycle(2)
    assert cyc.versions.tolist() == [1, 2, 3, 4] and cyc.cursor.tolist() == [2, 4, 6, 8]


def test_grouped_rounds_mean_of_group_means_is_the_global_mean():
    # Sec. 3.3, last paragraph: two equal groups, everybody selected inside each group, then an inter-group round over
    # everybody: group members hold their group's mean after the intra-group rounds, so the inter-group mean is the mean
    # of the group means -- for equal groups, the plain mean of all devices (FedAvg's aggregation equation).
    net, w0, x, y, cyc = _toy(4, [1, 2, 3, 4], 2)
    cyc.local_steps()
    before = cyc.params.copy()
    groups = [np.array([1, 1, 0, 0], dtype=np.uint8), np.array([0, 0, 1, 1], dtype=np.uint8)]
    for g, members in enumerate(groups):
        sel = cyc.select_group(g, members, 2)
        assert sorted(sel.tolist()) == np.flatnonzero(members).tolist()          # nobody outside the group is drawn
        agg = cyc.aggregate_group(members)
        assert np.abs(agg - before[members.astype(bool)].mean(axis=0)).max() < 1e-15
        other = groups[1 - g].astype(bool)
        if g == 0:
            assert np.array_equal(cyc.params[other], before[other])               # the other group is untouched
    assert np.array_equal(cyc.params[0], cyc.params[1]) and np.array_equal(cyc.params[2], cyc.params[3])
    cyc.n_select = 4
    cyc.select(9); cyc.aggregate(resync=True)
    assert np.abs(cyc.agg - before.mean(axis=0)).max() < 1e-15
