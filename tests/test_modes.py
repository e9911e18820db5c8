"""Comparator modes (paper Sec. 2.1 distributed-SGD equation, Sec. 2.2 FedAvg equations, Sec. 4 Table 1) as
configurations of the same cycle, and the simulated clock of Sec. 2.3 (fast devices wait for slow ones)."""
import numpy as np
import pytest

import oracle
from oracle import nets
from paper_2111_08274_amd import modes


def test_mode_arguments_steps_and_clock_by_hand():
    r = [4, 2, 2, 1]                                   # Fig. 1's heterogeneity: powers 4 : 2 : 2 : 1
    a = modes.mode_arguments("hadfl", r, 2)
    assert a["ratio"].tolist() == r and a["n_select"] == 2 and a["t_sync"] == 1
    assert modes.steps_per_cycle("hadfl", r).tolist() == [4, 2, 2, 1]
    # every device is busy for the same time: E_k / r_k = 1 for all k, nobody waits
    assert modes.cycle_time("hadfl", r) == 1.0
    a = modes.mode_arguments("fedavg", r, 2, local_steps=4)
    assert a["ratio"].tolist() == [1, 1, 1, 1] and a["n_select"] == 4 and a["t_sync"] == 4
    assert modes.steps_per_cycle("fedavg", r, local_steps=4).tolist() == [4, 4, 4, 4]
    # the slowest device (power 1) needs 4 time units for its 4 steps and gates the round
    assert modes.cycle_time("fedavg", r, local_steps=4) == 4.0
    a = modes.mode_arguments("sync_sgd", r, 2)
    assert a["n_select"] == 4 and a["t_sync"] == 1
    assert modes.cycle_time("sync_sgd", r) == 1.0 and modes.steps_per_cycle("sync_sgd", r).sum() == 4
    # steps done per unit of simulated time: hadfl 9, fedavg 16/4 = 4, sync 4: the waiting the method removes
    assert modes.steps_per_cycle("hadfl", r).sum() / modes.cycle_time("hadfl", r) == 9.0
    assert modes.exchange_time(1, 100.0, 10.0) == 0.0
    assert modes.exchange_time(4, 100.0, 10.0) == pytest.approx(2 * 3 / 4 * 10.0)
    with pytest.raises(ValueError):
        modes.mode_arguments("gossip", r, 2)
    c = modes.Clock("fedavg", r, local_steps=4, t_comm=0.5)
    c.tick(); c.tick()
    assert c.t == 9.0 and c.steps == 32
    assert modes.speedup_table({"hadfl": 2.0, "fedavg": 6.0, "sync_sgd": 9.0}) == {"fedavg": 3.0, "sync_sgd": 4.5}


def _softmax_regression_grad(W, b, X, y):
    Z = X @ W + b
    Z = Z - Z.max(axis=1, keepdims=True)
    P = np.exp(Z); P /= P.sum(axis=1, keepdims=True)
    P[np.arange(len(y)), y] -= 1.0
    return X.T @ P / len(y), P.sum(axis=0) / len(y)


def test_sync_sgd_mode_is_momentum_sgd_on_the_mean_gradient():
    # One dense layer + softmax cross-entropy has the textbook gradient X^T (softmax - onehot) / B.  N devices take one
    # step each from the common model and all are averaged: the common model follows momentum SGD on the mean of the N
    # gradients, although every device keeps its own momentum buffer (the update is linear in the buffers).
    rng = np.random.default_rng(5)
    N, n, B, din, dout, lr, mom = 3, 8, 4, 5, 3, 0.05, 0.9
    b = nets._Builder(); b.dense(0, dout)
    net = oracle.Net(b.array(), (1, 1, din))
    w0 = rng.standard_normal(net.m_total) * 0.3
    x = rng.standard_normal((N, n, din)).astype(np.float32)
    y = rng.integers(0, dout, size=(N, n)).astype(np.int32)
    a = modes.mode_arguments("sync_sgd", [3, 1, 2], 1)
    cyc = oracle.Cycle(net, N, a["n_select"], w0, x, y, B, lr, mom, a["ratio"], seed=1, t_sync=a["t_sync"])
    assert cyc.steps.tolist() == [1, 1, 1]
    W = w0[:din * dout].reshape(din, dout).copy(); bias = w0[din * dout:].copy()
    VW, Vb = np.zeros_like(W), np.zeros_like(bias)
    for cycle in range(3):
        agg = cyc.run_cycle(cycle)
        lo = (cycle * B) % n
        gs = [_softmax_regression_grad(W, bias, x[k, lo:lo + B].astype(np.float64), y[k, lo:lo + B]) for k in range(N)]
        VW = mom * VW + np.mean([g[0] for g in gs], axis=0)
        Vb = mom * Vb + np.mean([g[1] for g in gs], axis=0)
        W = W - lr * VW; bias = bias - lr * Vb
        assert np.abs(agg[:din * dout].reshape(din, dout) - W).max() < 1e-13
        assert np.abs(agg[din * dout:] - bias).max() < 1e-13


def test_fedavg_mode_is_the_mean_of_equal_length_local_runs():
    rng = np.random.default_rng(6)
    N, n, B, din, dout = 4, 12, 4, 6, 3
    b = nets._Builder(); b.dense(0, dout)
    net = oracle.Net(b.array(), (1, 1, din))
    w0 = rng.standard_normal(net.m_total) * 0.3
    x = rng.standard_normal((N, n, din)).astype(np.float32)
    y = rng.integers(0, dout, size=(N, n)).astype(np.int32)
    a = modes.mode_arguments("fedavg", [4, 2, 2, 1], 2, local_steps=3)
    cyc = oracle.Cycle(net, N, a["n_select"], w0, x, y, B, 0.1, 0.0, a["ratio"], seed=2, t_sync=a["t_sync"])
    assert cyc.steps.tolist() == [3, 3, 3, 3]
    agg = cyc.run_cycle(0)
    singles = []
    for k in range(N):
        one = oracle.Cycle(net, 1, 1, w0, x[k:k + 1], y[k:k + 1], B, 0.1, 0.0, [1], seed=2, t_sync=3)
        one.local_steps(); singles.append(one.params[0].copy())
    assert np.abs(agg - np.mean(singles, axis=0)).max() < 1e-15
    assert cyc.flag.all() and np.allclose(cyc.weights, 0.25)
