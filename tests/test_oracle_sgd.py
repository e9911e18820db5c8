"""Pins for the oracle's local update (paper Sec. 2.2, local-update equation; Algorithm 1 inner loop)."""
import numpy as np

import oracle
from oracle import nets


def _linear(din, dout):
    b = nets._Builder(); b.dense(0, dout, bias=False)
    return oracle.Net(b.array(), (1, 1, din))


def test_least_squares_gradient_is_the_closed_form():
    # loss = 1/(2B) ||XW - T||^2  =>  grad = X^T (XW - T) / B
    rng = np.random.default_rng(0)
    B, din, dout = 7, 5, 3
    net = _linear(din, dout)
    W = rng.standard_normal((din, dout)); X = rng.standard_normal((B, din)).astype(np.float32)
    T = rng.standard_normal((B, dout))
    loss, g = net.loss_grad(W.reshape(-1), X, target=T)
    Xd = X.astype(np.float64)
    assert abs(loss - 0.5 * np.sum((Xd @ W - T) ** 2) / B) < 1e-13
    assert np.abs(g.reshape(din, dout) - Xd.T @ (Xd @ W - T) / B).max() < 1e-13


def _softmax_regression_grad(W, b, X, y):
    Z = X @ W + b
    Z = Z - Z.max(axis=1, keepdims=True)
    P = np.exp(Z); P /= P.sum(axis=1, keepdims=True)
    P[np.arange(len(y)), y] -= 1.0
    return X.T @ P / len(y), P.sum(axis=0) / len(y)


def test_local_steps_are_minibatch_sgd_with_sequential_wrapping_batches():
    # one dense layer + softmax CE has the textbook gradient X^T (softmax - onehot)/B; replay Algorithm 1's
    # inner loop by hand (plain SGD, momentum 0) over a shard that wraps around
    rng = np.random.default_rng(1)
    din, dout, n, B, lr = 6, 4, 12, 4, 0.1
    b = nets._Builder(); b.dense(0, dout)
    net = oracle.Net(b.array(), (1, 1, din))
    w0 = rng.standard_normal(net.m_total) * 0.3
    x = rng.standard_normal((2, n, din)).astype(np.float32)
    y = rng.integers(0, dout, size=(2, n)).astype(np.int32)
    cyc = oracle.Cycle(net, 2, 1, w0, x, y, B, lr, 0.0, [2, 5], seed=1)
    assert cyc.steps.tolist() == [2, 5]
    v = cyc.local_steps()
    assert v.tolist() == [2, 5] and cyc.cursor.tolist() == [2, 5]
    for k, E in enumerate([2, 5]):
        W = w0[:din * dout].reshape(din, dout).copy(); bias = w0[din * dout:].copy()
        for e in range(E):
            first = (e * B) % n
            gW, gb = _softmax_regression_grad(W, bias, x[k, first:first + B].astype(np.float64), y[k, first:first + B])
            W -= lr * gW; bias -= lr * gb
        assert np.abs(cyc.params[k, :din * dout] - W.reshape(-1)).max() < 1e-13
        assert np.abs(cyc.params[k, din * dout:] - bias).max() < 1e-13
    # the cursor persists: a second call continues from batch 2 (replica 0) and wraps for replica 1
    cyc.local_steps()
    assert cyc.cursor.tolist() == [4, 10]


def test_momentum_two_steps_closed_form():
    rng = np.random.default_rng(2)
    din, dout, n, B, lr, mom = 5, 3, 8, 4, 0.05, 0.9
    b = nets._Builder(); b.dense(0, dout)
    net = oracle.Net(b.array(), (1, 1, din))
    w0 = rng.standard_normal(net.m_total) * 0.3
    x = rng.standard_normal((1, n, din)).astype(np.float32)
    y = rng.integers(0, dout, size=(1, n)).astype(np.int32)
    cyc = oracle.Cycle(net, 1, 1, w0, x, y, B, lr, mom, [1], seed=1, t_sync=2)
    cyc.local_steps()
    W = w0[:din * dout].reshape(din, dout).copy(); bias = w0[din * dout:].copy()
    g1W, g1b = _softmax_regression_grad(W, bias, x[0, :B].astype(np.float64), y[0, :B])
    W1, b1 = W - lr * g1W, bias - lr * g1b
    g2W, g2b = _softmax_regression_grad(W1, b1, x[0, B:2 * B].astype(np.float64), y[0, B:2 * B])
    W2 = W1 - lr * (mom * g1W + g2W); b2 = b1 - lr * (mom * g1b + g2b)
    assert np.abs(cyc.params[0, :din * dout] - W2.reshape(-1)).max() < 1e-13
    assert np.abs(cyc.params[0, din * dout:] - b2).max() < 1e-13


def test_step_counts_by_hand(golden_dir):
    import os
    for line in open(os.path.join(golden_dir, "step_counts.txt")):
        if line.startswith("#") or not line.strip():
            continue
        r, t, s = [p.strip() for p in line.split("|")]
        got = oracle.step_counts([int(v) for v in r.split(",")], int(t))
        assert got.tolist() == [int(v) for v in s.split(",")], line
    assert oracle.step_counts([1, 2], 1, 3).tolist() == [3, 6]
    import pytest
    with pytest.raises(ValueError):
        oracle.step_counts([1, 0, 2])


def test_version_predictor_constant_and_linear_series():
    # Brown's double exponential smoothing: a constant series is forecast exactly; a linear series
    # v_j = c + d*j is forecast exactly in the limit (one step ahead: c + d*(j+1))
    p = oracle.Predictor(0.5)
    for _ in range(10):
        assert p.update(3.0, m=2) == 3.0
    q = oracle.Predictor(0.6)
    for j in range(80):
        f = q.update(2.0 + 0.5 * j, m=1)
    assert abs(f - (2.0 + 0.5 * 80)) < 1e-9
    # one explicit hand-worked update, alpha = 0.5, series 4, 2: s1 = 3, s2 = 3.5, a = 2.5, b = -0.5
    r = oracle.Predictor(0.5); r.update(4.0)
    assert r.update(2.0, m=1) == 2.0 and r.update.__self__.s1.value == 3.0 and r.s2.value == 3.5


def test_step_counts_from_warm_up_times_by_hand():
    # Sec. 3.2 / Sec. 3.3: per-unit times 1, 2, 4 -> hyperperiod 4 -> 4, 2, 1 units per hyperperiod
    assert oracle.steps_from_times([1.0, 2.0, 4.0], 1, 1.0).tolist() == [4, 2, 1]
    # three warm-up units each, noisy clocks, quantum 0.5: 1.02, 1.967, 4.067 -> 2, 4, 8 quanta -> lcm 8
    assert oracle.steps_from_times([3.06, 5.9, 12.2], 3, 0.5).tolist() == [4, 2, 1]
    # times proportional to 1 / power reproduce the ratio rule: powers 1 : 2 : 3 : 4 -> times 12, 6, 4, 3
    assert oracle.steps_from_times([12.0, 6.0, 4.0, 3.0], 1, 1.0).tolist() == oracle.step_counts([1, 2, 3, 4]).tolist() == [1, 2, 3, 4]
    # Fig. 1's 4 : 2 : 1 powers with t_sync 2 and 5 steps per unit
    assert oracle.steps_from_times([1.0, 2.0, 4.0], 1, 1.0, t_sync=2, steps_per_unit=5).tolist() == [40, 20, 10]
    # equal devices: everybody takes t_sync units; a time below half a quantum still counts as one quantum
    assert oracle.steps_from_times([7.0, 7.0, 7.0], 7, 0.25, t_sync=3).tolist() == [3, 3, 3]
    assert oracle.steps_from_times([0.1, 2.0], 1, 1.0).tolist() == [2, 1]
    import pytest
    for bad in ([1.0, 0.0], [1.0, -2.0]):
        with pytest.raises(ValueError):
            oracle.steps_from_times(bad, 1, 1.0)
    with pytest.raises(ValueError):
        oracle.steps_from_times([1.0, 2.0], 1, 0.0)
    with pytest.raises(ValueError):
        oracle.steps_from_times([1.0, 1.0e6 + 0.37], 1, 1e-3)          # lcm of incommensurable fine counts explodes
