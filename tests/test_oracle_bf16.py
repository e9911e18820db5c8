"""CPU pins of the oracle's bf16 mode (the workload with bf16 weights and activations, fp32 master weights and
accumulation).  What the mode rounds, to nearest-even bfloat16: the input batch, the convolution / dense weights as the
arithmetic uses them, every stored activation (logits included) and every stored activation gradient.  What it leaves
alone: biases, batch-norm parameters, sums, weight gradients, the update and the master weights.  Each of these is fixed
here without the GPU: the rounding function against an independent conversion, one small case worked by hand, a
dyadic network on which rounding must change nothing, and invariants of the update."""
import numpy as np

import oracle
from oracle import nets


def test_bf16_rounding_of_the_oracle_is_round_to_nearest_even():
    import torch
    rng = np.random.default_rng(0)
    v = np.concatenate([rng.standard_normal(2000) * 10.0 ** rng.integers(-6, 6, size=2000),
                        [1.00390625, 1.01171875, 0.0, -0.0, 3.0e38]]).astype(np.float32)
    want = torch.as_tensor(v).to(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([oracle.lib().hadfl_oracle_round_bf16(float(x)) for x in v], dtype=np.float32)
    assert np.array_equal(got, want)
    # by hand: bfloat16 keeps 8 significant bits, so the spacing in [1, 2) is 2^-7
    r = lambda x: oracle.lib().hadfl_oracle_round_bf16(x)
    assert r(1 + 2.0 ** -8 + 2.0 ** -9) == 1 + 2.0 ** -7          # above the midpoint: up
    assert r(1 + 2.0 ** -8 - 2.0 ** -20) == 1.0                   # below the midpoint: down
    assert r(1 + 2.0 ** -8) == 1.0                                # a tie goes to the even neighbour (1.0)
    assert r(1 + 3 * 2.0 ** -8) == 1 + 2 * 2.0 ** -7              # a tie above an odd neighbour goes up
    assert r(-(1 + 2.0 ** -8 + 2.0 ** -9)) == -(1 + 2.0 ** -7)


def _dense_2_1():
    b = nets._Builder()
    b.dense(0, 1)
    return b.array(), (1, 1, 2)


def test_rounding_points_of_one_dense_layer_worked_by_hand():
    """dense 2 -> 1 with bias, one sample, half squared error against a target.

    x = (1 + 2^-9, 9 * 2^-7): the first is not a bfloat16 and is rounded to 1.0 when the batch is stored.
    w = (1 + 2^-8 + 2^-9, 1 + 2^-8): as used they are 1 + 2^-7 (up) and 1.0 (tie to even).
    b = 2^-8 + 2^-20, not a bfloat16 (it would be 2^-8) and NOT rounded.
    z = (1 + 2^-7) * 1 + 1 * 9 * 2^-7 + b = 1 + 10 * 2^-7 + 2^-8 + 2^-20: just above the midpoint of 1 + 10 * 2^-7 and
        1 + 11 * 2^-7, so the stored logit is 1 + 11 * 2^-7 = 1.0859375.  (With a rounded bias z would sit exactly on the
        midpoint and go to the even neighbour 1 + 10 * 2^-7: the two readings give different logits.)
    target t = 0.5 + 2^-10:  d = z - t = 0.5849609375, loss = d^2 / 2 = 358801 / 2097152.
    The stored logit gradient is d rounded: 0.5849609375 = 149.75 * 2^-8 -> 150 * 2^-8 = 0.5859375.
    Bias gradient = 0.5859375.  Weight gradient = stored x times that, NOT rounded: (0.5859375, 9/128 * 150/256 =
    1350 / 32768), the second of which needs 11 significant bits."""
    ops, shape = _dense_2_1()
    net = oracle.Net(ops, shape, bf16=True)
    assert net.layout() == [(0, 2, "weight", 2), (2, 1, "bias", 2)]
    params = np.array([1 + 2.0 ** -8 + 2.0 ** -9, 1 + 2.0 ** -8, 2.0 ** -8 + 2.0 ** -20])
    x = np.array([[1 + 2.0 ** -9, 9 * 2.0 ** -7]], dtype=np.float32)
    t = np.array([[0.5 + 2.0 ** -10]])
    loss, grad, logits, _ = net.loss_grad(params, x, target=t, want_logits=True)
    assert logits[0, 0] == 1.0859375
    assert loss == 358801.0 / 2097152.0
    assert grad.tolist() == [0.5859375, 1350.0 / 32768.0, 0.5859375]
    # the same numbers without rounding, for contrast (also by hand): z = w.x + b exactly
    plain = oracle.Net(ops, shape)
    l2, g2, z2, _ = plain.loss_grad(params, x, target=t, want_logits=True)
    xe = x.astype(np.float64)[0]
    assert z2[0, 0] == params[0] * xe[0] + params[1] * xe[1] + params[2] and z2[0, 0] != logits[0, 0]


def test_convolution_weights_are_rounded_as_used_by_hand():
    """3x3 convolution (pad 1, no bias) on one 3x3 single-channel image that is 1 at the centre and 0 elsewhere, only
    the centre tap non-zero: w_c = 1 + 2^-8 + 2^-9.  The output image is w_c-as-used at the centre, 0 elsewhere; a dense
    layer of ones (bias 0) sums it: the logit is 1 + 2^-7 in bf16 mode and w_c itself without rounding."""
    b = nets._Builder()
    b.dense(b.conv(0, 1, bias=False), 1)
    ops, shape = b.array(), (3, 3, 1)
    wc = 1 + 2.0 ** -8 + 2.0 ** -9
    params = np.zeros(9 + 9 + 1)
    params[4] = wc
    params[9:18] = 1.0
    x = np.zeros((1, 3, 3, 1), dtype=np.float32); x[0, 1, 1, 0] = 1.0
    t = np.zeros((1, 1))
    _, g, z, _ = oracle.Net(ops, shape, bf16=True).loss_grad(params, x, target=t, want_logits=True)
    assert z[0, 0] == 1 + 2.0 ** -7
    # dL/dz = z (target 0), stored rounded = z, and every output pixel receives it (dense weights 1).  Tap (dy, dx) pairs
    # the centre input with the output pixel at (1 - dy, 1 - dx), which exists for all nine taps: every tap's gradient
    # is x_centre * z = z.  The dense weights' gradient is the stored convolution output times z: z^2 at the centre.
    assert g[:9].tolist() == [1 + 2.0 ** -7] * 9
    assert g[9 + 4] == (1 + 2.0 ** -7) ** 2 and g[9] == 0.0
    _, _, z_plain, _ = oracle.Net(ops, shape).loss_grad(params, x, target=t, want_logits=True)
    assert z_plain[0, 0] == wc


def _dyadic_case():
    b = nets._Builder()
    t = b.maxpool(b.relu(b.conv(0, 4)))
    b.dense(t, 2)
    ops, shape = b.array(), (4, 4, 2)
    net_args = (ops, shape)
    rng = np.random.default_rng(3)
    layout = oracle.Net(ops, shape).layout()
    m = max(o + c for o, c, _, _ in layout)
    params = np.zeros(m)
    for o, c, kind, _ in layout:
        params[o:o + c] = rng.integers(-2, 3, size=c) * 0.5          # multiples of 1/2 in [-1, 1]
    x = rng.integers(-2, 3, size=(4, 4, 4, 2)).astype(np.float32)      # small integers
    target = rng.integers(-3, 4, size=(4, 2)).astype(np.float64)
    return net_args, params, x, target


def test_rounding_changes_nothing_where_every_value_is_a_bfloat16():
    """Small-integer inputs, weights that are multiples of 1/2, batch 4, integer targets: every activation is a
    multiple of 1/4 below 2^7 and every activation gradient a multiple of 1/16 below 2^4, all exact in 8 bits... so the
    bf16 mode and the fp64 mode must agree bit for bit on the loss, the logits and every gradient."""
    (ops, shape), params, x, target = _dyadic_case()
    a = oracle.Net(ops, shape, bf16=True).loss_grad(params, x, target=target, want_logits=True)
    b = oracle.Net(ops, shape).loss_grad(params, x, target=target, want_logits=True)
    assert a[0] == b[0] and np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])
    assert np.abs(a[1]).max() > 0
    # every logit and every logit gradient really is a bfloat16, or the case would prove nothing
    r = np.vectorize(oracle.lib().hadfl_oracle_round_bf16)
    assert np.array_equal(r(a[2]), a[2]) and np.array_equal(r((a[2] - target) / 4), (a[2] - target) / 4)


def test_master_weights_and_update_stay_unrounded():
    """One local step in bf16 mode: new parameters = old - lr * gradient exactly in fp64 (Sec. 2.2's update on the
    master weights), where the gradient is what the bf16-mode backward pass returns; the new master weights are not
    bfloat16 values; and moving a master weight by less than the distance to its rounding boundary changes no
    gradient bit (only the rounded copy is used)."""
    b = nets._Builder()
    b.dense(b.relu(b.conv(0, 4)), 3)
    ops, shape = b.array(), (4, 4, 2)
    net = oracle.Net(ops, shape, bf16=True)
    rng = np.random.default_rng(9)
    w0 = rng.standard_normal(net.m_total) * 0.3
    x = rng.standard_normal((1, 8, 4 * 4 * 2)).astype(np.float32)
    y = rng.integers(0, 3, size=(1, 8)).astype(np.int32)
    _, g = net.loss_grad(w0.copy(), x[0], y=y[0])
    cyc = oracle.Cycle(net, 1, 1, w0, x, y, 8, 0.05, 0.0, [1], seed=1)
    cyc.local_steps()
    assert np.array_equal(cyc.params[0][:net.m_train], w0[:net.m_train] - 0.05 * g)
    r = np.vectorize(oracle.lib().hadfl_oracle_round_bf16)
    assert np.mean(r(cyc.params[0]) != cyc.params[0]) > 0.9
    # nudge every conv / dense weight towards its own rounded value by a quarter of the gap: same rounded copy
    w1 = w0.copy()
    for o, c, kind, _ in net.layout():
        if kind == "weight":
            w1[o:o + c] = w0[o:o + c] + 0.25 * (r(w0[o:o + c]) - w0[o:o + c])
    assert not np.array_equal(w1, w0)
    _, g1 = net.loss_grad(w1.copy(), x[0], y=y[0])
    assert np.array_equal(g1, g)
    # a bias is used as it is: the same nudge on the biases changes the gradient
    w2 = w0.copy()
    for o, c, kind, _ in net.layout():
        if kind == "bias":
            w2[o:o + c] = w0[o:o + c] + 0.25 * (r(w0[o:o + c]) - w0[o:o + c])
    _, g2 = net.loss_grad(w2.copy(), x[0], y=y[0])
    assert not np.array_equal(g2, g)
