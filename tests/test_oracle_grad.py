"""Pins for the oracle's forward/backward (paper Sec. 2.1: forward, loss, gradients of the loss).

Two independent checks, chosen so a transposed operand, a wrong index, a dropped term or a wrong sign fails:
  * central finite differences of the oracle's own loss (gradient consistent with the forward);
  * loss, logits and gradient against PyTorch's fp64 CPU library routines with autograd (forward right too).
"""
import numpy as np
import pytest

import oracle
from oracle import nets
from tests import torch_ref


def tiny_nets():
    out = {}
    b = nets._Builder(); b.dense(b.relu(b.dense(0, 4)), 3)
    out["mlp_5_4_3"] = (b.array(), (1, 1, 5))
    b = nets._Builder(); b.dense(b.conv(0, 3), 4)
    out["conv3x3_2x5x5"] = (b.array(), (5, 5, 2))
    b = nets._Builder(); b.dense(b.relu(b.conv(0, 3, stride=2, bias=False)), 3)
    out["conv3x3_s2"] = (b.array(), (6, 6, 2))
    b = nets._Builder(); t = b.conv(0, 4); b.dense(b.conv(t, 3, k=1, stride=2, pad=0), 3)
    out["conv1x1_s2"] = (b.array(), (4, 4, 2))
    b = nets._Builder(); b.dense(b.relu(b.bn(b.conv(0, 3, bias=False))), 3)
    out["bn"] = (b.array(), (4, 4, 2))
    b = nets._Builder(); b.dense(b.maxpool(b.relu(b.conv(0, 3))), 3)
    out["maxpool"] = (b.array(), (4, 6, 2))
    b = nets._Builder()
    t = b.relu(b.bn(b.conv(0, 4, bias=False)))
    u = b.bn(b.conv(b.relu(b.bn(b.conv(t, 4, bias=False))), 4, bias=False))
    b.dense(b.gap(b.relu(b.add(u, t))), 3)
    out["residual_gap"] = (b.array(), (4, 4, 3))
    b = nets._Builder()
    t = b.relu(b.bn(b.conv(0, 4, bias=False)))
    u = b.bn(b.conv(b.relu(b.bn(b.conv(t, 6, stride=2, bias=False))), 6, bias=False))
    sc = b.bn(b.conv(t, 6, k=1, stride=2, pad=0, bias=False))
    b.dense(b.gap(b.relu(b.add(u, sc))), 3)
    out["residual_proj"] = (b.array(), (4, 4, 3))
    return out


TINY = tiny_nets()


def _setup(name, B=4, seed=0):
    ops, shape = TINY[name]
    net = oracle.Net(ops, shape)
    rng = np.random.default_rng(seed)
    w = rng.standard_normal(net.m_total) * 0.5
    for off, cnt, kind, _ in net.layout():
        if kind == "gamma":
            w[off:off + cnt] = 1.0 + 0.3 * rng.standard_normal(cnt)
        if kind == "running_var":
            w[off:off + cnt] = 1.0
    x = rng.standard_normal((B,) + shape).astype(np.float32)
    y = rng.integers(0, net.n_out, size=B).astype(np.int32)
    return net, ops, shape, w, x, y


@pytest.mark.parametrize("name", sorted(TINY))
def test_gradient_matches_finite_differences(name):
    net, ops, shape, w, x, y = _setup(name)
    loss, grad = net.loss_grad(w, x, y)
    h = 1e-5
    fd = np.zeros(net.m_train)
    for j in range(net.m_train):
        wp = w.copy(); wp[j] += h
        wm = w.copy(); wm[j] -= h
        fd[j] = (net.loss_grad(wp, x, y)[0] - net.loss_grad(wm, x, y)[0]) / (2 * h)
    scale = max(np.abs(fd).max(), 1e-3)
    assert np.abs(fd - grad).max() / scale <= 1e-6, name


@pytest.mark.parametrize("name", sorted(TINY))
def test_forward_and_gradient_match_torch_fp64(name):
    net, ops, shape, w, x, y = _setup(name, B=5, seed=3)
    loss, grad, logits, _ = net.loss_grad(w, x, y, want_logits=True)
    tl, tg, tz = torch_ref.loss_grad(ops, shape, w, x, y)
    assert np.abs(logits - tz).max() <= 1e-11
    assert abs(loss - tl) <= 1e-12
    assert np.abs(grad - tg).max() <= 1e-11


@pytest.mark.parametrize("name,B", [("mlp", 3), ("cnn2", 2)])
def test_named_small_nets_match_torch_fp64(name, B):
    net = oracle.Net.named(name)
    fn, shape = nets.NETS[name]
    rng = np.random.default_rng(5)
    w = rng.standard_normal(net.m_total) * 0.05
    x = rng.standard_normal((B,) + shape).astype(np.float32)
    y = rng.integers(0, 10, size=B).astype(np.int32)
    loss, grad, logits, _ = net.loss_grad(w, x, y, want_logits=True)
    tl, tg, tz = torch_ref.loss_grad(fn(), shape, w, x, y)
    assert np.abs(logits - tz).max() <= 1e-10
    assert np.abs(grad - tg).max() <= 1e-10


def test_parameter_counts_of_the_paper_sized_nets():
    # published sizes of the two architectures in 32x32-input form, worked out layer by layer
    r = oracle.Net.named("resnet18")
    assert r.m_train == 11173962 and r.m_total - r.m_train == 9600
    v = oracle.Net.named("vgg16")
    assert v.m_train == 14728266
    assert oracle.Net.named("mlp").m_train == 784 * 128 + 128 + 128 * 10 + 10 == 101770
    assert oracle.Net.named("cnn2").m_train == 27 * 32 + 32 + 288 * 64 + 64 + 4096 * 10 + 10 == 60362


def test_resnet_block_and_vgg_group_match_torch_fp64():
    # whole paper-sized nets are too slow for a unit test; a narrow copy keeps every op kind and connection
    b = nets._Builder()
    t = b.relu(b.bn(b.conv(0, 4, bias=False)))
    cin = 4
    for cout, stride in ((4, 1), (8, 2)):
        for blk in range(2):
            s = stride if blk == 0 else 1
            u = b.relu(b.bn(b.conv(t, cout, stride=s, bias=False)))
            u = b.bn(b.conv(u, cout, bias=False))
            sc = b.bn(b.conv(t, cout, k=1, stride=s, pad=0, bias=False)) if (s != 1 or cin != cout) else t
            t = b.relu(b.add(u, sc)); cin = cout
    b.dense(b.gap(t), 10)
    ops, shape = b.array(), (8, 8, 3)
    net = oracle.Net(ops, shape)
    rng = np.random.default_rng(9)
    w = rng.standard_normal(net.m_total) * 0.3
    x = rng.standard_normal((4,) + shape).astype(np.float32)
    y = rng.integers(0, 10, size=4).astype(np.int32)
    loss, grad, logits, _ = net.loss_grad(w, x, y, want_logits=True)
    tl, tg, tz = torch_ref.loss_grad(ops, shape, w, x, y)
    assert np.abs(logits - tz).max() <= 1e-10 and np.abs(grad - tg).max() <= 1e-10


def test_bn_running_statistics_follow_the_stated_rule():
    net, ops, shape, w, x, y = _setup("bn", B=6, seed=2)
    import torch
    w2 = w.copy()
    _, _, _, after = net.loss_grad(w2, x, y, update_stats=True, want_logits=True)
    # the BN input is the conv output: recompute it with torch and apply momentum 0.1, unbiased variance
    leaves, _, m_train = torch_ref.split_params(ops, shape, w)
    xin = torch.as_tensor(x.astype(np.float64)).permute(0, 3, 1, 2)
    z = torch.nn.functional.conv2d(xin, leaves[0, "w"].permute(3, 2, 0, 1), None, padding=1)
    mean = z.mean(dim=(0, 2, 3)).detach().numpy()
    var = z.var(dim=(0, 2, 3), unbiased=True).detach().numpy()
    c = 3
    assert np.allclose(after[m_train:m_train + c], 0.9 * w[m_train:m_train + c] + 0.1 * mean, atol=1e-12)
    assert np.allclose(after[m_train + c:m_train + 2 * c], 0.9 * w[m_train + c:] + 0.1 * var, atol=1e-12)
    assert np.array_equal(after[:m_train], w[:m_train])
