"""GPU parity of the bf16 configuration (bf16 activations / activation gradients / weights as used, fp32 master
weights and accumulation) against the oracle's bf16-rounding mode.  Bar: 2e-2 relative on the parameters."""
import numpy as np
import pytest

import oracle
from oracle import nets
from paper_2111_08274_amd import hadfl, synth
from tests import parity_metrics as pm
from tests.pair import Pair
from tests.test_gpu_train import CASES, _data

pytestmark = pytest.mark.gpu
REL = 2e-2


@pytest.mark.parametrize("name", sorted(CASES))
def test_layer_kinds_bf16(name):
    ops, shape, batch = CASES[name]
    N, n = 3, batch * 3
    net = oracle.Net(ops, shape)
    x, y = _data(N, n, shape, net.n_out, seed=len(name))
    p = Pair(ops, shape, N, 2, x, y, batch, 0.01, 0.9, [1, 3, 2], bf16=True)
    w = p.forced_steps()                      # every step from a common state: each tensor's update within 2e-2
    d = p.max_rel_diff()
    print(name, "bf16 rel", d, "updates:", pm.show(w), "loss", p.gpu.losses(), p.cpu.loss, flush=True)
    assert w["max"] <= pm.UPDATE_REL_BF16          # one or two layers: element-wise within 2e-2, no twin needed
    assert d <= REL, (name, d)
    assert np.abs(p.gpu.losses() - p.cpu.loss).max() <= 0.05 * max(1.0, np.abs(p.cpu.loss).max())
    p.select_aggregate(0)
    w2 = p.local_steps(check_updates=True)   # one free-running call of 1, 3 and 2 steps
    print(name, "free-running updates:", pm.show(w2), flush=True)
    assert p.max_rel_diff() <= REL
    p.close()


def _regular_cases():
    """Layers wide enough (channels multiple of 64, power-of-two images) for the lean bf16 convolution kernels."""
    c = {}
    b = nets._Builder()
    t = b.relu(b.conv(0, 64))
    b.dense(b.relu(b.conv(t, 64)), 5)
    c["conv64_bias_relu"] = (b.array(), (8, 8, 3), 8)
    b = nets._Builder()
    t = b.relu(b.bn(b.conv(0, 64)))
    t = b.maxpool(b.relu(b.bn(b.conv(t, 64))))
    t = b.maxpool(b.relu(b.bn(b.conv(t, 128))))
    b.dense(t, 5)
    c["vgg_block_64_128"] = (b.array(), (8, 8, 3), 8)
    b = nets._Builder()
    t = b.relu(b.bn(b.conv(0, 64, bias=False)))
    u = b.bn(b.conv(b.relu(b.bn(b.conv(t, 64, bias=False))), 64, bias=False))
    b.dense(b.gap(b.relu(b.add(u, t))), 5)
    c["residual64"] = (b.array(), (4, 8, 3), 6)
    b = nets._Builder()
    t = b.relu(b.conv(0, 128, k=1, pad=0))
    b.dense(b.relu(b.conv(t, 192, k=1, pad=0)), 5)          # 1x1 "same" convolution, N = 192 -> 64-wide tiles
    c["conv1x1_128_192"] = (b.array(), (4, 4, 3), 10)
    return c


REGULAR = _regular_cases()


@pytest.mark.parametrize("name", sorted(REGULAR))
def test_regular_layers_bf16_lean_kernels(name):
    ops, shape, batch = REGULAR[name]
    N, n = 3, batch * 3
    net = oracle.Net(ops, shape)
    x, y = _data(N, n, shape, net.n_out, seed=len(name))
    p = Pair(ops, shape, N, 2, x, y, batch, 0.01, 0.9, [1, 3, 2], bf16=True)
    w = p.forced_steps()
    d = p.max_rel_diff()
    print(name, "bf16 rel", d, "updates:", pm.show(w), "loss", p.gpu.losses(), p.cpu.loss, flush=True)
    assert d <= REL, (name, d)
    p.select_aggregate(0)
    p.local_steps(check_updates=True)
    assert p.max_rel_diff() <= REL
    p.close()


def test_regular_layer_bf16_tall_tiles():
    """Enough output rows (12 x 64 x 64 per replica, 3 replicas) that the lean kernels pick their 256-row tiles."""
    b = nets._Builder()
    t = b.relu(b.conv(0, 64))
    t = b.relu(b.conv(t, 64))
    b.dense(b.gap(t), 5)
    ops, shape, batch = b.array(), (64, 64, 3), 12
    N = 3
    x, y = _data(N, batch, shape, 5, seed=77)
    p = Pair(ops, shape, N, 2, x, y, batch, 0.01, 0.9, [1, 1, 1], bf16=True)
    w = p.forced_steps()
    d = p.max_rel_diff()
    print("tall tiles bf16 rel", d, "updates:", pm.show(w), "loss", p.gpu.losses(), p.cpu.loss, flush=True)
    assert d <= REL
    p.close()


def _narrow_vgg():
    b = nets._Builder()
    t = 0
    for width, reps in ((16, 2), (32, 2), (64, 3)):
        for _ in range(reps):
            t = b.relu(b.bn(b.conv(t, width)))
        t = b.maxpool(t)
    b.dense(t, 10)
    return b.array()


def test_vgg_structure_bf16_three_cycles():
    # The first step agrees to 0.5% of the update (the layer cases above: 1e-7..5e-5 of the weights).  After it, master
    # weights that differ by a few percent of a bf16 ulp round to different bf16 weights in about that fraction of
    # the positions, each a 0.4% change of the weight used by the next forward pass: the two trajectories separate at
    # bf16 resolution whatever the kernel does.  Measured at lr 0.01 on this net: 3.6e-3, 1.3e-2, 2.8e-2 of max|w|
    # after cycles 0, 1, 2.  The bar is asserted at lr 0.003, where three cycles stay inside it.
    ops, shape = _narrow_vgg(), (16, 16, 3)
    N, batch, n = 4, 16, 64
    x, y = synth.class_shift_images(N, n, shape, 10, seed=105, dirichlet=0.3)
    p = Pair(ops, shape, N, 2, x, y, batch, 0.003, 0.9, [1, 3, 2, 4], bf16=True)
    for cycle in range(3):
        w = p.local_steps(check_updates=cycle == 0)          # later cycles start from states that already differ
        d = p.max_rel_diff()
        p.select_aggregate(cycle)
        print("narrow vgg bf16 cycle", cycle, "rel", d, "updates:", pm.show(w), flush=True)
        assert d <= REL
    p.close()


def test_vgg_structure_bf16_every_step_at_the_workload_lr_from_a_common_state():
    """The same net at the workload's lr 0.01 for five cycles, every sub-step from a common state: each tensor's update
    within 2e-2 of its size, whatever the free-running trajectories do."""
    ops, shape = _narrow_vgg(), (16, 16, 3)
    N, batch, n = 4, 16, 64
    x, y = synth.class_shift_images(N, n, shape, 10, seed=105, dirichlet=0.3)
    p = Pair(ops, shape, N, 2, x, y, batch, 0.01, 0.9, [1, 3, 2, 4], bf16=True)
    for cycle in range(5):
        w = p.forced_steps()
        d = p.max_rel_diff()
        p.select_aggregate(cycle)
        print("narrow vgg bf16 forced cycle", cycle, "rel", d, "updates:", pm.show(w), flush=True)
        assert d <= REL
    p.close()


def test_vgg16_full_width_bf16_against_oracle():
    fn, shape = nets.NETS["vgg16"]
    N, batch, n = 2, 32, 32          # 32 images: the deepest batch norms still see 128 rows
    x, y = synth.class_shift_images(N, n, shape, 10, seed=105)
    p = Pair(fn(), shape, N, 1, x, y, batch, 0.01, 0.9, [1, 1], net_name="vgg16", bf16=True)
    w = p.forced_steps()
    d = p.max_rel_diff()
    p.select_aggregate(0)
    print("vgg16 bf16 rel", d, "updates:", pm.show(w), flush=True)
    assert d <= REL
    p.close()


def test_regular_layer_bf16_256_tiles():
    """Forward and data-gradient kernels with 256 x 256 tiles (one workgroup of eight waves per compute unit).  The
    launcher only picks them when a launch fills the chip; the hint makes this small problem take them."""
    b = nets._Builder()
    t = b.relu(b.conv(0, 64))
    t = b.relu(b.conv(t, 256))
    t = b.relu(b.bn(b.conv(t, 256, bias=False)))         # the convolution also leaves the BN's sums (ragged last tile)
    b.dense(b.gap(t), 5)
    ops, shape, batch = b.array(), (8, 8, 3), 5          # 320 rows per replica: one full and one ragged 256-row tile
    N = 3
    x, y = _data(N, batch, shape, 5, seed=78)
    p = Pair(ops, shape, N, 2, x, y, batch, 0.01, 0.9, [2, 1, 1], bf16=True, options={hadfl.OPT_TILE_HINT: 1})
    w = p.forced_steps()
    d = p.max_rel_diff()
    print("256 tiles bf16 rel", d, "updates:", pm.show(w), "loss", p.gpu.losses(), p.cpu.loss, flush=True)
    assert d <= REL
    p.close()


@pytest.mark.parametrize("hint", [0, 1])
def test_regular_layers_bf16_position_sorted_rows(hint):
    """Batch 64 on 8x8 / 4x4 / 2x2 images: the lean kernels order GEMM rows (and the weight gradient's contraction) by
    pixel position and leave out the taps no row of a tile can reach.  hint 1 also sends the 128- and 256-wide layers
    through the 256-row tiles."""
    b = nets._Builder()
    t = b.relu(b.conv(0, 64))
    t = b.relu(b.bn(b.conv(t, 64)))
    t = b.maxpool(t)
    t = b.relu(b.conv(t, 128))
    t = b.relu(b.bn(b.conv(t, 256)))
    t = b.maxpool(t)
    t = b.relu(b.conv(t, 256))
    b.dense(b.gap(t), 5)
    ops, shape, batch = b.array(), (8, 8, 3), 64
    N = 3
    x, y = _data(N, 2 * batch, shape, 5, seed=79)
    p = Pair(ops, shape, N, 2, x, y, batch, 0.01, 0.9, [2, 1, 1], bf16=True, options={hadfl.OPT_TILE_HINT: hint})
    w = p.forced_steps()
    d = p.max_rel_diff()
    print("position-sorted rows bf16 rel", d, "updates:", pm.show(w), "loss", p.gpu.losses(), p.cpu.loss, flush=True)
    assert d <= REL
    p.close()


@pytest.mark.parametrize("side,batch", [(16, 6), (32, 3)])
def test_wide_image_layers_bf16_patch_kernel(side, batch):
    """16- and 32-pixel-wide images with 64 / 128 channels: forward and data gradient run in the kernel that keeps a
    256-pixel tile with its border in LDS and serves all nine taps from it (one and two 64-channel slices, 64 and 128
    output channels, tiles at the top, middle and bottom of an image)."""
    b = nets._Builder()
    t = b.relu(b.conv(0, 64))
    t = b.relu(b.bn(b.conv(t, 64)))
    t = b.relu(b.conv(t, 128))
    t = b.relu(b.bn(b.conv(t, 128)))
    t = b.relu(b.conv(t, 64))
    b.dense(b.gap(t), 5)
    ops, shape = b.array(), (side, side, 3)
    N = 3
    x, y = _data(N, 2 * batch, shape, 5, seed=80 + side)
    p = Pair(ops, shape, N, 2, x, y, batch, 0.01, 0.9, [2, 1, 1], bf16=True)
    w = p.forced_steps()
    d = p.max_rel_diff()
    print("patch kernel bf16 rel", side, d, "updates:", pm.show(w), "loss", p.gpu.losses(), p.cpu.loss, flush=True)
    assert d <= REL
    p.close()


def test_many_convolutions_more_update_pieces_than_one_launch_takes():
    """Twenty convolutions that each apply their own update (epilogue or split-K reduction) leave 21 separate pieces of
    the parameter row (the BN parameters between them, the classifier) for the update kernel: more than one launch's
    table holds.  The convolutions sit side by side on one stem and are summed, not stacked: a stack of twenty
    batch-normalised layers amplifies bf16 rounding so much that the oracle disagrees with its own twin by half an update
    (tests/test_oracle_sensitivity.py), and nothing could be told from it.  Two steps, so the second runs on weights
    every path has updated."""
    b = nets._Builder()
    stem = b.relu(b.bn(b.conv(0, 64, bias=False)))
    t = b.bn(b.conv(stem, 64, bias=False))
    for _ in range(18):
        t = b.add(t, b.bn(b.conv(stem, 64, bias=False)))
    b.dense(b.gap(b.relu(t)), 5)
    ops, shape, batch = b.array(), (4, 4, 3), 8
    N = 2
    x, y = _data(N, 2 * batch, shape, 5, seed=91)
    p = Pair(ops, shape, N, 1, x, y, batch, 0.01, 0.9, [2, 1], bf16=True)
    w = p.forced_steps()
    d = p.max_rel_diff()
    print("many convolutions bf16 rel", d, "updates:", pm.show(w), "loss", p.gpu.losses(), p.cpu.loss, flush=True)
    assert d <= REL
    w2 = p.local_steps(check_updates=True)
    print("many convolutions free-running", pm.show(w2), flush=True)
    p.close()


def test_batch_norm_scales_of_exactly_zero_bf16():
    """The batch-norm backward pass takes its sums from the data gradient of the convolution above, as sum g and
    sum g * y with y the BN's own output -- which says nothing about x where the scale gamma is exactly zero.  Channels with
    gamma = 0 (beta positive and negative) in every position such a BN can have: BN -> ReLU -> conv, BN -> ReLU -> pool ->
    conv, and BN -> conv with no ReLU between; their gamma gradients must still match the oracle's."""
    b = nets._Builder()
    t = b.relu(b.bn(b.conv(0, 64)))
    t = b.relu(b.bn(b.conv(t, 64)))
    t = b.maxpool(b.relu(b.bn(b.conv(t, 64))))
    t = b.bn(b.conv(t, 64))
    t = b.relu(b.conv(t, 64))
    b.dense(b.gap(t), 5)
    ops, shape, batch = b.array(), (8, 8, 3), 16
    N = 2
    x, y = _data(N, 2 * batch, shape, 5, seed=93)
    p = Pair(ops, shape, N, 1, x, y, batch, 0.01, 0.9, [2, 1], bf16=True)
    gammas = [(o, c) for o, c, kind, _ in p.layout if kind == "gamma"]
    assert len(gammas) == 4
    for o, c in gammas:
        p.cpu.params[:, o + 3] = 0.0; p.cpu.params[:, o + c + 3] = 0.5        # gamma 0, beta > 0: the ReLU passes everything
        p.cpu.params[:, o + 9] = 0.0; p.cpu.params[:, o + c + 9] = -0.5       # gamma 0, beta < 0: the ReLU passes nothing
        p.cpu.params[:, o + 20] = 0.0                                         # gamma 0, beta 0
    # one step by hand first, from a common state, looking at the special channels themselves
    p.share_state()
    before = p.cpu.params.copy()
    ones = np.ones(N, dtype=np.int32)
    p.gpu.set_steps(ones); p.gpu.local_steps(); p.cpu.local_steps(steps=ones)
    for k in range(N):
        got = p.gpu.params(k).astype(np.float64)
        for o, c in gammas:
            want = p.cpu.params[k][o:o + c] - before[k][o:o + c]
            have = got[o:o + c] - before[k][o:o + c]
            scale = np.abs(want).max()
            for ch in (3, 9, 20):
                assert abs(have[ch] - want[ch]) <= 0.05 * scale, (k, o, ch, have[ch], want[ch], scale)
            assert np.abs(want[[3, 20]]).max() > 0          # the scale's gradient is not zero just because the scale is
    p.gpu.set_steps(p.cpu.steps)
    w = p.forced_steps()                 # then the cycle's two sub-steps (the scales are tiny, no longer zero, in the second)
    d = p.max_rel_diff()
    print("zero scales bf16 rel", d, "updates:", pm.show(w), flush=True)
    assert d <= REL
    p.close()
