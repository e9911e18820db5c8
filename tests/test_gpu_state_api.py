"""The entry points that move a replica's state across the boundary (model backup of Sec. 3.1, step 4) and the
execution options: round trips, effect on the next local steps, error codes."""
import numpy as np
import pytest

from oracle import nets
from paper_2111_08274_amd import hadfl, synth
from tests.pair import Pair
from tests.test_gpu_train import CASES, _data

pytestmark = pytest.mark.gpu


def test_params_and_momentum_round_trip_and_drive_the_next_steps():
    ops, shape, batch = CASES["residual_projection"]
    N = 3
    x, y = _data(N, batch * 3, shape, 5, seed=4)
    p = Pair(ops, shape, N, 2, x, y, batch, 0.05, 0.9, [2, 1, 1])
    m_total, m_train = p.net.m_total, p.net.m_train
    rng = np.random.default_rng(1)
    w = (rng.standard_normal(m_total) * 0.1).astype(np.float32)
    b = (rng.standard_normal(m_train) * 0.01).astype(np.float32)
    p.gpu.set_params(1, w)
    p.gpu.set_momentum(1, b)
    assert np.array_equal(p.gpu.params(1), w) and np.array_equal(p.gpu.momentum(1), b)
    assert np.array_equal(p.gpu.params(0), p.w0) and not p.gpu.momentum(0).any()       # the other rows are untouched
    p.gpu.set_params(1, w[:100] * 2)                                                    # a prefix only
    assert np.array_equal(p.gpu.params(1)[:100], w[:100] * 2) and np.array_equal(p.gpu.params(1)[100:], w[100:])
    # the state that was put in is the state the next steps start from: take a checkpoint after one cycle, run the
    # second cycle, put the checkpoint back into a context at the same batch cursors and repeat it -- the same bits
    q = Pair(ops, shape, N, 2, x, y, batch, 0.05, 0.9, [2, 1, 1])
    q.gpu.local_steps()
    ckpt = [(q.gpu.params(k), q.gpu.momentum(k)) for k in range(N)]
    q.gpu.local_steps()
    after = [q.gpu.params(k) for k in range(N)]
    r = Pair(ops, shape, N, 2, x, y, batch, 0.05, 0.9, [2, 1, 1])
    r.gpu.local_steps()                                    # advances the cursors as q's first cycle did
    for k in range(N):
        r.gpu.set_params(k, np.zeros(m_total, dtype=np.float32))      # wipe, then restore
        r.gpu.set_params(k, ckpt[k][0]); r.gpu.set_momentum(k, ckpt[k][1])
    r.gpu.local_steps()
    for k in range(N):
        assert np.array_equal(r.gpu.params(k), after[k])
    r.close()
    for bad in (-1, N):
        with pytest.raises(hadfl.HadflError) as e:
            p.gpu.set_params(bad, w)
        assert e.value.status == hadfl.EINVAL
    with pytest.raises(hadfl.HadflError) as e:
        p.gpu.set_momentum(0, np.zeros(m_train + 1, dtype=np.float32))
    assert e.value.status == hadfl.EINVAL
    p.close(); q.close()


def test_options_change_no_bit_and_reject_unknown_values():
    b = nets._Builder()
    t = b.relu(b.conv(0, 64))
    t = b.relu(b.bn(b.conv(t, 64)))
    b.dense(b.gap(t), 5)
    ops, shape, batch = b.array(), (8, 8, 3), 8
    N = 3
    x, y = _data(N, 2 * batch, shape, 5, seed=6)
    outs = []
    for opts in ({}, {hadfl.OPT_SIDE_STREAM: 0}, {hadfl.OPT_TILE_HINT: 1}):
        p = Pair(ops, shape, N, 2, x, y, batch, 0.01, 0.9, [2, 1, 1], bf16=True, options=opts)
        p.gpu.local_steps()
        outs.append(np.stack([p.gpu.params(k) for k in range(N)]))
        if not opts:
            for opt, val in ((hadfl.OPT_SIDE_STREAM, 2), (hadfl.OPT_TILE_HINT, 3), (7, 0)):
                with pytest.raises(hadfl.HadflError) as e:
                    p.gpu.set_option(opt, val)
                assert e.value.status == hadfl.EINVAL
        p.close()
    assert np.array_equal(outs[0], outs[1])            # one stream or two: the same bits
    # other tiles add the same products in another order: equal to rounding, not to the bit
    assert np.abs(outs[0] - outs[2]).max() <= 1e-5


def test_selection_size_is_reported_with_the_selection():
    import torch
    hc = hadfl.make_config(8, 4, net="none", m_none=256)
    ctx = hadfl.Context(hc, np.ones(8, dtype=np.int32), replicas=torch.zeros(8 * 256, device="cuda"))
    v = torch.arange(8, dtype=torch.int32, device="cuda")
    ctx.select(0, versions=v)
    assert len(ctx.selected()[0]) == 4
    members = np.array([1, 1, 1, 0, 0, 0, 0, 0], dtype=np.uint8)
    ctx.select_group(1, members, 2, versions=v)
    sel, flag, _ = ctx.selected()
    assert len(sel) == 2 and flag.sum() == 2 and set(sel.tolist()) <= {0, 1, 2}
    # two masked selections in a row use the two staging slots; a third reuses the first
    for cycle in range(2, 7):
        avail = np.ones(8, dtype=np.uint8); avail[cycle % 8] = 0
        ctx.select(cycle, versions=v, avail=avail)
        sel, flag, _ = ctx.selected()
        assert (cycle % 8) not in sel.tolist() and len(sel) == 4
    with pytest.raises(hadfl.HadflError) as e:
        ctx.set_option(hadfl.OPT_SIDE_STREAM, 0)        # no trainable network
    assert e.value.status == hadfl.ESTATE
    ctx.close()
