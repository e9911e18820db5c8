"""GPU parity of selection (bit-exact) and partial aggregation (fp32 sum vs the oracle's fp64 sum) through the C-ABI."""
import numpy as np
import pytest

import oracle
from paper_2111_08274_amd import hadfl, synth

pytestmark = pytest.mark.gpu
EPS32 = float(np.finfo(np.float32).eps)


def _ctx(N, n_select, m, rows=None, weight_mode=0, seed=synth.SELECT_SEED):
    import torch
    hc = hadfl.make_config(N, n_select, net="none", m_none=m, weight_mode=weight_mode, seed=seed)
    _, _, stride = hadfl.param_count(hc)
    rep = torch.zeros(N * stride, dtype=torch.float32, device="cuda")
    if rows is not None:
        rep.view(N, stride)[:, :m] = torch.as_tensor(rows[:, :m]).cuda()
    return hadfl.Context(hc, np.ones(N, dtype=np.int32), replicas=rep), stride


@pytest.mark.parametrize("N,n_select", [(1, 1), (4, 2), (8, 4), (16, 4), (64, 8), (100, 17), (64, 64), (1024, 3)])
def test_selection_is_bit_exact(N, n_select):
    import torch
    rng = np.random.default_rng(N * 131 + n_select)
    ctx, _ = _ctx(N, n_select, 64)
    for trial in range(12):
        hi = [4, 50, 8, 1000][trial % 4]
        v = rng.integers(0, hi + 1, size=N).astype(np.int32)
        avail = None
        if trial % 3 == 2 and N > n_select:
            avail = np.ones(N, dtype=np.uint8)
            avail[rng.choice(N, size=rng.integers(1, N - n_select + 1), replace=False)] = 0
        vd = torch.as_tensor(v).cuda()
        for cycle in (0, trial, 2 ** 40 + trial):
            ctx.select(cycle, versions=vd, avail=avail)
            sel, flag, w = ctx.selected()
            osel, oflag, of, _ = oracle.select(v, n_select, synth.SELECT_SEED, cycle, avail)
            assert sel.tolist() == osel.tolist(), (N, n_select, trial, cycle)
            assert flag.tolist() == oflag.tolist()
            assert np.array_equal(w, oracle.aggregation_weights(oflag).astype(np.float32))
    ctx.close()


def test_selection_weight_mode_1_and_errors():
    import torch
    v = np.array([1, 2, 3, 4, 4, 2, 9, 0], dtype=np.int32)
    ctx, _ = _ctx(8, 3, 64, weight_mode=1, seed=77)
    with pytest.raises(hadfl.HadflError) as e:
        ctx.aggregate()
    assert e.value.status == hadfl.ESTATE
    ctx.select(5, versions=torch.as_tensor(v).cuda())
    sel, flag, w = ctx.selected()
    osel, oflag, of, _ = oracle.select(v, 3, 77, 5)
    assert sel.tolist() == osel.tolist()
    ow = oracle.aggregation_weights(oflag, of, 1)
    assert np.allclose(w, ow, rtol=4 * EPS32, atol=0) and abs(float(w.sum()) - 1) < 4 * EPS32
    with pytest.raises(hadfl.HadflError) as e:
        ctx.select(6, versions=torch.as_tensor(v).cuda(), avail=np.array([1, 1, 0, 0, 0, 0, 0, 0], dtype=np.uint8))
    assert e.value.status == hadfl.EINVAL
    ctx.close()


@pytest.mark.parametrize("N,n_select", [(64, 9), (150, 20)])
def test_selection_weight_mode_1_weights_match_the_oracle(N, n_select):
    """f-weighted aggregation weights (the extension, not in the paper) with one chunk of 64 replicas and with
    several: the denominator adds the selected replicas' f in ascending index, in fp64, on both sides."""
    import torch
    rng = np.random.default_rng(N + n_select)
    ctx, _ = _ctx(N, n_select, 64, weight_mode=1, seed=91)
    for cycle in range(6):
        v = rng.integers(0, 30, size=N).astype(np.int32)
        avail = np.ones(N, dtype=np.uint8)
        avail[rng.choice(N, size=N // 5, replace=False)] = 0
        ctx.select(cycle, versions=torch.as_tensor(v).cuda(), avail=avail)
        sel, flag, w = ctx.selected()
        osel, oflag, of, _ = oracle.select(v, n_select, 91, cycle, avail)
        assert sel.tolist() == osel.tolist() and flag.tolist() == oflag.tolist()
        ow = oracle.aggregation_weights(oflag, of, 1)
        assert np.array_equal(w, ow.astype(np.float32)), (N, cycle)
    ctx.close()


@pytest.mark.parametrize("N,n_select,m", [(6, 3, 100037), (4, 1, 5), (9, 8, 70001), (12, 11, 4099), (3, 3, 1 << 20)])
def test_aggregate_matches_fp64_sum_and_resync_copies_it(N, n_select, m):
    import torch
    rng = np.random.default_rng(m)
    rows = (rng.standard_normal((N, m)) * 0.02).astype(np.float32)
    ctx, stride = _ctx(N, n_select, m, rows)
    v = rng.integers(0, 5, size=N).astype(np.int32)
    ctx.select(3, versions=torch.as_tensor(v).cuda())
    ctx.aggregate(resync=False)
    sel, flag, w = ctx.selected()
    got = ctx.params(-1)
    exact = oracle.aggregate_f32(rows, oracle.aggregation_weights(flag))
    tol = (n_select + 1) * EPS32 * float(np.abs(rows).max())
    assert np.abs(got.astype(np.float64) - exact).max() <= tol
    for k in range(N):                      # without resync the rows are untouched
        assert np.array_equal(ctx.params(k), rows[k])
    ctx.aggregate(resync=True)
    agg = ctx.params(-1)
    assert np.array_equal(agg, got)
    for k in range(N):
        assert np.array_equal(ctx.params(k), agg)
    assert float(ctx.replicas.view(N, stride)[:, m:].abs().max()) == 0.0 if stride > m else True
    ctx.close()


def test_identical_replicas_and_fedavg_special_cases():
    import torch
    rng = np.random.default_rng(5)
    m = 33333
    w = (rng.standard_normal(m) * 0.02).astype(np.float32)
    for n_select in (1, 2, 4):
        ctx, _ = _ctx(4, n_select, m, np.tile(w, (4, 1)))
        ctx.select(0, versions=torch.zeros(4, dtype=torch.int32, device="cuda"))
        ctx.aggregate(resync=False)
        assert np.array_equal(ctx.params(-1), w)      # weights 1, 1/2, 1/4 are exact in binary
        ctx.close()
    rows = (rng.standard_normal((5, m)) * 0.02).astype(np.float32)
    ctx, _ = _ctx(5, 5, m, rows)
    ctx.select(0, versions=torch.zeros(5, dtype=torch.int32, device="cuda"))
    ctx.aggregate(resync=False)
    assert np.abs(ctx.params(-1) - rows.astype(np.float64).mean(axis=0)).max() <= 6 * EPS32 * np.abs(rows).max()
    ctx.close()


def test_aggregation_stress_workload_full_size():
    """64 replicas x 11,173,962 values, versions U{0..50}, 8 selected: every cycle's selection bit-exact, the
    aggregate checked on sampled columns (the oracle sums them one by one) in the launch shape the benchmark times."""
    import torch
    cfg = synth.CONFIGS[4]
    N, n_select, m = cfg["n_replicas"], cfg["n_select"], cfg["m"]
    hc = hadfl.make_config(N, n_select, net="none", m_none=m, seed=synth.SELECT_SEED)
    _, _, stride = hadfl.param_count(hc)
    rep = torch.zeros(N * stride, dtype=torch.float32, device="cuda")
    rng = np.random.default_rng(11)
    cols = np.unique(np.concatenate([rng.integers(0, m, size=4000), np.arange(0, 64), np.arange(m - 64, m)]))
    sampled = np.zeros((N, len(cols)), dtype=np.float32)
    for k in range(N):
        row = synth.replica_rows_gaussian(1, m, cfg["std"], seed=400 + k)[0]
        sampled[k] = row[cols]
        rep.view(N, stride)[k, :m] = torch.as_tensor(row).cuda()
    versions = synth.versions_uniform(N, *cfg["version_range"], seed=304)
    vd = torch.as_tensor(versions).cuda()
    ctx = hadfl.Context(hc, np.ones(N, dtype=np.int32), replicas=rep)
    tol = (n_select + 1) * EPS32 * float(np.abs(sampled).max())
    for cycle in range(cfg["cycles"]):
        ctx.select(cycle, versions=vd)
        ctx.aggregate(resync=False)
        sel, flag, w = ctx.selected()
        osel, oflag, _, _ = oracle.select(versions, n_select, synth.SELECT_SEED, cycle)
        assert sel.tolist() == osel.tolist(), cycle
        if cycle % 100 == 0 or cycle == cfg["cycles"] - 1:
            got = ctx.params(-1)[cols]
            exact = oracle.aggregate_f32(sampled, oracle.aggregation_weights(oflag))
            assert np.abs(got.astype(np.float64) - exact).max() <= tol, cycle
    ctx.close()
