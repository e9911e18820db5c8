"""hadfl_select_static -- the selection for callers that cannot allocate -- against hadfl_select, through the C-ABI:
the same replicas drawn, the same flags and the same weights, bit for bit, on calls in a row that shrink and grow the
input (every call on a GPU shares one static working array, which keeps the last call's contents)."""
import numpy as np
import pytest

from paper_2111_08274_amd import hadfl

pytestmark = pytest.mark.gpu


def _with_context(N, n_select, versions, avail, cycle, seed, weight_mode):
    import torch
    hc = hadfl.make_config(N, n_select, net="none", m_none=64, weight_mode=weight_mode, seed=seed)
    ctx = hadfl.Context(hc, np.ones(N, dtype=np.int32), replicas=torch.zeros(N * 64, dtype=torch.float32, device="cuda"))
    ctx.select(cycle, versions=torch.as_tensor(versions).cuda(), avail=avail)
    out = ctx.selected()
    ctx.close()
    return out


def test_static_selection_equals_the_context_one_on_calls_in_a_row():
    import torch
    rng = np.random.default_rng(12)
    # the second call is smaller than the first, the third larger again, the fourth the maximum size
    cases = [(64, 8, 0, False), (16, 4, 0, True), (5, 5, 1, False), (200, 17, 1, True), (1024, 3, 0, False), (4, 2, 0, False)]
    outs = []
    for i, (N, n_select, weight_mode, masked) in enumerate(cases):
        versions = rng.integers(0, 51, size=N).astype(np.int32)
        avail = None
        if masked:
            avail = np.ones(N, dtype=np.uint8)
            avail[rng.choice(N, size=N - n_select - 1, replace=False)] = 0
        cycle, seed = 1000 + i, 2021 + i
        vd = torch.as_tensor(versions).cuda()
        ad = None if avail is None else torch.as_tensor(avail).cuda()
        sel = torch.full((n_select,), -7, dtype=torch.int32, device="cuda")
        flag = torch.full((N,), 9, dtype=torch.uint8, device="cuda")
        wts = torch.full((N,), -1.0, dtype=torch.float32, device="cuda")
        hadfl.select_static(vd, n_select, seed, cycle, sel, flag, wts, avail=ad, weight_mode=weight_mode)
        outs.append((sel, flag, wts, N, n_select, versions, avail, cycle, seed, weight_mode))
    torch.cuda.synchronize()
    for sel, flag, wts, N, n_select, versions, avail, cycle, seed, weight_mode in outs:
        want_sel, want_flag, want_w = _with_context(N, n_select, versions, avail, cycle, seed, weight_mode)
        assert sel.cpu().numpy().tolist() == want_sel.tolist(), (N, n_select)
        assert np.array_equal(flag.cpu().numpy(), want_flag)
        assert np.array_equal(wts.cpu().numpy(), want_w)
        assert abs(float(want_w.sum()) - 1.0) < 1e-6


def test_static_selection_rejects_what_its_working_array_cannot_hold():
    import torch
    v = torch.zeros(2048, dtype=torch.int32, device="cuda")
    sel = torch.zeros(16, dtype=torch.int32, device="cuda")
    flag = torch.zeros(2048, dtype=torch.uint8, device="cuda")
    wts = torch.zeros(2048, dtype=torch.float32, device="cuda")
    with pytest.raises(hadfl.HadflError) as e:
        hadfl.select_static(v, 4, 1, 0, sel, flag, wts)
    assert e.value.status == hadfl.EINVAL and "1024" in str(e.value)
    with pytest.raises(hadfl.HadflError) as e:
        hadfl.select_static(v[:8], 9, 1, 0, sel, flag, wts)
    assert e.value.status == hadfl.EINVAL
    # fewer present than asked for: the surplus draws are -1, nothing is written out of bounds
    avail = torch.zeros(8, dtype=torch.uint8, device="cuda"); avail[3] = 1; avail[5] = 1
    hadfl.select_static(v[:8], 4, 1, 0, sel, flag, wts, avail=avail)
    torch.cuda.synchronize()
    got = sel.cpu().numpy().tolist()
    assert sorted(got[:2]) == [3, 5] and got[2:4] == [-1, -1]
    assert flag[:8].cpu().numpy().tolist() == [0, 0, 0, 1, 0, 1, 0, 0]
