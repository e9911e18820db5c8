"""Runs the oracle and the HIP library side by side on the same seeded inputs (helper for the GPU parity tests)."""
import numpy as np

import oracle
from paper_2111_08274_amd import hadfl, synth
from tests import parity_metrics as pm


def oracle_ops_to_custom(ops):
    """Oracle op rows (type,in0,in1,out,k,stride,pad,cout,bias) -> library rows (type,in0,in1,k,stride,pad,cout,bias)."""
    return np.asarray(ops, dtype=np.int32)[:, [0, 1, 2, 4, 5, 6, 7, 8]]


class Pair:
    def __init__(self, ops, in_shape, n_replicas, n_select, x, y, batch, lr, momentum, ratio, net_name=None,
                 seed=synth.SELECT_SEED, t_sync=1, init_seed=0, weight_mode=0, bf16=False, options=None):
        self.net = oracle.Net(ops, in_shape, bf16=bf16)
        n_classes = self.net.n_out
        kw = dict(batch=batch, n_samples=x.shape[1], in_shape=in_shape, n_classes=n_classes, lr=lr,
                  momentum=momentum, t_sync=t_sync, seed=seed, weight_mode=weight_mode, bf16=int(bf16))
        if net_name is None:
            self.hc = hadfl.make_config(n_replicas, n_select, net="custom", custom_ops=oracle_ops_to_custom(ops), **kw)
        else:
            self.hc = hadfl.make_config(n_replicas, n_select, net=net_name, **kw)
        self.layout = hadfl.param_layout(self.hc)
        assert self.layout == self.net.layout()
        self.w0 = synth.he_normal_init(self.layout, seed=init_seed)
        self.gpu = hadfl.Context(self.hc, ratio, w0=self.w0, x=x, y=y, options=options)
        self.cpu = oracle.Cycle(self.net, n_replicas, n_select, self.w0, x.reshape(n_replicas, x.shape[1], -1), y,
                                batch, lr, momentum, ratio, seed=seed, t_sync=t_sync, weight_mode=weight_mode)
        self.N = n_replicas
        self.bf16 = bool(bf16)
        self.momentum = float(momentum)
        self.versions_after_forced = None
        self.twin = None

    def max_param_diff(self, trainable_only=False):
        n = self.net.m_train if trainable_only else self.net.m_total
        d = 0.0
        for k in range(self.N):
            d = max(d, float(np.abs(self.gpu.params(k)[:n].astype(np.float64) - self.cpu.params[k][:n]).max()))
        return d

    def max_rel_diff(self):
        """max over replicas of max|w_gpu - w_oracle| / max|w_oracle| over the trainable vector."""
        n = self.net.m_train
        d = 0.0
        for k in range(self.N):
            ref = self.cpu.params[k][:n]
            d = max(d, float(np.abs(self.gpu.params(k)[:n].astype(np.float64) - ref).max() / np.abs(ref).max()))
        return d

    def share_state(self):
        """Gives both sides one state: the oracle's parameters, running statistics and momentum rounded to fp32."""
        for k in range(self.N):
            w32 = self.cpu.params[k].astype(np.float32)
            self.cpu.params[k] = w32
            self.gpu.set_params(k, w32)
            if self.momentum != 0.0:
                b32 = self.cpu.buf[k].astype(np.float32)
                self.cpu.buf[k] = b32
                self.gpu.set_momentum(k, b32)

    def _twin_start(self):
        """The oracle's twin: the same replicas from weights perturbed by pm.TWIN_PERTURBATION (relative, Gaussian),
        same momentum and batch cursors.  It shows how well conditioned each tensor's update is (tests/parity_metrics.py)."""
        if self.twin is None:
            c = self.cpu
            self.twin = oracle.Cycle(self.net, self.N, c.n_select, self.w0, c.x, c.y, c.batch, c.lr, c.momentum,
                                     np.ones(self.N, dtype=np.int32), seed=c.seed)
            self.twin_rng = np.random.default_rng(12345)
        self.twin.params[:] = self.cpu.params * (1.0 + pm.TWIN_PERTURBATION * self.twin_rng.standard_normal(self.cpu.params.shape))
        self.twin.buf[:] = self.cpu.buf
        self.twin.cursor[:] = self.cpu.cursor
        return self.twin.params.copy()

    def _check_updates(self, before, twin_before, stepped, what):
        bounds = pm.BOUNDS_BF16 if self.bf16 else pm.BOUNDS_F32
        worst = None
        for k in range(self.N):
            got = self.gpu.params(k)
            if stepped[k]:
                w = pm.assert_updates_within_twin(self.layout, before[k], got, self.cpu.params[k], twin_before[k],
                                                  self.twin.params[k], bounds, "%s, replica %d" % (what, k))
                worst = pm.merge(worst, w)
            else:
                assert np.array_equal(got, before[k].astype(np.float32)), (what, k)    # sat out: not a bit changes
        return worst

    def local_steps(self, check_updates=False):
        """One hadfl_local_steps call on each side (replica k runs E_k steps on its own).  With check_updates, every
        tensor's total update over the call is also held to the gross-mistake bounds of tests/parity_metrics.py (after
        the first step the two sides are no longer in one state; forced_steps is the sharp comparison)."""
        self.versions_after_forced = None
        if check_updates:
            before = self.cpu.params.copy()
        self.gpu.local_steps()
        self.cpu.local_steps()
        v, c = self.gpu.versions()
        assert v.tolist() == self.cpu.versions.tolist()
        assert c.tolist() == self.cpu.cursor.tolist()
        if not check_updates:
            return None
        worst = None
        for k in range(self.N):
            if self.cpu.versions[k] > 0:
                worst = pm.merge(worst, pm.assert_updates_fixed(self.layout, before[k], self.gpu.params(k), self.cpu.params[k],
                                                                pm.BOUNDS_FREE, "one call, replica %d" % k))
        return worst

    def forced_steps(self):
        """The sub-steps of one cycle (Algorithm 1's inner loop) one library call at a time.  Sub-step s is run by the
        replicas with E_k > s, exactly the groups one hadfl_local_steps call forms; before each, both sides are given
        one common state, so every step of every replica is compared on its own: each parameter tensor's update (and
        the batch-norm statistics') against the oracle's, in the three measures of tests/parity_metrics.py, or to what the
        oracle's twin allows.  Replicas that sit a sub-step out must not change by a bit.  -> that module's result dict."""
        steps = self.cpu.steps.copy()
        worst = None
        for s in range(int(steps.max())):
            sub = (steps > s).astype(np.int32)
            self.share_state()
            before = self.cpu.params.copy()
            twin_before = self._twin_start()
            self.twin.local_steps(steps=sub)
            self.gpu.set_steps(sub)
            self.gpu.local_steps()
            self.cpu.local_steps(steps=sub)
            v, c = self.gpu.versions()
            assert v.tolist() == sub.tolist() == self.cpu.versions.tolist()
            assert c.tolist() == self.cpu.cursor.tolist()
            worst = pm.merge(worst, self._check_updates(before, twin_before, sub > 0,
                                                        "sub-step %d (%d active)" % (s, int(sub.sum()))))
        self.gpu.set_steps(steps)
        # the library's counters hold the last sub-step's versions; the cycle's versions are the step counts
        self.cpu.versions[:] = steps
        self.versions_after_forced = steps
        return worst

    def select_aggregate(self, cycle, resync=True):
        if self.versions_after_forced is not None:
            import torch
            self.gpu.select(cycle, versions=torch.as_tensor(self.versions_after_forced, dtype=torch.int32).cuda())
        else:
            self.gpu.select(cycle)
        self.cpu.select(cycle)
        sel, flag, w = self.gpu.selected()
        assert sel.tolist() == self.cpu.selected.tolist()
        assert flag.tolist() == self.cpu.flag.tolist()
        self.gpu.aggregate(resync)
        self.cpu.aggregate(resync)
        return float(np.abs(self.gpu.params(-1).astype(np.float64) - self.cpu.agg).max())

    def close(self):
        self.gpu.close()
