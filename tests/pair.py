"""Runs the oracle and the HIP library side by side on the same seeded inputs (helper for the GPU parity tests)."""
import numpy as np

import oracle
from paper_2111_08274_amd import hadfl, synth


def oracle_ops_to_custom(ops):
    """Oracle op rows (type,in0,in1,out,k,stride,pad,cout,bias) -> library rows (type,in0,in1,k,stride,pad,cout,bias)."""
    return np.asarray(ops, dtype=np.int32)[:, [0, 1, 2, 4, 5, 6, 7, 8]]


class Pair:
    def __init__(self, ops, in_shape, n_replicas, n_select, x, y, batch, lr, momentum, ratio, net_name=None,
                 seed=synth.SELECT_SEED, t_sync=1, init_seed=0, weight_mode=0, bf16=False):
        self.net = oracle.Net(ops, in_shape, bf16=bf16)
        n_classes = self.net.n_out
        kw = dict(batch=batch, n_samples=x.shape[1], in_shape=in_shape, n_classes=n_classes, lr=lr,
                  momentum=momentum, t_sync=t_sync, seed=seed, weight_mode=weight_mode, bf16=int(bf16))
        if net_name is None:
            self.hc = hadfl.make_config(n_replicas, n_select, net="custom", custom_ops=oracle_ops_to_custom(ops), **kw)
        else:
            self.hc = hadfl.make_config(n_replicas, n_select, net=net_name, **kw)
        layout = hadfl.param_layout(self.hc)
        assert layout == self.net.layout()
        self.w0 = synth.he_normal_init(layout, seed=init_seed)
        self.gpu = hadfl.Context(self.hc, ratio, w0=self.w0, x=x, y=y)
        self.cpu = oracle.Cycle(self.net, n_replicas, n_select, self.w0, x.reshape(n_replicas, x.shape[1], -1), y,
                                batch, lr, momentum, ratio, seed=seed, t_sync=t_sync, weight_mode=weight_mode)
        self.N = n_replicas

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

    def local_steps(self):
        self.gpu.local_steps()
        self.cpu.local_steps()
        v, c = self.gpu.versions()
        assert v.tolist() == self.cpu.versions.tolist()
        assert c.tolist() == self.cpu.cursor.tolist()

    def select_aggregate(self, cycle, resync=True):
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
