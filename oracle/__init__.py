"""Python face of the HADFL oracle (TEST INFRASTRUCTURE, not the product).

The arithmetic lives in ``hadfl_oracle.c`` (plain fp64 loops); this module only
compiles it with gcc, marshals numpy arrays, and strings the calls of one
aggregation cycle together in the order of the paper's Algorithm 1:
local steps -> selection (Sec. 3.3) -> partial aggregation -> global sync.
Nothing here imports the GPU package.
"""
import ctypes
import os
import subprocess

import numpy as np

from . import nets

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hadfl_oracle.c")
_LIB = os.path.join(_HERE, "libhadfl_oracle.so")

c_i32p = ctypes.POINTER(ctypes.c_int32)
c_i64p = ctypes.POINTER(ctypes.c_int64)
c_u8p = ctypes.POINTER(ctypes.c_uint8)
c_u32p = ctypes.POINTER(ctypes.c_uint32)
c_f32p = ctypes.POINTER(ctypes.c_float)
c_f64p = ctypes.POINTER(ctypes.c_double)


def build(force=False):
    """Compile the oracle with gcc.  -ffp-contract=off keeps every fp64 operation separately rounded."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-fno-fast-math", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.hadfl_oracle_net_create.restype = ctypes.c_void_p
        L.hadfl_oracle_net_create.argtypes = [c_i32p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        L.hadfl_oracle_net_destroy.argtypes = [ctypes.c_void_p]
        L.hadfl_oracle_net_set_rounding.argtypes = [ctypes.c_void_p, ctypes.c_int]
        L.hadfl_oracle_net_m_train.restype = ctypes.c_int64
        L.hadfl_oracle_net_m_train.argtypes = [ctypes.c_void_p]
        L.hadfl_oracle_net_m_total.restype = ctypes.c_int64
        L.hadfl_oracle_net_m_total.argtypes = [ctypes.c_void_p]
        L.hadfl_oracle_net_n_out.argtypes = [ctypes.c_void_p]
        L.hadfl_oracle_net_layout.argtypes = [ctypes.c_void_p, c_i64p, ctypes.c_int]
        L.hadfl_oracle_round_bf16.restype = ctypes.c_double
        L.hadfl_oracle_round_bf16.argtypes = [ctypes.c_double]
        L.hadfl_oracle_loss_grad.restype = ctypes.c_double
        L.hadfl_oracle_loss_grad.argtypes = [ctypes.c_void_p, c_f64p, c_f32p, c_i32p, c_f64p, ctypes.c_int,
                                             ctypes.c_int, c_f64p, ctypes.c_int, c_f64p]
        L.hadfl_oracle_step_counts.argtypes = [c_i32p, ctypes.c_int, ctypes.c_int, ctypes.c_int, c_i32p]
        L.hadfl_oracle_local_steps.argtypes = [ctypes.c_void_p, ctypes.c_int, c_f64p, c_f64p, c_i64p, c_i32p,
                                               c_i32p, c_f32p, c_i32p, ctypes.c_int, ctypes.c_int,
                                               ctypes.c_double, ctypes.c_double, c_f64p]
        L.hadfl_oracle_philox4x32_10.argtypes = [c_u32p, c_u32p, c_u32p]
        L.hadfl_oracle_uniform.restype = ctypes.c_double
        L.hadfl_oracle_uniform.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint32]
        L.hadfl_oracle_exp.restype = ctypes.c_double
        L.hadfl_oracle_exp.argtypes = [ctypes.c_double]
        L.hadfl_oracle_select.argtypes = [c_f64p, c_u8p, ctypes.c_int, ctypes.c_int, ctypes.c_uint64,
                                          ctypes.c_uint64, c_i32p, c_u8p, c_f64p, c_f64p]
        L.hadfl_oracle_aggregate.argtypes = [c_f64p, ctypes.c_int, ctypes.c_int64, c_f64p, c_f64p]
        L.hadfl_oracle_aggregate_f32.argtypes = [c_f32p, ctypes.c_int64, ctypes.c_int, ctypes.c_int64,
                                                 c_f64p, c_f64p]
        L.hadfl_oracle_resync.argtypes = [c_f64p, ctypes.c_int, ctypes.c_int64, c_f64p]
        L.hadfl_oracle_predict.restype = ctypes.c_double
        L.hadfl_oracle_predict.argtypes = [c_f64p, c_f64p, ctypes.c_double, ctypes.c_double, ctypes.c_int,
                                           ctypes.c_int]
        L.hadfl_oracle_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _p(a, typ):
    return a.ctypes.data_as(typ)


KIND_NAMES = ("weight", "bias", "gamma", "beta", "running_mean", "running_var")


class Net:
    """A network description held by the C oracle."""

    def __init__(self, ops, in_shape, bf16=False):
        ops = np.ascontiguousarray(ops, dtype=np.int32).reshape(-1, 9)
        self.ops = ops
        self.in_shape = tuple(int(v) for v in in_shape)
        self.h = lib().hadfl_oracle_net_create(_p(ops, c_i32p), len(ops), *self.in_shape)
        if not self.h:
            raise ValueError("inconsistent network description")
        if bf16:
            lib().hadfl_oracle_net_set_rounding(self.h, 1)
        self.m_train = int(lib().hadfl_oracle_net_m_train(self.h))
        self.m_total = int(lib().hadfl_oracle_net_m_total(self.h))
        self.n_out = int(lib().hadfl_oracle_net_n_out(self.h))

    @classmethod
    def named(cls, name, bf16=False):
        fn, shape = nets.NETS[name]
        return cls(fn(), shape, bf16=bf16)

    def __del__(self):
        try:
            if self.h:
                lib().hadfl_oracle_net_destroy(self.h)
                self.h = None
        except Exception:
            pass

    def layout(self):
        """[(offset, count, kind_name, fan_in)] in parameter-vector order."""
        n = lib().hadfl_oracle_net_layout(self.h, None, 0)
        rows = np.zeros((n, 4), dtype=np.int64)
        lib().hadfl_oracle_net_layout(self.h, _p(rows, c_i64p), n)
        return [(int(o), int(c), KIND_NAMES[int(k)], int(f)) for o, c, k, f in rows]

    def loss_grad(self, params, x, y=None, target=None, update_stats=False, want_logits=False):
        """Loss and gradient of one batch.  params: fp64 [m_total] (running stats updated in place if asked)."""
        params = np.ascontiguousarray(params, dtype=np.float64)
        assert params.size == self.m_total
        x = np.ascontiguousarray(x, dtype=np.float32)
        B = x.shape[0]
        assert x.size == B * int(np.prod(self.in_shape))
        grad = np.zeros(self.m_train, dtype=np.float64)
        logits = np.zeros((B, self.n_out), dtype=np.float64) if want_logits else None
        if target is not None:
            t = np.ascontiguousarray(target, dtype=np.float64)
            loss = lib().hadfl_oracle_loss_grad(self.h, _p(params, c_f64p), _p(x, c_f32p), None, _p(t, c_f64p), 1,
                                                B, _p(grad, c_f64p), int(update_stats),
                                                _p(logits, c_f64p) if want_logits else None)
        else:
            yy = np.ascontiguousarray(y, dtype=np.int32)
            loss = lib().hadfl_oracle_loss_grad(self.h, _p(params, c_f64p), _p(x, c_f32p), _p(yy, c_i32p), None, 0,
                                                B, _p(grad, c_f64p), int(update_stats),
                                                _p(logits, c_f64p) if want_logits else None)
        if want_logits:
            return loss, grad, logits, params
        return loss, grad


def step_counts(ratio, t_sync=1, steps_per_unit=1):
    r = np.ascontiguousarray(ratio, dtype=np.int32)
    out = np.zeros_like(r)
    rc = lib().hadfl_oracle_step_counts(_p(r, c_i32p), len(r), t_sync, steps_per_unit, _p(out, c_i32p))
    if rc != 0:
        raise ValueError("ratios, t_sync and steps_per_unit must be positive")
    return out


def steps_from_times(times, e_warmup, quantum, t_sync=1, steps_per_unit=1):
    t = np.ascontiguousarray(times, dtype=np.float64)
    out = np.zeros(t.size, dtype=np.int32)
    L = lib()
    L.hadfl_oracle_steps_from_times.restype = ctypes.c_int
    L.hadfl_oracle_steps_from_times.argtypes = [c_f64p, ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_int,
                                                ctypes.c_int, c_i32p]
    rc = L.hadfl_oracle_steps_from_times(_p(t, c_f64p), int(t.size), int(e_warmup), float(quantum), int(t_sync),
                                         int(steps_per_unit), _p(out, c_i32p))
    if rc != 0:
        raise ValueError("times, quantum, e_warmup, t_sync and steps_per_unit must be positive and the counts at most 2^20")
    return out


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    o = np.zeros(4, dtype=np.uint32)
    lib().hadfl_oracle_philox4x32_10(_p(c, c_u32p), _p(k, c_u32p), _p(o, c_u32p))
    return o


def uniform(seed, cycle, t):
    return float(lib().hadfl_oracle_uniform(seed, cycle, t))


def exp_det(x):
    return float(lib().hadfl_oracle_exp(float(x)))


def select(versions, n_select, seed, cycle, avail=None):
    """Returns (selected[n_select] in draw order, flag[N], f[N], mu)."""
    v = np.ascontiguousarray(versions, dtype=np.float64)
    N = len(v)
    av = None if avail is None else np.ascontiguousarray(avail, dtype=np.uint8)
    sel = np.zeros(n_select, dtype=np.int32)
    flag = np.zeros(N, dtype=np.uint8)
    f = np.zeros(N, dtype=np.float64)
    mu = ctypes.c_double(0.0)
    rc = lib().hadfl_oracle_select(_p(v, c_f64p), None if av is None else _p(av, c_u8p), N, n_select,
                                   seed, cycle, _p(sel, c_i32p), _p(flag, c_u8p), _p(f, c_f64p),
                                   ctypes.byref(mu))
    if rc != 0:
        raise ValueError("fewer available replicas than n_select")
    return sel, flag, f, mu.value


def probabilities(versions, avail=None):
    """P(i) of the selection function for the given versions."""
    _, _, f, _ = select(versions, 1, 0, 0, avail)
    return f / f.sum()


def aggregation_weights(flag, f=None, mode=0):
    """mode 0: a_k = Flag_k / sum Flag (the paper's aggregate with the divisor read as the number selected).
    mode 1 (an extension, not in the paper): a_k = Flag_k f_k / sum Flag f."""
    flag = np.asarray(flag, dtype=np.float64)
    if mode == 0:
        return flag / flag.sum()
    w = flag * np.asarray(f, dtype=np.float64)
    return w / w.sum()


def aggregate(params, a):
    """params fp64 [N][M]; a [N] weights -> [M]."""
    P = np.ascontiguousarray(params, dtype=np.float64)
    a = np.ascontiguousarray(a, dtype=np.float64)
    N, M = P.shape
    out = np.zeros(M, dtype=np.float64)
    lib().hadfl_oracle_aggregate(_p(P, c_f64p), N, M, _p(a, c_f64p), _p(out, c_f64p))
    return out


def aggregate_f32(params_f32, a, m=None):
    """params fp32 [N][stride] (first m columns used); a [N] -> fp64 [m]."""
    P = params_f32
    assert P.dtype == np.float32 and P.flags.c_contiguous
    N, stride = P.shape
    m = stride if m is None else m
    a = np.ascontiguousarray(a, dtype=np.float64)
    out = np.zeros(m, dtype=np.float64)
    lib().hadfl_oracle_aggregate_f32(_p(P, c_f32p), stride, N, m, _p(a, c_f64p), _p(out, c_f64p))
    return out


class Predictor:
    """Brown double exponential smoothing of one replica's version series (Sec. 3.2)."""

    def __init__(self, alpha):
        self.alpha = float(alpha)
        self.s1 = ctypes.c_double(0.0)
        self.s2 = ctypes.c_double(0.0)
        self.first = True

    def update(self, v, m=1):
        out = lib().hadfl_oracle_predict(ctypes.byref(self.s1), ctypes.byref(self.s2), float(v), self.alpha,
                                         int(m), int(self.first))
        self.first = False
        return float(out)


class Cycle:
    """State of N replicas and the calls of one aggregation cycle, in the paper's order."""

    def __init__(self, net, n_replicas, n_select, w0, x, y, batch, lr, momentum, ratio, seed,
                 t_sync=1, steps_per_unit=1, weight_mode=0):
        self.net, self.N, self.n_select = net, int(n_replicas), int(n_select)
        self.batch, self.lr, self.momentum = int(batch), float(lr), float(momentum)
        self.seed, self.weight_mode = int(seed), int(weight_mode)
        w0 = np.asarray(w0, dtype=np.float64)
        assert w0.size == net.m_total
        # Algorithm 1, first line: every replica starts from the same model
        self.params = np.tile(w0, (self.N, 1))
        self.buf = np.zeros((self.N, net.m_train), dtype=np.float64)
        self.cursor = np.zeros(self.N, dtype=np.int64)
        self.x = None if x is None else np.ascontiguousarray(x, dtype=np.float32)
        self.y = None if y is None else np.ascontiguousarray(y, dtype=np.int32)
        self.n_samples = 0 if x is None else self.x.shape[1]
        self.steps = step_counts(ratio, t_sync, steps_per_unit)
        self.versions = np.zeros(self.N, dtype=np.int32)
        self.loss = np.zeros(self.N, dtype=np.float64)
        self.selected = self.flag = self.f = self.weights = self.agg = None

    def local_steps(self, steps=None):
        st = self.steps if steps is None else np.ascontiguousarray(steps, dtype=np.int32)
        lib().hadfl_oracle_local_steps(self.net.h, self.N, _p(self.params, c_f64p), _p(self.buf, c_f64p),
                                       _p(self.cursor, c_i64p), _p(st, c_i32p), _p(self.versions, c_i32p),
                                       _p(self.x, c_f32p), _p(self.y, c_i32p), self.n_samples, self.batch,
                                       self.lr, self.momentum, _p(self.loss, c_f64p))
        return self.versions.copy()

    def select(self, cycle, versions=None, avail=None):
        v = self.versions if versions is None else versions
        self.selected, self.flag, self.f, self.mu = select(v, self.n_select, self.seed, cycle, avail)
        self.weights = aggregation_weights(self.flag, self.f, self.weight_mode)
        return self.selected.copy()

    def aggregate(self, resync=True):
        self.agg = aggregate(self.params, self.weights)
        if resync:
            lib().hadfl_oracle_resync(_p(self.params, c_f64p), self.N, self.net.m_total, _p(self.agg, c_f64p))
        return self.agg

    # Sec. 3.3, last paragraph: devices divided into groups; an intra-group round selects and aggregates among the
    # members of one group and synchronises only them
    def select_group(self, cycle, members, n_select, versions=None):
        v = self.versions if versions is None else versions
        self.selected, self.flag, self.f, self.mu = select(v, n_select, self.seed, cycle, np.asarray(members, dtype=np.uint8))
        self.weights = aggregation_weights(self.flag, self.f, self.weight_mode)
        return self.selected.copy()

    def aggregate_group(self, members):
        self.agg = aggregate(self.params, self.weights)
        for k in range(self.N):
            if members[k]:
                self.params[k, :] = self.agg
        return self.agg

    def run_cycle(self, cycle, resync=True):
        self.local_steps()
        self.select(cycle)
        return self.aggregate(resync)
