"""Thin ctypes binding over libhadfl.so -- argument marshalling only; every step of the cycle runs in the
library's HIP kernels.  PyTorch supplies device memory and the stream.  There is no fallback: if the library
is not built, loading raises."""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhadfl.so")

OK, EINVAL, ENOMEM, EDEVICE, ESTATE, EUNSUPPORTED = range(6)
STATUS_NAMES = ("HADFL_OK", "HADFL_EINVAL", "HADFL_ENOMEM", "HADFL_EDEVICE", "HADFL_ESTATE", "HADFL_EUNSUPPORTED")
NET_MLP, NET_CNN2, NET_RESNET18, NET_VGG16, NET_NONE, NET_CUSTOM = range(6)
NET_IDS = {"mlp": NET_MLP, "cnn2": NET_CNN2, "resnet18": NET_RESNET18, "vgg16": NET_VGG16, "none": NET_NONE,
           "custom": NET_CUSTOM}
KIND_NAMES = ("weight", "bias", "gamma", "beta", "running_mean", "running_var")


class HadflOp(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("type", "in0", "in1", "k", "stride", "pad", "cout", "bias")]


class HadflConfig(ctypes.Structure):
    _fields_ = [("n_replicas", ctypes.c_int32), ("n_select", ctypes.c_int32), ("net", ctypes.c_int32),
                ("bf16", ctypes.c_int32), ("batch", ctypes.c_int32), ("n_samples", ctypes.c_int32),
                ("in_dim", ctypes.c_int32 * 3), ("n_classes", ctypes.c_int32), ("lr", ctypes.c_float),
                ("momentum", ctypes.c_float), ("t_sync", ctypes.c_int32), ("steps_per_unit", ctypes.c_int32),
                ("weight_mode", ctypes.c_int32), ("n_custom_ops", ctypes.c_int32), ("seed", ctypes.c_uint64),
                ("m_none", ctypes.c_int64), ("custom_ops", ctypes.POINTER(HadflOp))]


class HadflTensorInfo(ctypes.Structure):
    _fields_ = [("offset", ctypes.c_int64), ("count", ctypes.c_int64), ("kind", ctypes.c_int32),
                ("fan_in", ctypes.c_int32)]


class HadflKernelTime(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 48), ("launches", ctypes.c_int64), ("total_ms", ctypes.c_double),
                ("flops", ctypes.c_double), ("bytes", ctypes.c_double)]


OPT_SIDE_STREAM, OPT_TILE_HINT = 0, 1

EXPORTS = ("hadfl_param_count", "hadfl_param_layout", "hadfl_workspace_bytes", "hadfl_init_replicas",
           "hadfl_local_steps", "hadfl_select", "hadfl_aggregate", "hadfl_step_counts", "hadfl_steps_from_times",
           "hadfl_set_lr", "hadfl_set_steps", "hadfl_set_params", "hadfl_get_momentum", "hadfl_set_momentum",
           "hadfl_set_option", "hadfl_select_static",
           "hadfl_select_group", "hadfl_aggregate_group", "hadfl_predict_versions",
           "hadfl_select_real", "hadfl_get_predicted", "hadfl_get_steps", "hadfl_get_versions",
           "hadfl_get_selected", "hadfl_get_params", "hadfl_get_losses", "hadfl_profile_enable",
           "hadfl_profile_read", "hadfl_last_error", "hadfl_destroy")

_lib = None


class HadflError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("%s: %s" % (STATUS_NAMES[status] if 0 <= status < 6 else status, text))
        self.status = status


def lib():
    """Loads libhadfl.so (built in-tree by paper_2111_08274_amd.build).  Raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libhadfl.so is not built: run `python -m paper_2111_08274_amd.build`")
        # PyTorch ships its own HIP runtime; load it first so the library binds to the same runtime instance
        # that owns the tensors and streams handed to it (two runtimes in one process do not share devices).
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64p = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_int64)
        cfgp = ctypes.POINTER(HadflConfig)
        L.hadfl_param_count.argtypes = [cfgp, i64p, i64p, i64p]
        L.hadfl_param_layout.argtypes = [cfgp, ctypes.POINTER(HadflTensorInfo), i32, ctypes.POINTER(i32)]
        L.hadfl_workspace_bytes.argtypes = [cfgp, ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(ctypes.c_size_t)]
        L.hadfl_init_replicas.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, ctypes.POINTER(vp)]
        L.hadfl_local_steps.argtypes = [vp]
        L.hadfl_select.argtypes = [vp, vp, vp, ctypes.c_uint64]
        L.hadfl_aggregate.argtypes = [vp, i32]
        L.hadfl_set_steps.argtypes = [vp, vp]
        L.hadfl_step_counts.argtypes = [vp, i32, i32, i32, vp]
        L.hadfl_steps_from_times.argtypes = [vp, i32, i32, ctypes.c_double, i32, i32, vp]
        L.hadfl_set_params.argtypes = [vp, i32, vp, ctypes.c_size_t]
        L.hadfl_get_momentum.argtypes = [vp, i32, vp, ctypes.c_size_t]
        L.hadfl_set_momentum.argtypes = [vp, i32, vp, ctypes.c_size_t]
        L.hadfl_set_option.argtypes = [vp, i32, i32]
        L.hadfl_select_static.argtypes = [vp, vp, i32, i32, i32, ctypes.c_uint64, ctypes.c_uint64, vp, vp, vp, vp]
        L.hadfl_set_lr.argtypes = [vp, ctypes.c_float]
        L.hadfl_select_group.argtypes = [vp, vp, vp, i32, ctypes.c_uint64]
        L.hadfl_aggregate_group.argtypes = [vp, vp]
        L.hadfl_predict_versions.argtypes = [vp, vp, ctypes.c_double, i32]
        L.hadfl_select_real.argtypes = [vp, vp, vp, ctypes.c_uint64]
        L.hadfl_get_predicted.argtypes = [vp, vp]
        L.hadfl_get_steps.argtypes = [vp, vp]
        L.hadfl_get_versions.argtypes = [vp, vp, vp]
        L.hadfl_get_selected.argtypes = [vp, vp, ctypes.POINTER(i32), vp, vp]
        L.hadfl_get_params.argtypes = [vp, i32, vp, ctypes.c_size_t]
        L.hadfl_get_losses.argtypes = [vp, vp]
        L.hadfl_profile_enable.argtypes = [vp, i32]
        L.hadfl_profile_read.argtypes = [vp, ctypes.POINTER(HadflKernelTime), i32, ctypes.POINTER(i32)]
        L.hadfl_last_error.argtypes = [vp]
        L.hadfl_last_error.restype = ctypes.c_char_p
        L.hadfl_destroy.argtypes = [vp]
        L.hadfl_destroy.restype = None
        for name in EXPORTS:
            if name not in ("hadfl_last_error", "hadfl_destroy"):
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def make_config(n_replicas, n_select, net="none", bf16=0, batch=1, n_samples=1, in_shape=(1, 1, 1), n_classes=10,
                lr=0.01, momentum=0.0, t_sync=1, steps_per_unit=1, weight_mode=0, seed=2021, m_none=0,
                custom_ops=None):
    """custom_ops: rows (type, in0, in1, k, stride, pad, cout, bias)."""
    c = HadflConfig()
    c.n_replicas, c.n_select = int(n_replicas), int(n_select)
    c.net = NET_IDS[net] if isinstance(net, str) else int(net)
    c.bf16, c.batch, c.n_samples = int(bf16), int(batch), int(n_samples)
    c.in_dim[0], c.in_dim[1], c.in_dim[2] = (int(v) for v in in_shape)
    c.n_classes, c.lr, c.momentum = int(n_classes), float(lr), float(momentum)
    c.t_sync, c.steps_per_unit, c.weight_mode = int(t_sync), int(steps_per_unit), int(weight_mode)
    c.seed, c.m_none = int(seed), int(m_none)
    c._keep = None
    if custom_ops is not None:
        rows = np.asarray(custom_ops, dtype=np.int32).reshape(-1, 8)
        arr = (HadflOp * len(rows))()
        for i, r in enumerate(rows):
            arr[i] = HadflOp(*[int(v) for v in r])
        c._keep = arr
        c.custom_ops = ctypes.cast(arr, ctypes.POINTER(HadflOp))
        c.n_custom_ops = len(rows)
    return c


def _check(status, ctx=None):
    if status != OK:
        raise HadflError(status, lib().hadfl_last_error(ctx).decode())


def param_count(cfg):
    a, b, c = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    _check(lib().hadfl_param_count(ctypes.byref(cfg), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
    return a.value, b.value, c.value


def param_layout(cfg):
    n = ctypes.c_int32()
    _check(lib().hadfl_param_layout(ctypes.byref(cfg), None, 0, ctypes.byref(n)))
    rows = (HadflTensorInfo * n.value)()
    _check(lib().hadfl_param_layout(ctypes.byref(cfg), rows, n.value, ctypes.byref(n)))
    return [(r.offset, r.count, KIND_NAMES[r.kind], r.fan_in) for r in rows]


def workspace_bytes(cfg):
    a, b = ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().hadfl_workspace_bytes(ctypes.byref(cfg), ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value


def _np_ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def step_counts(ratio, t_sync=1, steps_per_unit=1):
    """The step-count rule from computing-power ratios (host only) -> int32[n]."""
    r = np.ascontiguousarray(ratio, dtype=np.int32)
    out = np.zeros(r.size, dtype=np.int32)
    _check(lib().hadfl_step_counts(_np_ptr(r), int(r.size), int(t_sync), int(steps_per_unit), _np_ptr(out)))
    return out


def steps_from_times(times, e_warmup, quantum, t_sync=1, steps_per_unit=1):
    """Step counts from measured warm-up times (host only) -> int32[n]."""
    t = np.ascontiguousarray(times, dtype=np.float64)
    out = np.zeros(t.size, dtype=np.int32)
    _check(lib().hadfl_steps_from_times(_np_ptr(t), int(t.size), int(e_warmup), float(quantum), int(t_sync),
                                        int(steps_per_unit), _np_ptr(out)))
    return out


def select_static(versions, n_select, seed, cycle, selected, flag, weights, avail=None, weight_mode=0, stream=None):
    """hadfl_select_static on torch device tensors the CALLER has allocated: versions int32[n], avail uint8[n] or None;
    outputs selected int32[n_select], flag uint8[n], weights float32[n].  The library allocates nothing."""
    import torch
    n = versions.numel()
    assert versions.dtype == torch.int32 and versions.is_cuda and versions.is_contiguous()
    assert selected.dtype == torch.int32 and selected.numel() >= n_select and selected.is_cuda
    assert flag.dtype == torch.uint8 and flag.numel() >= n and flag.is_cuda
    assert weights.dtype == torch.float32 and weights.numel() >= n and weights.is_cuda
    if avail is not None:
        assert avail.dtype == torch.uint8 and avail.numel() == n and avail.is_cuda
    st = (torch.cuda.current_stream() if stream is None else stream).cuda_stream
    _check(lib().hadfl_select_static(versions.data_ptr(), avail.data_ptr() if avail is not None else None, int(n),
                                     int(n_select), int(weight_mode), int(seed), int(cycle), selected.data_ptr(),
                                     flag.data_ptr(), weights.data_ptr(), st))


class Context:
    """One set of replicas on the current torch device.  Holds the torch tensors the library works in."""

    def __init__(self, cfg, ratio, w0=None, x=None, y=None, replicas=None, stream=None, options=None):
        import torch
        self.cfg = cfg
        self.m_train, self.m_total, self.row_stride = param_count(cfg)
        pb, sb = workspace_bytes(cfg)
        dev = torch.device("cuda", torch.cuda.current_device())
        if replicas is None:
            replicas = torch.empty(pb // 4, dtype=torch.float32, device=dev)
        assert replicas.numel() * 4 >= pb and replicas.is_contiguous()
        self.replicas = replicas
        self.scratch = torch.empty(sb, dtype=torch.uint8, device=dev)
        self.w0 = None if w0 is None else torch.as_tensor(w0, dtype=torch.float32).to(dev).contiguous()
        self.x = None if x is None else (x if hasattr(x, "data_ptr") else torch.as_tensor(x)).to(dev).contiguous()
        self.y = None if y is None else (y if hasattr(y, "data_ptr") else torch.as_tensor(y)).to(dev).to(torch.int32).contiguous()
        if self.w0 is not None:
            assert self.w0.numel() == self.m_total
        self.stream = torch.cuda.current_stream() if stream is None else stream
        ratio = np.ascontiguousarray(ratio, dtype=np.int32)
        assert len(ratio) == cfg.n_replicas
        h = ctypes.c_void_p()
        torch.cuda.synchronize()
        _check(lib().hadfl_init_replicas(ctypes.byref(cfg), self.w0.data_ptr() if self.w0 is not None else None,
                                         self.replicas.data_ptr(), self.scratch.data_ptr(),
                                         self.x.data_ptr() if self.x is not None else None,
                                         self.y.data_ptr() if self.y is not None else None,
                                         _np_ptr(ratio), self.stream.cuda_stream, ctypes.byref(h)))
        self.h = h
        for opt, value in (options or {}).items():
            self.set_option(opt, value)

    def set_option(self, option, value):
        _check(lib().hadfl_set_option(self.h, int(option), int(value)), self.h)

    def set_params(self, replica, values):
        v = np.ascontiguousarray(values, dtype=np.float32)
        _check(lib().hadfl_set_params(self.h, int(replica), _np_ptr(v), v.size), self.h)

    def momentum(self, replica, n=None):
        out = np.zeros(self.m_train if n is None else n, dtype=np.float32)
        _check(lib().hadfl_get_momentum(self.h, int(replica), _np_ptr(out), out.size), self.h)
        return out

    def set_momentum(self, replica, values):
        v = np.ascontiguousarray(values, dtype=np.float32)
        _check(lib().hadfl_set_momentum(self.h, int(replica), _np_ptr(v), v.size), self.h)

    def close(self):
        if getattr(self, "h", None):
            lib().hadfl_destroy(self.h)
            self.h = None

    def __del__(self):
        # at interpreter shutdown module globals may already be gone; the process is ending anyway
        try:
            self.close()
        except TypeError:
            pass

    def local_steps(self):
        _check(lib().hadfl_local_steps(self.h), self.h)

    def select(self, cycle, versions=None, avail=None):
        """versions: torch int32 device tensor or None; avail: host array of bytes or None."""
        av = None if avail is None else np.ascontiguousarray(avail, dtype=np.uint8)
        if versions is not None:
            assert versions.dtype.__str__() == "torch.int32" and versions.is_cuda and versions.numel() == self.cfg.n_replicas
        _check(lib().hadfl_select(self.h, versions.data_ptr() if versions is not None else None,
                                  _np_ptr(av) if av is not None else None, int(cycle)), self.h)

    def set_lr(self, lr):
        _check(lib().hadfl_set_lr(self.h, float(lr)), self.h)

    def set_steps(self, steps):
        st = np.ascontiguousarray(steps, dtype=np.int32)
        assert st.size == self.cfg.n_replicas
        _check(lib().hadfl_set_steps(self.h, _np_ptr(st)), self.h)

    def predict_versions(self, alpha, horizon=1, versions=None):
        """versions: torch int32 device tensor or None (the counters of the last local_steps)."""
        if versions is not None:
            assert versions.dtype.__str__() == "torch.int32" and versions.is_cuda and versions.numel() == self.cfg.n_replicas
        _check(lib().hadfl_predict_versions(self.h, versions.data_ptr() if versions is not None else None,
                                            float(alpha), int(horizon)), self.h)

    def select_real(self, cycle, versions=None, avail=None):
        """versions: torch float64 device tensor or None (the forecast of predict_versions)."""
        av = None if avail is None else np.ascontiguousarray(avail, dtype=np.uint8)
        if versions is not None:
            assert versions.dtype.__str__() == "torch.float64" and versions.is_cuda and versions.numel() == self.cfg.n_replicas
        _check(lib().hadfl_select_real(self.h, versions.data_ptr() if versions is not None else None,
                                       _np_ptr(av) if av is not None else None, int(cycle)), self.h)

    def predicted(self):
        out = np.zeros(self.cfg.n_replicas, dtype=np.float64)
        _check(lib().hadfl_get_predicted(self.h, _np_ptr(out)), self.h)
        return out

    def select_group(self, cycle, members, n_select, versions=None):
        mb = np.ascontiguousarray(members, dtype=np.uint8)
        assert mb.size == self.cfg.n_replicas
        if versions is not None:
            assert versions.dtype.__str__() == "torch.int32" and versions.is_cuda and versions.numel() == self.cfg.n_replicas
        _check(lib().hadfl_select_group(self.h, versions.data_ptr() if versions is not None else None, _np_ptr(mb),
                                        int(n_select), int(cycle)), self.h)

    def aggregate_group(self, members):
        mb = np.ascontiguousarray(members, dtype=np.uint8)
        assert mb.size == self.cfg.n_replicas
        _check(lib().hadfl_aggregate_group(self.h, _np_ptr(mb)), self.h)

    def aggregate(self, resync=True):
        _check(lib().hadfl_aggregate(self.h, int(bool(resync))), self.h)

    def steps(self):
        out = np.zeros(self.cfg.n_replicas, dtype=np.int32)
        _check(lib().hadfl_get_steps(self.h, _np_ptr(out)), self.h)
        return out

    def versions(self):
        v = np.zeros(self.cfg.n_replicas, dtype=np.int32)
        c = np.zeros(self.cfg.n_replicas, dtype=np.int64)
        _check(lib().hadfl_get_versions(self.h, _np_ptr(v), _np_ptr(c)), self.h)
        return v, c

    def selected(self):
        sel = np.zeros(self.cfg.n_select, dtype=np.int32)
        cnt = ctypes.c_int32()
        flag = np.zeros(self.cfg.n_replicas, dtype=np.uint8)
        w = np.zeros(self.cfg.n_replicas, dtype=np.float32)
        _check(lib().hadfl_get_selected(self.h, _np_ptr(sel), ctypes.byref(cnt), _np_ptr(flag), _np_ptr(w)), self.h)
        return sel[:cnt.value], flag, w

    def params(self, replica, n=None):
        n = self.m_total if n is None else n
        out = np.zeros(n, dtype=np.float32)
        _check(lib().hadfl_get_params(self.h, int(replica), _np_ptr(out), n), self.h)
        return out

    def losses(self):
        out = np.zeros(self.cfg.n_replicas, dtype=np.float32)
        _check(lib().hadfl_get_losses(self.h, _np_ptr(out)), self.h)
        return out

    def profile(self, on):
        _check(lib().hadfl_profile_enable(self.h, int(on)), self.h)

    def profile_read(self):
        n = ctypes.c_int32()
        rows = (HadflKernelTime * 4096)()
        _check(lib().hadfl_profile_read(self.h, rows, 4096, ctypes.byref(n)), self.h)
        return {rows[i].name.decode(): dict(launches=rows[i].launches, ms=rows[i].total_ms, flops=rows[i].flops,
                                            bytes=rows[i].bytes) for i in range(min(n.value, 4096))}
