"""Seeded synthetic inputs shaped like the paper's workloads (Sec. 4.1: 32x32 colour images,
10 classes, per-device batch 64) and the configurations they are used in.

This module holds no arithmetic of the method: it only draws arrays.  Both the GPU
path and the CPU oracle are fed from here; neither generates its own inputs.
"""
import numpy as np

# The five workloads.  `ratio` None means "drawn uniformly from ratio_range with seed 200+c".
CONFIGS = {
    1: dict(name="mlp-n4", net="mlp", n_replicas=4, n_select=2, n_samples=512, batch=32, lr=0.05,
            momentum=0.0, ratio=[1, 2, 3, 4], cycles=5, bf16=0, in_shape=(1, 1, 784)),
    # workload 2 states no learning rate: the paper's (Sec. 4.1, 0.01 after the warm-up)
    2: dict(name="cnn2-n8", net="cnn2", n_replicas=8, n_select=4, n_samples=2048, batch=64, lr=0.01,
            momentum=0.9, ratio=[1, 1, 2, 2, 3, 3, 4, 4], cycles=10, bf16=0, in_shape=(32, 32, 3)),
    3: dict(name="resnet18-n16", net="resnet18", n_replicas=16, n_select=4, n_samples=4096, batch=64,
            lr=0.1, momentum=0.9, ratio=None, ratio_range=(1, 4), cycles=20, bf16=0,
            in_shape=(32, 32, 3), dirichlet=0.5),
    4: dict(name="agg-stress-n64", net="none", n_replicas=64, n_select=8, m=11173962, cycles=1000,
            version_range=(0, 50), std=0.02),
    5: dict(name="vgg16-bf16-n32", net="vgg16", n_replicas=32, n_select=8, n_samples=4096, batch=128,
            lr=0.01, momentum=0.9, ratio=None, ratio_range=(1, 8), cycles=20, bf16=1,
            in_shape=(32, 32, 3), dirichlet=0.3),
}
SELECT_SEED = 2021


def he_normal_init(layout, seed=0):
    """layout: [(offset, count, kind, fan_in)] in vector order; kind in weight/bias/gamma/beta/
    running_mean/running_var.  Weights ~ N(0, 2/fan_in); biases, beta, running mean 0; gamma, running var 1."""
    rng = np.random.default_rng(seed)
    total = max(o + c for o, c, _, _ in layout)
    w = np.zeros(total, dtype=np.float32)
    for off, cnt, kind, fan_in in layout:
        if kind == "weight":
            w[off:off + cnt] = rng.standard_normal(cnt, dtype=np.float32) * np.float32(np.sqrt(2.0 / fan_in))
        elif kind in ("gamma", "running_var"):
            w[off:off + cnt] = 1.0
    return w


def balanced_labels(n_replicas, n_samples, n_classes, rng):
    y = np.empty((n_replicas, n_samples), dtype=np.int32)
    for k in range(n_replicas):
        y[k] = rng.permutation(np.arange(n_samples, dtype=np.int32) % n_classes)
    return y


def dirichlet_labels(n_replicas, n_samples, n_classes, alpha, rng):
    """Non-IID label split: each replica's class proportions ~ Dirichlet(alpha), counts rounded
    (largest remainder) to n_samples, order shuffled."""
    y = np.empty((n_replicas, n_samples), dtype=np.int32)
    for k in range(n_replicas):
        p = rng.dirichlet(np.full(n_classes, alpha))
        cnt = np.floor(p * n_samples).astype(np.int64)
        rem = n_samples - cnt.sum()
        order = np.argsort(-(p * n_samples - cnt), kind="stable")
        cnt[order[:rem]] += 1
        y[k] = rng.permutation(np.repeat(np.arange(n_classes, dtype=np.int32), cnt))
    return y


def class_gaussian_vectors(n_replicas, n_samples, dim, n_classes=10, seed=101, mean_std=0.5):
    """x ~ N(mu_c, I), mu_c ~ N(0, mean_std^2) per dimension; balanced classes.  -> x [N][n][dim], y [N][n]."""
    rng = np.random.default_rng(seed)
    mu = rng.standard_normal((n_classes, dim), dtype=np.float32) * np.float32(mean_std)
    y = balanced_labels(n_replicas, n_samples, n_classes, rng)
    x = rng.standard_normal((n_replicas, n_samples, dim), dtype=np.float32)
    x += mu[y]
    return x, y


def class_shift_images(n_replicas, n_samples, shape=(32, 32, 3), n_classes=10, seed=102, shift=0.3,
                       dirichlet=None):
    """x = z + shift*m_c with z ~ N(0,1) and one fixed m_c ~ N(0,1) image per class.
    -> x [N][n][H][W][C] (channels last), y [N][n]."""
    rng = np.random.default_rng(seed)
    m = rng.standard_normal((n_classes,) + tuple(shape), dtype=np.float32)
    if dirichlet is None:
        y = balanced_labels(n_replicas, n_samples, n_classes, rng)
    else:
        y = dirichlet_labels(n_replicas, n_samples, n_classes, dirichlet, rng)
    x = np.empty((n_replicas, n_samples) + tuple(shape), dtype=np.float32)
    for k in range(n_replicas):
        x[k] = rng.standard_normal((n_samples,) + tuple(shape), dtype=np.float32)
        x[k] += np.float32(shift) * m[y[k]]
    return x, y


def compute_ratios(n_replicas, lo, hi, seed):
    return np.random.default_rng(seed).integers(lo, hi + 1, size=n_replicas).astype(np.int32)


def versions_uniform(n_replicas, lo, hi, seed):
    return np.random.default_rng(seed).integers(lo, hi + 1, size=n_replicas).astype(np.int32)


def replica_rows_gaussian(n_replicas, m, std, seed, row_stride=None):
    """Independent N(0, std^2) parameter rows for the aggregation stress workload -> fp32 [N][row_stride]
    (columns beyond m are zero)."""
    row_stride = m if row_stride is None else row_stride
    out = np.zeros((n_replicas, row_stride), dtype=np.float32)
    for k in range(n_replicas):
        rng = np.random.default_rng([seed, k])
        out[k, :m] = rng.standard_normal(m, dtype=np.float32) * np.float32(std)
    return out


def config_inputs(c, n_replicas=None, n_samples=None):
    """Data, labels and ratios of training workload c (1, 2, 3 or 5), optionally cut down in replicas/samples."""
    cfg = dict(CONFIGS[c])
    N = cfg["n_replicas"] if n_replicas is None else n_replicas
    n = cfg["n_samples"] if n_samples is None else n_samples
    if cfg["net"] == "mlp":
        x, y = class_gaussian_vectors(N, n, 784, 10, seed=100 + c)
    else:
        x, y = class_shift_images(N, n, cfg["in_shape"], 10, seed=100 + c, shift=0.3,
                                  dirichlet=cfg.get("dirichlet"))
    if cfg["ratio"] is None:
        ratio = compute_ratios(cfg["n_replicas"], *cfg["ratio_range"], seed=200 + c)[:N]
    else:
        ratio = np.asarray(cfg["ratio"], dtype=np.int32)[:N]
    cfg.update(n_replicas=N, n_samples=n, ratio=ratio)
    return cfg, x, y
