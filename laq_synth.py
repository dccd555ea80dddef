"""Seeded synthetic inputs for the LAQ workloads.

Input generation only: nothing here performs any step of the method.  Both the
HIP path and the CPU reference take their inputs from this module so that they
see identical bytes.  Host arrays come from numpy's counter-based Philox
generator keyed by ``SEED0 + workload number``.

The paper's experiments use MNIST (60000 x 784, about 80 % zero pixels, 10
classes, split uniformly over M = 10 workers).  That data is not available
here; these generators produce stand-ins of the same shapes and sparsity.
"""
from dataclasses import dataclass, field

import numpy as np

SEED0 = 190907588

KIND_NONE, KIND_BINLOG, KIND_SOFTMAX, KIND_MLP = 0, 1, 2, 3


@dataclass
class Workload:
    name: str
    cfg: int
    kind: int
    M: int
    N_m: int
    dims: tuple          # binlog: (F,), softmax: (F, C), mlp: layer widths
    p: int
    b: int
    D: int = 10
    xi: float = 0.8 / 10
    t_bar: int = 100
    alpha: float = 0.01
    lam: float = 0.01
    iterations: int = 100
    extra: dict = field(default_factory=dict)


def _rng(cfg, stream=0):
    return np.random.Generator(np.random.Philox(key=[SEED0 + cfg, stream]))


def mlp_param_count(dims):
    return sum(dims[i] * dims[i + 1] + dims[i + 1] for i in range(len(dims) - 1))


def pad4(n):
    return (n + 3) // 4 * 4


def workload(cfg, scale=1.0):
    """The five workloads; scale < 1 shrinks N_m (and p for cfg 4) for tests."""
    if cfg == 1:
        return Workload("cfg1_binlog_p50", 1, KIND_BINLOG, 10, max(4, int(100 * scale)), (50,), 50,
                        b=3, alpha=0.01, iterations=200)
    if cfg == 2:
        return Workload("cfg2_softmax_785x10", 2, KIND_SOFTMAX, 10, max(8, int(6000 * scale)),
                        (785, 10), 7850, b=3, alpha=0.02, iterations=1000)
    if cfg == 3:
        dims = (784, 200, 10)
        return Workload("cfg3_mlp_784_200_10", 3, KIND_MLP, 10, max(8, int(6000 * scale)), dims,
                        mlp_param_count(dims), b=8, alpha=0.005, iterations=500)
    if cfg == 4:
        p = max(64, int((1 << 24) * scale))
        return Workload("cfg4_synthetic_grads", 4, KIND_NONE, 64, 0, (), p, b=4, t_bar=50,
                        alpha=0.01, iterations=50)
    if cfg == 5:
        dims = (784, 2048, 2048, 10)
        return Workload("cfg5_mlp_784_2048_2048_10", 5, KIND_MLP, 32, max(8, int(8192 * scale)),
                        dims, mlp_param_count(dims), b=4, alpha=0.002, iterations=300)
    raise ValueError(cfg)


def sparse_uniform_features(rng, shape):
    """Each entry 0 with probability 0.8, else Uniform[0,1)."""
    x = rng.random(shape, dtype=np.float32)
    keep = rng.random(shape, dtype=np.float32) < np.float32(0.2)
    return np.where(keep, x, np.float32(0)).astype(np.float32)


def model_inputs(w):
    """Host inputs of a model workload: X[M][N_m][ldx] float32 (rows padded with
    zeros to a multiple of 4 floats), y[M][N_m] int32, theta0[p] float32."""
    rng = _rng(w.cfg)
    M, N_m = w.M, w.N_m
    if w.kind == KIND_BINLOG:
        F = w.dims[0]
        ldx = pad4(F)
        X = np.zeros((M, N_m, ldx), np.float32)
        X[:, :, :F] = rng.standard_normal((M, N_m, F), dtype=np.float32)
        theta_star = rng.standard_normal(F, dtype=np.float32)
        y = np.sign(X[:, :, :F].astype(np.float64) @ theta_star.astype(np.float64))
        y[y == 0] = 1
        flip = rng.random((M, N_m)) < 0.05
        y = np.where(flip, -y, y).astype(np.int32)
        theta0 = np.zeros(F, np.float32)
        return X, y, theta0
    if w.kind == KIND_SOFTMAX:
        F, Cn = w.dims
        ldx = pad4(F)
        X = np.zeros((M, N_m, ldx), np.float32)
        X[:, :, :F - 1] = sparse_uniform_features(rng, (M, N_m, F - 1))
        X[:, :, F - 1] = 1.0                       # bias column
        y = rng.integers(0, Cn, (M, N_m)).astype(np.int32)
        theta0 = np.zeros(F * Cn, np.float32)
        return X, y, theta0
    if w.kind == KIND_MLP:
        F, Cn = w.dims[0], w.dims[-1]
        ldx = pad4(F)
        X = np.zeros((M, N_m, ldx), np.float32)
        X[:, :, :F] = sparse_uniform_features(rng, (M, N_m, F))
        y = rng.integers(0, Cn, (M, N_m)).astype(np.int32)
        parts = []
        for i in range(len(w.dims) - 1):
            fan_in, out = w.dims[i], w.dims[i + 1]
            W = rng.standard_normal((fan_in, out), dtype=np.float32) / np.float32(np.sqrt(fan_in))
            parts += [W.reshape(-1).astype(np.float32), np.zeros(out, np.float32)]
        theta0 = np.concatenate(parts)
        assert theta0.size == w.p
        return X, y, theta0
    raise ValueError("workload has no model")


def heterogeneous(w, X, y, level):
    """Copies of a model workload's (X, y) with the shards made unlike each other; level in [0, 1],
    0 returns the inputs unchanged.  Worker m's features (not a bias column) are scaled by
    10^(-level * m / (M - 1)), so the workers' smoothness constants spread over 10^(2 level); and each
    label is, with probability level, replaced by the class m mod C (label skew).  Stands in for the
    heterogeneity sweep announced at the end of Sec. 4, whose recipe the paper does not print."""
    if not 0.0 <= level <= 1.0:
        raise ValueError("level must lie in [0, 1]")
    if level == 0.0:
        return X, y
    rng = _rng(w.cfg, stream=500)
    M = w.M
    F = w.dims[0] - (1 if w.kind == KIND_SOFTMAX else 0)      # the softmax workload's last column is the bias
    Xh, yh = X.copy(), y.copy()
    if w.kind != KIND_BINLOG:
        Cn = w.dims[-1]
        swap = rng.random(y.shape) < level
    for m in range(M):
        Xh[m, :, :F] *= np.float32(10.0 ** (-level * m / max(M - 1, 1)))
        if w.kind != KIND_BINLOG:
            yh[m][swap[m]] = m % Cn
    return Xh, yh


def minibatch_indices(w, B, iteration):
    """Sample indices idx[M][B] (int32, into each worker's own shard, without repeats inside
    a batch) for one stochastic iteration; a function of (workload, B, iteration) only."""
    rng = _rng(w.cfg, stream=1000 + iteration)
    return np.stack([rng.permutation(w.N_m)[:B] for _ in range(w.M)]).astype(np.int32)


def worker_scales(M, cfg=4):
    """s_m log-uniform in [1e-3, 1]."""
    u = _rng(cfg, 1).random(M)
    return (10.0 ** (-3.0 * u)).astype(np.float32)


def host_gradients(M, p, cfg=4, stream=2, scales=None):
    """G[M][p] ~ N(0, s_m^2) on the host (test sizes)."""
    s = worker_scales(M, cfg) if scales is None else scales
    g = _rng(cfg, stream).standard_normal((M, p), dtype=np.float32)
    return (g * s[:, None]).astype(np.float32)


def host_drift(G, it, cfg=4, scales=None):
    """G + N(0, 0.01 s_m^2): the per-iteration drift of the synthetic gradients."""
    M, p = G.shape
    s = worker_scales(M, cfg) if scales is None else scales
    n = _rng(cfg, 100 + it).standard_normal((M, p), dtype=np.float32)
    return (G + n * (np.float32(0.1) * s)[:, None]).astype(np.float32)


def device_gradients(M, p, p_stride, device, cfg=4):
    """Full-size synthetic gradients generated in device memory with torch's
    seeded generator (an input generator, not part of the method).  Returns
    (G[M][p_stride] torch.float32, scales torch.float32[M], generator)."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(SEED0 + cfg)
    s = torch.from_numpy(worker_scales(M, cfg)).to(device)
    G = torch.empty((M, p_stride), dtype=torch.float32, device=device)
    for m in range(M):
        G[m].normal_(0.0, 1.0, generator=gen)
        G[m].mul_(s[m])
    return G, s, gen


def device_drift_(G, s, gen, tmp=None):
    """In-place drift G += N(0, 0.01 s_m^2) in device memory."""
    import torch
    M = G.shape[0]
    if tmp is None:
        tmp = torch.empty_like(G[0])
    for m in range(M):
        tmp.normal_(0.0, 1.0, generator=gen)
        G[m].add_(tmp, alpha=float(0.1 * s[m].item()))
    return G
