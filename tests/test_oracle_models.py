"""Pins for the oracle's model gradients (supplement, "Simulation details"):
central finite differences of the loss it reports, and torch's float64
autograd on the same models written with library ops."""
import numpy as np
import pytest
import torch

import laq_synth
import oracle


def _tiny(kind, seed=0):
    rng = np.random.default_rng(seed)
    M, N_m = 3, 7
    if kind == 1:
        dims, F = (6,), 6
    elif kind == 2:
        dims, F = (6, 4), 6
    else:
        dims, F = (6, 5, 3, 4), 6
    ldx = laq_synth.pad4(F)
    X = np.zeros((M, N_m, ldx), np.float32)
    X[:, :, :F] = np.round(rng.standard_normal((M, N_m, F)) * 64) / 64
    if kind == 1:
        y = rng.choice([-1, 1], (M, N_m)).astype(np.int32)
    else:
        y = rng.integers(0, dims[-1], (M, N_m)).astype(np.int32)
    p = oracle.model_params(kind, dims)
    theta = (np.round(rng.standard_normal(p) * 256) / 1024).astype(np.float32)
    return X, y, theta, dims


@pytest.mark.parametrize("kind", [1, 2, 3])
def test_gradient_matches_central_differences_of_the_loss(kind):
    X, y, theta, dims = _tiny(kind)
    lam = 0.01
    G, _ = oracle.grads_all(kind, theta, X, y, dims, lam)
    g = G.astype(np.float64).sum(0)               # sum of worker shares = gradient of global loss
    h = 2.0 ** -14                                # theta +- h is exact in fp32
    fd = np.zeros_like(g)
    for i in range(theta.size):
        tp, tm = theta.copy(), theta.copy()
        tp[i] += np.float32(h)
        tm[i] -= np.float32(h)
        fd[i] = (oracle.grads_all(kind, tp, X, y, dims, lam)[1]
                 - oracle.grads_all(kind, tm, X, y, dims, lam)[1]) / (2 * h)
    assert np.abs(fd - g).max() <= 2e-4 * np.abs(g).max()


def _torch_loss(kind, theta, X, y, dims, lam, m=None):
    """Global loss, or worker m's share f_m/N, in float64 torch ops."""
    Xt = torch.from_numpy(X.astype(np.float64))
    M, N_m, _ = X.shape
    N = M * N_m
    ms = range(M) if m is None else [m]
    tot = 0.0
    for mm in ms:
        x = Xt[mm][:, :dims[0]]
        if kind == 1:
            z = x @ theta
            tot = tot + torch.nn.functional.softplus(-torch.from_numpy(y[mm].astype(np.float64)) * z).sum()
        elif kind == 2:
            W = theta.reshape(dims[1], dims[0])            # theta in R^{C x F}
            tot = tot + torch.nn.functional.cross_entropy(x @ W.T, torch.from_numpy(y[mm]).long(),
                                                          reduction="sum")
        else:
            a, off = x, 0
            for l in range(len(dims) - 1):
                W = theta[off:off + dims[l] * dims[l + 1]].reshape(dims[l], dims[l + 1])
                off += dims[l] * dims[l + 1]
                bb = theta[off:off + dims[l + 1]]
                off += dims[l + 1]
                a = a @ W + bb
                if l + 2 < len(dims):
                    a = torch.relu(a)
            tot = tot + torch.nn.functional.cross_entropy(a, torch.from_numpy(y[mm]).long(),
                                                          reduction="sum")
    return tot / N + (len(list(ms)) * N_m / N) * 0.5 * lam * (theta ** 2).sum()


@pytest.mark.parametrize("kind", [1, 2, 3])
def test_worker_shares_match_float64_autograd(kind):
    X, y, theta, dims = _tiny(kind, seed=1)
    lam = 0.01
    G, loss = oracle.grads_all(kind, theta, X, y, dims, lam)
    th = torch.from_numpy(theta.astype(np.float64)).requires_grad_(True)
    assert loss == pytest.approx(float(_torch_loss(kind, th, X, y, dims, lam)), rel=1e-9)
    for m in range(X.shape[0]):
        th.grad = None
        _torch_loss(kind, th, X, y, dims, lam, m=m).backward()
        ref = th.grad.numpy()
        assert np.abs(G[m] - ref).max() <= 2e-7 * np.abs(ref).max()


def test_mlp_matches_autograd_at_a_wider_shape_with_sparse_inputs():
    w = laq_synth.Workload("t", 3, laq_synth.KIND_MLP, 2, 33, (20, 16, 12, 5), 0, 8)
    w.p = laq_synth.mlp_param_count(w.dims)
    X, y, theta = laq_synth.model_inputs(w)
    G, _ = oracle.grads_all(3, theta, X, y, w.dims, 0.01)
    th = torch.from_numpy(theta.astype(np.float64)).requires_grad_(True)
    for m in range(2):
        th.grad = None
        _torch_loss(3, th, X, y, w.dims, 0.01, m=m).backward()
        ref = th.grad.numpy()
        assert np.abs(G[m] - ref).max() <= 2e-7 * np.abs(ref).max()


# ---- minibatch gradients (SLAQ, Sec. 4 "Stochastic gradient-based tests") ----

@pytest.mark.parametrize("kind", [1, 2, 3])
def test_minibatch_gradient_matches_float64_autograd_of_the_minibatch_loss(kind):
    """g_m = grad of (1/(M B)) sum_{j} CE_{idx[m][j]} + (1/M)(lambda/2)||theta||^2, written with
    torch float64 ops on the rows picked out by idx (repeats allowed)."""
    X, y, theta, dims = _tiny(kind, seed=2)
    M, N_m, _ = X.shape
    lam = 0.01
    rng = np.random.default_rng(5)
    B = 4
    idx = rng.integers(0, N_m, (M, B)).astype(np.int32)
    idx[0] = [3, 3, 0, 6]                                   # a repeated sample
    G = oracle.grads_minibatch(kind, theta, X, y, dims, lam, idx)
    th = torch.from_numpy(theta.astype(np.float64)).requires_grad_(True)
    for m in range(M):
        th.grad = None
        xs = torch.from_numpy(X[m][idx[m]][:, :dims[0]].astype(np.float64))
        ys = y[m][idx[m]]
        if kind == 1:
            ce = torch.nn.functional.softplus(-torch.from_numpy(ys.astype(np.float64)) * (xs @ th)).sum()
        elif kind == 2:
            ce = torch.nn.functional.cross_entropy(xs @ th.reshape(dims[1], dims[0]).T,
                                                   torch.from_numpy(ys).long(), reduction="sum")
        else:
            a, off = xs, 0
            for l in range(len(dims) - 1):
                W = th[off:off + dims[l] * dims[l + 1]].reshape(dims[l], dims[l + 1])
                off += dims[l] * dims[l + 1]
                bb = th[off:off + dims[l + 1]]
                off += dims[l + 1]
                a = a @ W + bb
                if l + 2 < len(dims):
                    a = torch.relu(a)
            ce = torch.nn.functional.cross_entropy(a, torch.from_numpy(ys).long(), reduction="sum")
        (ce / (M * B) + (1.0 / M) * 0.5 * lam * (th ** 2).sum()).backward()
        ref = th.grad.numpy()
        assert np.abs(G[m] - ref).max() <= 2e-7 * np.abs(ref).max()


@pytest.mark.parametrize("kind", [1, 2, 3])
def test_minibatch_gradients_over_a_partition_average_to_the_full_gradient(kind):
    """Unbiasedness: the minibatch gradients of disjoint batches that cover the shard
    average to the worker's full gradient (equal shards)."""
    rng = np.random.default_rng(7)
    X, y, theta, dims = _tiny(kind, seed=3)
    X, y = np.concatenate([X, X[:, :1]], 1), np.concatenate([y, y[:, :1]], 1)   # N_m = 8
    M, N_m, _ = X.shape
    lam = 0.01
    full, _ = oracle.grads_all(kind, theta, X, y, dims, lam)
    B = 2
    perm = np.stack([rng.permutation(N_m) for _ in range(M)]).astype(np.int32)
    acc = np.zeros(full.shape, np.float64)
    for k in range(N_m // B):
        acc += oracle.grads_minibatch(kind, theta, X, y, dims, lam, perm[:, k * B:(k + 1) * B])
    mean = acc / (N_m // B)
    assert np.abs(mean - full).max() <= 1e-6 * np.abs(full).max()
    # and a batch that is the whole shard, in any order, is the full gradient
    whole = oracle.grads_minibatch(kind, theta, X, y, dims, lam, perm)
    assert np.abs(whole - full).max() <= 1e-6 * np.abs(full).max()


def test_parameter_counts():
    assert oracle.mlp_params((784, 200, 10)) == 159010
    assert oracle.mlp_params((784, 2048, 2048, 10)) == 5824522
    assert oracle.model_params(2, (785, 10)) == 7850
