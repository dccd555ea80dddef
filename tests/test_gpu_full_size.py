"""The model workloads at the sizes and in the launch configurations bench.py times.

Headline workload (multinomial logistic regression 785x10, M = 10 x 6000): the whole loop against the
oracle, with the samples tiled (as timed) and row-major; the stochastic variant (minibatch 500) on both
small models likewise.  784-200-10 network at full size: gradients of sampled workers against the oracle.  The
784-2048-2048-10 network (M = 32 x 8192) is too large for the oracle's plain loops, so its full-size
launch is tied to launches the oracle does check by a property that holds at any size: a worker's
full-batch gradient is the average of its minibatch gradients over a partition of its shard."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
import laq_synth
import oracle
from gpu_common import DEV, check_quantize, check_server, make_pair, push_state

pytestmark = pytest.mark.gpu


def _bind(w, theta0, b=None):
    X, y, _ = laq_synth.model_inputs(w)
    ctx, st, theta = make_pair(w.M, w.p, w.b if b is None else b, D=w.D, xi=w.xi, t_bar=w.t_bar,
                               alpha=w.alpha, theta0=theta0)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    ctx.laq_set_data(torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV))
    return ctx, st, theta, X, y


@pytest.mark.parametrize("tiled", [True, False], ids=["tiled_samples", "row_major_samples"])
def test_headline_workload_full_size_loop(tiled):
    """tiled: the samples laid out by laq_tile_data, the launch bench.py times."""
    w = laq_synth.workload(2)
    _, _, theta0 = laq_synth.model_inputs(w)
    ctx, st, theta, X, y = _bind(w, theta0)
    if tiled:
        assert ctx.laq_tiled_data_bytes() > 0
        ctx.laq_tile_data()
    Gd = ctx.alloc_G()
    msgs = ctx.alloc_messages()
    for it in range(4):
        ctx.laq_worker_grads(theta, Gd)
        torch.cuda.synchronize()
        G = Gd[:, :w.p].cpu().numpy()
        G_ref, _ = oracle.grads_all(w.kind, st.theta, X, y, w.dims, w.lam)
        err = np.abs(G - G_ref).max(axis=1) / np.abs(G_ref).max(axis=1)
        assert err.max() <= 1e-5, (it, err)
        msgs, _ = check_quantize(ctx, st, Gd, G, msgs)
        check_server(ctx, st, theta, msgs, G)
        push_state(ctx, st)


@pytest.mark.parametrize("cfg", [2, 3])
def test_stochastic_variant_full_size_loop(cfg):
    """Sec. 4's stochastic setting as bench.py times it: full shards, 500 drawn samples per worker,
    alpha = 0.008; the whole loop, teacher-forced."""
    w = laq_synth.workload(cfg)
    w.alpha = 0.008
    B = 500
    _, _, theta0 = laq_synth.model_inputs(w)
    ctx, st, theta, X, y = _bind(w, theta0)
    Gd = ctx.alloc_G()
    msgs = ctx.alloc_messages()
    for it in range(3):
        idx = laq_synth.minibatch_indices(w, B, it)
        ctx.laq_worker_grads_minibatch(theta, torch.from_numpy(idx).to(DEV), Gd)
        torch.cuda.synchronize()
        G = Gd[:, :w.p].cpu().numpy()
        G_ref = oracle.grads_minibatch(w.kind, st.theta, X, y, w.dims, w.lam, idx)
        err = np.abs(G - G_ref).max(axis=1) / np.abs(G_ref).max(axis=1)
        assert err.max() <= 1e-5, (it, err)
        msgs, _ = check_quantize(ctx, st, Gd, G, msgs)
        check_server(ctx, st, theta, msgs, G)
        push_state(ctx, st)
    assert ctx.laq_get_counters()[2] == 0


def test_small_network_full_size_sampled_workers():
    w = laq_synth.workload(3)
    X, y, theta0 = laq_synth.model_inputs(w)
    rng = np.random.default_rng(3)
    theta_h = (theta0 + 0.02 * rng.standard_normal(w.p)).astype(np.float32)
    ctx, st, theta, X, y = _bind(w, theta_h)
    Gd = ctx.alloc_G()
    ctx.laq_worker_grads(theta, Gd)
    torch.cuda.synchronize()
    G = Gd[:, :w.p].cpu().numpy()
    N = w.M * w.N_m
    for m in (0, 7):
        g_ref = oracle.grad_worker(w.kind, theta_h, X[m], y[m], w.dims, w.lam, N)
        err = np.abs(G[m] - g_ref).max() / np.abs(g_ref).max()
        assert err <= 1e-5, (m, err)


def test_largest_network_full_size_gradient_is_the_average_over_a_partition():
    w = laq_synth.workload(5)
    _, _, theta0 = laq_synth.model_inputs(w)
    ctx, st, theta, X, y = _bind(w, theta0)
    del X, y
    Gd, Gmb = ctx.alloc_G(), ctx.alloc_G()
    ctx.laq_worker_grads(theta, Gd)
    parts = 8
    B = w.N_m // parts
    acc = torch.zeros_like(Gd, dtype=torch.float64)
    base = torch.arange(B, dtype=torch.int32, device=DEV)
    for k in range(parts):
        idx = (base + k * B).repeat(w.M, 1).contiguous()
        ctx.laq_worker_grads_minibatch(theta, idx, Gmb)
        acc += Gmb.double()
    torch.cuda.synchronize()
    mean = (acc / parts)[:, :w.p]
    full = Gd[:, :w.p].double()
    err = ((mean - full).abs().amax(dim=1) / full.abs().amax(dim=1)).max().item()
    assert err <= 1e-5, err
    assert ctx.laq_get_counters()[2] == 0
