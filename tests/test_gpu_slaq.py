"""GPU parity of the stochastic variant (SLAQ, Sec. 4 "Stochastic gradient-based tests"):
minibatch gradients from laq_worker_grads_minibatch against the oracle's, and the LAQ loop run
on them, teacher-forced."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
import laq_synth
import oracle
from gpu_common import DEV, check_model_grads, check_quantize, check_server, make_pair, push_state

pytestmark = pytest.mark.gpu


def _bind(w, theta0):
    X, y, _ = laq_synth.model_inputs(w)
    ctx, st, theta = make_pair(w.M, w.p, w.b, D=w.D, xi=w.xi, t_bar=w.t_bar, alpha=w.alpha, theta0=theta0)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    ctx.laq_set_data(torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV))
    return ctx, st, theta, X, y


@pytest.mark.parametrize("cfg,scale,B", [(1, 1.0, 17), (2, 0.05, 64), (2, 0.02, 120), (3, 0.02, 50)])
def test_minibatch_gradients_match_the_oracle(cfg, scale, B):
    w = laq_synth.workload(cfg, scale)
    _, _, theta0 = laq_synth.model_inputs(w)
    rng = np.random.default_rng(cfg)
    theta_h = (theta0 + 0.05 * rng.standard_normal(w.p)).astype(np.float32)
    ctx, st, theta, X, y = _bind(w, theta_h)
    Gd = ctx.alloc_G()
    for it in range(3):
        idx = laq_synth.minibatch_indices(w, B, it)
        if it == 2:
            idx[:, 1] = idx[:, 0]                      # a repeated sample is a legal draw
        ctx.laq_worker_grads_minibatch(theta, torch.from_numpy(idx).to(DEV), Gd)
        torch.cuda.synchronize()
        G = Gd[:, :w.p].cpu().numpy()
        G_ref = oracle.grads_minibatch(w.kind, theta_h, X, y, w.dims, w.lam, idx)
        check_model_grads(w, G, G_ref, theta_h, X, y, idx=idx, tag=f"iteration {it}")
    # the full-batch call still sees the data bound by laq_set_data
    ctx.laq_worker_grads(theta, Gd)
    torch.cuda.synchronize()
    G_ref, _ = oracle.grads_all(w.kind, theta_h, X, y, w.dims, w.lam)
    G = Gd[:, :w.p].cpu().numpy()
    check_model_grads(w, G, G_ref, theta_h, X, y)
    assert ctx.laq_get_counters()[2] == 0


def test_whole_shard_as_one_batch_is_the_full_gradient():
    w = laq_synth.workload(2, 0.01)
    _, _, theta0 = laq_synth.model_inputs(w)
    ctx, st, theta, X, y = _bind(w, theta0 + np.float32(0.01))
    idx = np.stack([np.random.default_rng(m).permutation(w.N_m) for m in range(w.M)]).astype(np.int32)
    Ga, Gb = ctx.alloc_G(), ctx.alloc_G()
    ctx.laq_worker_grads_minibatch(theta, torch.from_numpy(idx).to(DEV), Ga)
    ctx.laq_worker_grads(theta, Gb)
    torch.cuda.synchronize()
    a, b = Ga[:, :w.p].cpu().numpy(), Gb[:, :w.p].cpu().numpy()
    assert np.abs(a - b).max() <= 1e-5 * np.abs(b).max()


def test_slaq_loop_teacher_forced():
    """LAQ on minibatch gradients (batch 50 of 300 per worker): every iteration the oracle
    quantizes the GPU's gradients from the same state; codes, masks, state compared as for LAQ."""
    w = laq_synth.workload(2, 0.05)
    w.alpha = 0.008
    _, _, theta0 = laq_synth.model_inputs(w)
    ctx, st, theta, X, y = _bind(w, theta0)
    Gd = ctx.alloc_G()
    msgs = ctx.alloc_messages()
    B = 50
    uploads = 0
    for it in range(25):
        idx = laq_synth.minibatch_indices(w, B, it)
        ctx.laq_worker_grads_minibatch(theta, torch.from_numpy(idx).to(DEV), Gd)
        torch.cuda.synchronize()
        G = Gd[:, :w.p].cpu().numpy()
        G_ref = oracle.grads_minibatch(w.kind, st.theta, X, y, w.dims, w.lam, idx)
        err = np.abs(G - G_ref).max() / np.abs(G_ref).max()
        assert err <= 1e-5, (it, err)
        msgs, _ = check_quantize(ctx, st, Gd, G, msgs)
        out = check_server(ctx, st, theta, msgs, G)
        uploads += int(out["upload"].sum())
        push_state(ctx, st)
    assert w.M < uploads <= 25 * w.M


def test_out_of_range_index_is_clamped_and_reported():
    w = laq_synth.workload(1)
    _, _, theta0 = laq_synth.model_inputs(w)
    ctx, st, theta, X, y = _bind(w, theta0)
    idx = laq_synth.minibatch_indices(w, 8, 0)
    idx[3, 2] = w.N_m + 5
    idx[4, 0] = -1
    Gd = ctx.alloc_G()
    ctx.laq_worker_grads_minibatch(theta, torch.from_numpy(idx).to(DEV), Gd)
    torch.cuda.synchronize()
    assert ctx.laq_get_counters()[2] == 1            # LAQ_EINVAL
    fixed = idx.copy()
    fixed[3, 2] = w.N_m - 1
    fixed[4, 0] = 0
    G_ref = oracle.grads_minibatch(w.kind, theta0, X, y, w.dims, w.lam, fixed)
    G = Gd[:, :w.p].cpu().numpy()
    assert np.abs(G - G_ref).max() <= 1e-5 * np.abs(G_ref).max()


def test_bad_minibatch_arguments():
    w = laq_synth.workload(1)
    _, _, theta0 = laq_synth.model_inputs(w)
    ctx, st, theta, X, y = _bind(w, theta0)
    Gd = ctx.alloc_G()
    idx = torch.zeros((w.M, w.N_m + 1), dtype=torch.int32, device=DEV)      # B > N_m
    with pytest.raises(Exception):
        ctx.laq_worker_grads_minibatch(theta, idx, Gd)
