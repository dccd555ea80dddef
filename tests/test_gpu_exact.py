"""GPU parity of the identity quantizer (b = LAQ_B_EXACT): lazy aggregation of exact gradients
(LAG, the many-bits limit noted after eqs. 7a-7b) and, with forced uploads, gradient descent
(eq. 2).  Messages, radii, stored gradients, nabla, theta, clocks and counters bit-exact; the
left side of (7a), a binary64 sum whose order is free, within 4 p 2^-53."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
import laq_synth
import oracle
import paper_1909_07588_amd as laq
from gpu_common import DEV, bits_equal, check_quantize, check_server, make_pair, push_state, to_dev_G

pytestmark = pytest.mark.gpu
BX = oracle.B_EXACT


def _random_state(st, rng):
    M, p = st.M, st.p
    st.H[:] = rng.standard_normal((M, p)).astype(np.float32)
    st.nabla[:] = st.H.sum(0)
    st.theta[:] = rng.standard_normal(p).astype(np.float32)
    st.t[:] = rng.integers(0, st.t_bar + 1, M)
    st.dtheta2[:] = rng.random(st.D) * 1e-2


@pytest.mark.parametrize("M,p", [(1, 1), (3, 7), (4, 8), (5, 2049), (3, 70001), (2, 300000)])
def test_one_iteration_from_a_random_state(M, p):
    assert laq.lib().laq_w_stride(p, BX) >= p
    rng = np.random.default_rng(p)
    ctx, st, theta = make_pair(M, p, BX, D=5, t_bar=8, alpha=0.05)
    _random_state(st, rng)
    theta.copy_(torch.from_numpy(st.theta))
    push_state(ctx, st)
    # innovations of very different sizes, so that some workers skip and some upload
    scale = (10.0 ** rng.uniform(-4, 0, (M, 1))).astype(np.float32)
    G = (st.H + scale * rng.standard_normal((M, p))).astype(np.float32)
    G[0, 0] = st.H[0, 0]                                      # a coordinate with zero innovation
    Gd = to_dev_G(ctx, G)
    msgs, ref = check_quantize(ctx, st, Gd, G)
    assert all(o["E2"] == 0.0 for o in ref)
    check_server(ctx, st, theta, msgs, G)


def test_zero_innovation_upload_stores_the_gradient_bits():
    """A forced upload with g == h in value: the stored gradient takes g's bits (-0.0 stays -0.0)."""
    M, p = 2, 19
    ctx, st, theta = make_pair(M, p, BX, D=2, t_bar=3, alpha=0.1)
    st.H[:] = 0.0
    push_state(ctx, st)
    G = np.zeros((M, p), np.float32)
    G[0, 3] = -0.0
    Gd = to_dev_G(ctx, G)
    msgs, _ = check_quantize(ctx, st, Gd, G)          # t = t_bar: both upload although R = 0
    out = check_server(ctx, st, theta, msgs, G)
    assert out["upload"].all()
    assert np.signbit(ctx.state()["H"][0, 3].item())


def test_lag_run_on_the_smallest_workload_skips_and_stays_on_the_oracle():
    w = laq_synth.workload(1)
    X, y, theta0 = laq_synth.model_inputs(w)
    ctx, st, theta = make_pair(w.M, w.p, BX, D=w.D, xi=w.xi, t_bar=w.t_bar, alpha=w.alpha, theta0=theta0)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    ctx.laq_set_data(torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV))
    Gd = ctx.alloc_G()
    msgs = ctx.alloc_messages()
    skipped = 0
    for it in range(120):
        ctx.laq_worker_grads(theta, Gd)
        torch.cuda.synchronize()
        G = Gd[:, :w.p].cpu().numpy()
        msgs, _ = check_quantize(ctx, st, Gd, G, msgs)
        out = check_server(ctx, st, theta, msgs, G)
        skipped += int((out["upload"] == 0).sum())
        push_state(ctx, st)
    assert skipped > 120
    up, bits, status = ctx.laq_get_counters()
    assert status == 0 and bits == int(up.sum()) * 32 * w.p


def test_forced_uploads_with_exact_messages_is_gradient_descent():
    """Every worker uploads its exact gradient: nabla^k = sum_m g_m^k (up to the rounding of the
    incremental update) and theta follows eq. 2."""
    rng = np.random.default_rng(3)
    M, p = 4, 1000
    ctx, st, theta = make_pair(M, p, BX, D=3, t_bar=5, alpha=0.1)
    ctx.laq_set_mode(laq.MODE_FORCE_UPLOAD)
    msgs = ctx.alloc_messages()
    th = np.zeros(p, np.float64)
    for it in range(10):
        G = rng.standard_normal((M, p)).astype(np.float32)
        Gd = to_dev_G(ctx, G)
        msgs, _ = check_quantize(ctx, st, Gd, G, msgs, force=True)
        check_server(ctx, st, theta, msgs, G, force=True)
        push_state(ctx, st)                      # the history entry is compared within a tolerance
        th -= 0.1 * G.astype(np.float64).sum(0)
        assert np.abs(theta.cpu().numpy() - th).max() <= 1e-5 * max(1.0, np.abs(th).max())
    assert ctx.laq_get_counters()[0].sum() == 10 * M
