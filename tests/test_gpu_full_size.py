"""The model workloads at the sizes and in the launch configurations bench.py times.

Headline workload (multinomial logistic regression 785x10, M = 10 x 6000): the whole loop against the
oracle, with the samples tiled (as timed) and row-major; the stochastic variant (minibatch 500) on both
small models likewise.  784-200-10 network at full size: gradients of sampled workers against the oracle.  The
784-2048-2048-10 network (M = 32 x 8192), in the launch bench.py times: the gradients of sampled workers
against the oracle's plain loops (a quarter of a TFLOP in binary64 per worker), then the quantizer, the skip
rule and the server step on the GPU's own gradients against the oracle for all 32 workers; and a property that
ties every worker to launches the oracle checks: a worker's full-batch gradient is the average of its minibatch
gradients over a partition of its shard."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
import laq_synth
import oracle
from gpu_common import (DEV, bits_equal, check_model_grads, check_quantize, check_server, make_pair,
                        push_state)

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
        check_model_grads(w, G, G_ref, st.theta, X, y, tag=f"iteration {it}")
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
        check_model_grads(w, G, G_ref, st.theta, X, y, idx=idx, tag=f"iteration {it}")
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
    report = []
    ref = {m: oracle.grad_worker(w.kind, theta_h, X[m], y[m], w.dims, w.lam, N) for m in (0, 7)}
    check_model_grads(w, G, ref, theta_h, X, y, workers=(0, 7), report=report)
    print("relu candidates / flips:", [(r[1], r[2]) for r in report])


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


def test_largest_network_full_size_against_the_oracle():
    """Workload 5 as bench.py runs it (M = 32 x 8192 samples, 784-2048-2048-10, b = 4), from a mid-run state:
    the gradients of two sampled workers against the oracle; every worker's radius (handed over by the
    weight-gradient epilogues), integer sums, both sides of (7a) and decision, and the packed codes of four
    workers, against the oracle quantizing the GPU's gradients; then one server step, bit for bit."""
    w = laq_synth.workload(5)
    X, y, theta0 = laq_synth.model_inputs(w)
    rng = np.random.default_rng(55)
    theta_h = (theta0 + 0.01 * rng.standard_normal(w.p)).astype(np.float32)
    ctx, st, theta = make_pair(w.M, w.p, w.b, D=w.D, xi=w.xi, t_bar=w.t_bar, alpha=w.alpha, theta0=theta_h)
    M, p, b = w.M, w.p, w.b
    for m in range(M):                                       # mid-run stored gradients, worker by worker
        st.H[m] = (2e-5 * rng.standard_normal(p)).astype(np.float32)
    st.nabla[:] = st.H.sum(0)
    st.Ehat2[:] = rng.random(M) * 1e-9
    st.t[:] = rng.integers(0, w.t_bar + 1, M)
    st.dtheta2[:] = rng.random(w.D) * 1e-10
    push_state(ctx, st)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    ctx.laq_set_data(torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV))
    Gd = ctx.alloc_G()
    ctx.laq_worker_grads(theta, Gd)
    codes, R, up = ctx.alloc_messages()
    ctx.laq_quantize_skip(Gd, codes, R, up)                  # single pass: the radius comes from the epilogues
    torch.cuda.synchronize()
    G = Gd[:, :p].cpu().numpy()
    # a1: sampled workers against the oracle's plain loops
    sampled = (5, 30)
    report = []
    ref = {m: oracle.grad_worker(w.kind, theta_h, X[m], y[m], w.dims, w.lam, M * w.N_m) for m in sampled}
    check_model_grads(w, G, ref, theta_h, X, y, workers=sampled, report=report)
    print("relu candidates / flips:", [(r[1], r[2]) for r in report], flush=True)
    del X, ref
    # a2 + a3: all workers
    sview = ctx.state()
    R_h, up_h = R.cpu().numpy(), up.cpu().numpy()
    Sq_h, E2_h = sview["Sq"].cpu().numpy(), sview["E2"].cpu().numpy()
    lhs_h, rhs_h = sview["lhs"].cpu().numpy(), sview["rhs"].cpu().numpy()
    nw = oracle.code_words(p, b)
    with_codes = {0, 5, 17, 31}
    for m in range(M):
        o = oracle.quantize(G[m], st.H[m], b, want_vectors=(m in with_codes))
        skip, rhs = oracle.skip(o["lhs"], o["E2"], st.Ehat2[m], st.xi, st.dtheta2, st.alpha, M, st.t[m], st.t_bar)
        assert bits_equal(np.float32(R_h[m]), np.float32(o["R"])), m
        assert int(Sq_h[m]) == o["Sq"] and bits_equal(np.float64(E2_h[m]), np.float64(o["E2"])), m
        assert bits_equal(np.float64(lhs_h[m]), np.float64(o["lhs"])), m
        assert bits_equal(np.float64(rhs_h[m]), np.float64(rhs)), m
        assert int(up_h[m]) == int(not skip), m
        if m in with_codes:
            got = codes[m, :nw].cpu().numpy().view(np.uint32)
            assert np.array_equal(got, oracle.pack(o["q"], b)), m
    assert 0 < int(up_h.sum())                               # the server step below has rows to aggregate
    # a4: one server step
    out = st.iteration(G, want_codes=False)
    ctx.laq_server_step(codes, R, up, theta)
    torch.cuda.synchronize()
    assert np.array_equal(up_h, out["upload"])
    assert bits_equal(theta.cpu().numpy(), st.theta)
    assert bits_equal(sview["nabla"][:p].cpu().numpy(), st.nabla)
    for m in (0, 17, 31):
        assert bits_equal(sview["H"][m, :p].cpu().numpy(), st.H[m]), m
    assert np.array_equal(sview["t"].cpu().numpy(), st.t)
    assert np.allclose(sview["dtheta2"].cpu().numpy(), st.dtheta2, rtol=4.0 * p * 2.0 ** -53, atol=0)
