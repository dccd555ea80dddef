"""Helpers shared by the GPU parity tests: run the HIP path through its C ABI
binding and the oracle on the same inputs and state."""
import numpy as np
import torch

import oracle
import paper_1909_07588_amd as laq

DEV = "cuda:0"


def make_pair(M, p, b, D=10, xi=0.08, t_bar=100, alpha=0.01, theta0=None):
    """A HIP context and an oracle state with identical parameters and initial state."""
    th0 = np.zeros(p, np.float32) if theta0 is None else np.asarray(theta0, np.float32)
    ctx = laq.Laq(M, p, b, D, xi, t_bar, alpha, device=DEV)
    st = oracle.State(M, p, b, D, xi, t_bar, alpha, th0)
    theta = torch.from_numpy(th0.copy()).to(DEV)
    return ctx, st, theta


def push_state(ctx, st):
    """Impose the oracle's state on the HIP context (teacher forcing)."""
    s = ctx.state()
    s["H"][:, :st.p].copy_(torch.from_numpy(st.H))
    s["nabla"][:st.p].copy_(torch.from_numpy(st.nabla))
    s["Ehat2"].copy_(torch.from_numpy(st.Ehat2))
    s["t"].copy_(torch.from_numpy(st.t))
    s["dtheta2"].copy_(torch.from_numpy(st.dtheta2))
    torch.cuda.synchronize()


def to_dev_G(ctx, G):
    Gd = ctx.alloc_G()
    Gd[:, :ctx.p].copy_(torch.from_numpy(np.ascontiguousarray(G, np.float32)))
    return Gd


def bits_equal(a, b):
    a = np.ascontiguousarray(a)
    b = np.ascontiguousarray(b)
    return a.shape == b.shape and np.array_equal(a.view(np.uint8), b.view(np.uint8))


def check_quantize(ctx, st, Gd, G, msgs=None, force=False):
    """laq_quantize_skip against the oracle's quantizer + skip rule on state st.
    Returns (codes, R, upload) device tensors and the oracle's per-worker outputs."""
    codes, R, up = msgs if msgs is not None else ctx.alloc_messages()
    ctx.laq_quantize_skip(Gd, codes, R, up)
    torch.cuda.synchronize()
    s = ctx.state()
    M, p, b = st.M, st.p, st.b
    nw = oracle.code_words(p, b)
    codes_h = codes.cpu().numpy().view(np.uint32)
    R_h, up_h = R.cpu().numpy(), up.cpu().numpy()
    Sq_h, E2_h = s["Sq"].cpu().numpy(), s["E2"].cpu().numpy()
    lhs_h, rhs_h = s["lhs"].cpu().numpy(), s["rhs"].cpu().numpy()
    ref = []
    for m in range(M):
        o = oracle.quantize(G[m], st.H[m], b)
        assert o["status"] == oracle.OK
        skip, rhs = oracle.skip(o["lhs"], o["E2"], st.Ehat2[m], st.xi, st.dtheta2, st.alpha, M,
                                st.t[m], st.t_bar)
        if force:
            skip = False
        assert bits_equal(np.float32(R_h[m]), np.float32(o["R"])), (m, R_h[m], o["R"])
        packed = oracle.pack(o["q"], b)
        assert np.array_equal(codes_h[m, :nw], packed), f"codes differ for worker {m}"
        assert int(Sq_h[m]) == o["Sq"], (m, Sq_h[m], o["Sq"])
        assert bits_equal(np.float64(E2_h[m]), np.float64(o["E2"])), (m, E2_h[m], o["E2"])
        near_tie = False
        if b == oracle.B_EXACT:
            # ||g - h||^2 is a binary64 sum of exact squares whose order is the implementation's
            tol = max(1e-13, 4.0 * p * 2.0 ** -53)
            assert abs(lhs_h[m] - o["lhs"]) <= tol * o["lhs"], (m, lhs_h[m], o["lhs"])
            near_tie = abs(o["lhs"] - rhs) <= 2 * tol * max(o["lhs"], rhs)
        else:
            assert bits_equal(np.float64(lhs_h[m]), np.float64(o["lhs"])), (m, lhs_h[m], o["lhs"])
        assert bits_equal(np.float64(rhs_h[m]), np.float64(rhs)), (m, rhs_h[m], rhs)
        assert near_tie or int(up_h[m]) == int(not skip), (m, up_h[m], skip, o["lhs"], rhs)
        ref.append(o)
    return (codes, R, up), ref


def check_server(ctx, st, theta, msgs, G, force=False, ring_rtol=None):
    """laq_server_step against the oracle's iteration (which also advances st)."""
    codes, R, up = msgs
    out = st.iteration(G, force_upload=force)
    assert out["status"] == oracle.OK
    ctx.laq_server_step(codes, R, up, theta)
    torch.cuda.synchronize()
    s = ctx.state()
    p = st.p
    assert np.array_equal(up.cpu().numpy(), out["upload"])
    assert bits_equal(s["H"][:, :p].cpu().numpy(), st.H), "stored quantized gradients differ"
    assert bits_equal(s["nabla"][:p].cpu().numpy(), st.nabla), "nabla differs"
    assert bits_equal(theta[:p].cpu().numpy(), st.theta), "theta differs"
    assert np.array_equal(s["t"].cpu().numpy(), st.t)
    assert bits_equal(s["Ehat2"].cpu().numpy(), st.Ehat2)
    assert np.array_equal(s["uploads"].cpu().numpy().astype(np.uint64), st.uploads)
    assert int(s["bits"].cpu().numpy()[0]) == st.bits.value
    d2 = s["dtheta2"].cpu().numpy()
    if ring_rtol is None:
        # binary64 sum of p exact squares; only its order differs between the two sides
        ring_rtol = max(1e-13, 4.0 * p * 2.0 ** -53)
    assert np.allclose(d2, st.dtheta2, rtol=ring_rtol, atol=0.0), (d2, st.dtheta2)
    return out


def check_model_grads(w, G, G_ref, theta, X, y, idx=None, workers=None, report=None, tag=""):
    """Model gradients of the HIP path against the oracle's, per worker, within 1e-5 of the worker's
    largest gradient entry.  The ReLU network has one discrete decision per hidden unit and sample
    (z > 0) that binary32 and binary64 sums cannot share at |z| within rounding of zero: there the
    comparison is the one relu_rule documents (flip a subset of the near-zero candidates, found by a
    fit, then compare as usual).  idx[M][B]: the rows a minibatch call drew.  G, G_ref: [M][p], or
    {m: g} for sampled workers."""
    import relu_rule
    ms = range(w.M) if workers is None else workers
    for m in ms:
        g, g_ref = G[m], G_ref[m]
        if w.kind == 3:
            Xm, ym = (X[m], y[m]) if idx is None else (X[m][idx[m]], y[m][idx[m]])
            relu_rule.assert_network_gradients_close(g, g_ref, theta, Xm, ym, w.dims, w.M * len(ym),
                                                     tag=f"{tag} worker {m}", report=report)
        else:
            err = np.abs(g - g_ref).max() / np.abs(g_ref).max()
            assert err <= 1e-5, (tag, m, err)
