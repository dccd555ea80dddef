"""Pins for the oracle's skip rule, server update and Algorithm 2 loop.

The reductions use a least-squares problem whose gradient is written here in
numpy float64, and comparison loops (GD, lazy aggregation, QGD) written here
from the paper's equations -- none of them calls the oracle's iteration.
"""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


class LeastSquares:
    """f_m(theta) = (1/(2N)) ||A_m theta - y_m||^2, heterogeneous over workers."""

    def __init__(self, M=5, n=40, p=24, seed=3):
        rng = np.random.default_rng(seed)
        self.M, self.p, self.N = M, p, M * n
        scale = 1.0 + np.arange(M)[:, None, None] * 0.7
        self.A = rng.standard_normal((M, n, p)) * scale
        self.y = rng.standard_normal((M, n))
        H = sum(a.T @ a for a in self.A) / self.N
        self.Lsmooth = float(np.linalg.eigvalsh(H).max())
        self.theta_star = np.linalg.solve(H, sum(a.T @ y for a, y in zip(self.A, self.y)) / self.N)

    def grads(self, theta):
        th = np.asarray(theta, np.float64)
        return np.stack([a.T @ (a @ th - y) / self.N for a, y in zip(self.A, self.y)])

    def loss(self, theta):
        th = np.asarray(theta, np.float64)
        return sum(0.5 * np.sum((a @ th - y) ** 2) for a, y in zip(self.A, self.y)) / self.N


def _run_laq(prob, b, xi, alpha, iters, D=5, t_bar=20, force=False, theta0=None):
    th0 = np.zeros(prob.p, np.float32) if theta0 is None else theta0
    st = oracle.State(prob.M, prob.p, b, D, xi, t_bar, alpha, th0)
    hist = []
    for _ in range(iters):
        G = prob.grads(st.theta).astype(np.float32)
        theta_before = st.theta.copy()
        out = st.iteration(G, force_upload=force)
        assert out["status"] == oracle.OK
        hist.append(dict(theta_before=theta_before, theta=st.theta.copy(), H=st.H.copy(),
                         nabla=st.nabla.copy(), t=st.t.copy(), G=G, **out))
    return st, hist


# --------------------------------------------------------------------------- skip rule

def test_skip_rule_scalar_cases():
    xi = np.array([0.5, 0.25], np.float32)
    d2 = np.array([8.0, 16.0])
    alpha, M = 0.5, 2
    # rhs = (1/(0.25*4)) * (0.5*8 + 0.25*16) + 3*(1 + 2) = 8 + 9 = 17 (all exact)
    s, rhs = oracle.skip(17.0, 1.0, 2.0, xi, d2, alpha, M, 0, 10)
    assert rhs == 17.0 and s is True                      # "<=" in (7a): equality skips
    s, _ = oracle.skip(np.nextafter(17.0, 18.0), 1.0, 2.0, xi, d2, alpha, M, 0, 10)
    assert s is False
    s, _ = oracle.skip(0.0, 1.0, 2.0, xi, d2, alpha, M, 10, 10)
    assert s is False                                     # clock reached t_bar: forced upload
    s, _ = oracle.skip(0.0, 1.0, 2.0, xi, d2, alpha, M, 9, 10)
    assert s is True


def test_skip_rule_rhs_matches_extended_precision():
    rng = np.random.default_rng(11)
    for _ in range(50):
        D = int(rng.integers(1, 12))
        xi = rng.random(D).astype(np.float32)
        d2 = rng.random(D) * 10.0 ** rng.integers(-12, 3)
        alpha = np.float32(rng.random() * 0.1 + 1e-3)
        M = int(rng.integers(1, 100))
        E2, Eh = rng.random(2) * 1e-3
        _, rhs = oracle.skip(0.0, E2, Eh, xi, d2, alpha, M, 0, 5)
        ld = np.longdouble
        ref = (np.sum(xi.astype(ld) * d2.astype(ld)) / (ld(alpha) ** 2 * ld(M) ** 2)
               + 3 * (ld(E2) + ld(Eh)))
        assert rhs == pytest.approx(float(ref), rel=1e-14)


# --------------------------------------------------------------------------- reductions

def test_exact_quantizer_and_zero_xi_is_gradient_descent():
    """Remark after eq. 8: enough bits and xi = 0 turn LAQ into GD."""
    prob = LeastSquares()
    alpha = 0.5 / prob.Lsmooth
    _, hist = _run_laq(prob, oracle.B_EXACT, 0.0, alpha, 60)
    th = np.zeros(prob.p)
    a = float(np.float32(alpha))
    for k, rec in enumerate(hist):
        th = th - a * prob.grads(th).sum(0)                # eq. 2
        assert rec["upload"].all()
        err = np.abs(rec["theta"] - th).max() / np.abs(th).max()
        assert err < 1e-5, (k, err)
    assert prob.loss(hist[-1]["theta"]) - prob.loss(prob.theta_star) < 1e-3 * prob.loss(np.zeros(prob.p))


def test_exact_quantizer_is_lazily_aggregated_gradient():
    """b -> infinity leaves lazy aggregation of unquantized gradients: same
    criterion with the eps terms gone."""
    prob = LeastSquares(seed=8)
    alpha = np.float32(0.5 / prob.Lsmooth)
    D, t_bar, xi = 5, 20, 0.16
    _, hist = _run_laq(prob, oracle.B_EXACT, xi, alpha, 80, D=D, t_bar=t_bar)
    # separately written lazy-aggregation loop (float64), fed the same fp32
    # gradients; its own decisions are compared wherever (7a) is not a near-tie
    M, p = prob.M, prob.p
    th = np.zeros(p)
    ghat = np.zeros((M, p))
    nab = np.zeros(p)
    t = np.full(M, t_bar)
    d2 = np.zeros(D)
    a = float(alpha)
    xi_ = float(np.float32(xi))
    n_skip = 0
    agree = 0
    for k, rec in enumerate(hist):
        g = rec["G"].astype(np.float64)
        thr = xi_ * d2.sum() / (a * a * M * M)
        inn = np.array([np.sum((g[m] - ghat[m]) ** 2) for m in range(M)])
        up = (t >= t_bar) | (inn > thr)
        clear = np.abs(inn - thr) > 1e-3 * max(thr, 1e-300)
        assert np.array_equal(up[clear], rec["upload"].astype(bool)[clear]), k
        agree += int(np.array_equal(up, rec["upload"].astype(bool)))
        up = rec["upload"].astype(bool)                    # stay on the same trajectory
        for m in range(M):
            if up[m]:
                nab += g[m] - ghat[m]
                ghat[m] = g[m]
                t[m] = 0
            else:
                t[m] += 1
                n_skip += 1
        step = a * nab
        th = th - step
        d2 = np.roll(d2, 1)
        d2[0] = np.sum(step ** 2)
        err = np.abs(rec["theta"] - th).max() / np.abs(th).max()
        assert err < 2e-5, (k, err)
        assert np.array_equal(rec["H"], ghat.astype(np.float32))
    assert n_skip > 40          # the rule does skip
    assert agree >= len(hist) - 2


@pytest.mark.parametrize("b", [2, 4, 8])
def test_forced_uploads_give_algorithm_1(b):
    """M^k = M turns eq. 4 into QGD: theta^{k+1} = theta^k - alpha sum_m Q_m(theta^k)."""
    prob = LeastSquares(seed=4)
    alpha = np.float32(0.4 / prob.Lsmooth)
    _, hist = _run_laq(prob, b, 0.08, alpha, 40, force=True)
    Q = np.zeros((prob.M, prob.p), np.float64)            # Q_m(theta^{k-1})
    L = 2 ** b - 1
    for k, rec in enumerate(hist):
        assert rec["upload"].all()
        R = rec["R"].astype(np.float64)
        Q = Q + (2 * (R / L))[:, None] * rec["q"].astype(np.float64) - R[:, None]   # eq. 6
        th = rec["theta_before"].astype(np.float64) - float(alpha) * Q.sum(0)        # eq. 3
        assert np.abs(rec["theta"] - th).max() <= 1e-5 * np.abs(th).max()
        assert np.abs(rec["H"] - Q).max() <= 1e-5 * np.abs(Q).max()


# --------------------------------------------------------------------------- invariants

@pytest.mark.parametrize("b", [3, 8])
def test_server_aggregate_equals_sum_of_stored_quantized_gradients(b):
    """nabla^k = sum_m Q_m(theta_hat_m^k) (text after eq. 4 and eq. 8a)."""
    prob = LeastSquares(seed=5)
    alpha = np.float32(0.5 / prob.Lsmooth)
    _, hist = _run_laq(prob, b, 0.16, alpha, 120, t_bar=15)
    skipped = 0
    for rec in hist:
        s = rec["H"].astype(np.float64).sum(0)
        # incremental fp32 sum of the innovations: rounding is relative to the
        # summands (per-worker gradients), which stay large while their sum decays
        assert np.abs(rec["nabla"] - s).max() <= 1e-5 * np.abs(rec["H"]).max()
        skipped += int((rec["upload"] == 0).sum())
        # theta^{k+1} = theta^k - alpha nabla^k
        th = rec["theta_before"].astype(np.float64) - float(alpha) * rec["nabla"].astype(np.float64)
        assert np.abs(rec["theta"] - th).max() <= 1e-6 * np.abs(th).max()
    assert skipped > 100


def test_skipping_workers_keep_their_stored_gradient_and_uploaders_replace_it():
    prob = LeastSquares(seed=6)
    alpha = np.float32(0.5 / prob.Lsmooth)
    _, hist = _run_laq(prob, 4, 0.16, alpha, 60, t_bar=15)
    prev_H = np.zeros_like(hist[0]["H"])
    prev_t = np.full(prob.M, 15)
    for rec in hist:
        for m in range(prob.M):
            if rec["upload"][m]:
                hq = oracle.quantize(rec["G"][m], prev_H[m], 4)
                assert np.array_equal(rec["H"][m], hq["h_new"])
                assert rec["t"][m] == 0
            else:
                assert np.array_equal(rec["H"][m], prev_H[m])
                assert rec["t"][m] == prev_t[m] + 1
        prev_H, prev_t = rec["H"], rec["t"]


def test_first_iteration_is_a_full_round_and_clock_never_exceeds_t_bar():
    prob = LeastSquares(seed=7, M=6)
    alpha = np.float32(0.05 / prob.Lsmooth)          # slow progress: innovations stay small
    t_bar = 4
    st, hist = _run_laq(prob, 8, 0.2, alpha, 80, D=4, t_bar=t_bar)
    assert hist[0]["upload"].all()
    ups = np.stack([r["upload"] for r in hist])
    assert (ups == 0).sum() > 50
    for rec in hist:
        assert rec["t"].max() <= t_bar
    # every worker uploads at least once in any window of t_bar + 1 iterations
    for k in range(len(hist) - t_bar):
        assert ups[k:k + t_bar + 1].sum(0).min() >= 1
    assert np.array_equal(st.uploads, ups.sum(0).astype(np.uint64))


def test_zero_xi_with_quantizer_still_skips_only_inside_the_error_ball():
    """With xi = 0 the rule compares ||deltaQ||^2 with 3(||eps||^2 + ||eps_hat||^2)."""
    prob = LeastSquares(seed=9)
    alpha = np.float32(0.5 / prob.Lsmooth)
    t_bar = 20
    _, hist = _run_laq(prob, 3, 0.0, alpha, 50, t_bar=t_bar)
    assert hist[0]["upload"].all()
    prev_E2 = hist[0]["E2"]                 # eps_hat: error of the last uploaded quantization
    prev_t = hist[0]["t"]
    n_skip = 0
    for rec in hist[1:]:
        assert np.array_equal(rec["rhs"], 3.0 * (rec["E2"] + prev_E2))
        skip = rec["upload"] == 0
        n_skip += int(skip.sum())
        assert np.all(rec["lhs"][skip] <= rec["rhs"][skip])
        up_free = (rec["upload"] == 1) & (prev_t < t_bar)
        assert np.all(rec["lhs"][up_free] > rec["rhs"][up_free])
        prev_E2 = np.where(rec["upload"] == 1, rec["E2"], prev_E2)
        prev_t = rec["t"]
    assert n_skip > 0


# --------------------------------------------------------------------------- bit accounting

def _rows():
    with open(os.path.join(GOLDEN, "table_bits.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                tab, alg, model, up, printed, qz, b, p = line.split()
                yield alg, model, int(up), printed, int(qz), int(b), int(p)


@pytest.mark.parametrize("row", list(_rows()), ids=lambda r: f"{r[0]}-{r[1]}")
def test_bit_accounting_reproduces_the_papers_tables(row):
    """The oracle's counter, driven for a few forced rounds at the row's (b, p)
    per-upload message size, extrapolates to the printed totals."""
    alg, model, ups, printed, qz, b, p = row
    mant, ex = printed.split("e")
    unit = 10.0 ** (int(ex) - 2)                      # one unit in the third digit
    M = 2
    st = oracle.State(M, p, b if qz else oracle.B_EXACT, 1, 0.0, 5, 0.1, np.zeros(p, np.float32))
    rng = np.random.default_rng(1)
    for _ in range(2):
        st.iteration(rng.standard_normal((M, p)).astype(np.float32), want_codes=False,
                     force_upload=True)
    per_upload = st.bits.value // int(st.uploads.sum())
    assert per_upload == (32 + b * p if qz else 32 * p)
    total = ups * per_upload
    slack = 0.51 if model == "network" else 1.01      # logistic p is 7840 or 7850 (bias)
    assert abs(total - float(printed)) <= slack * unit


# --------------------------------------------------------------------------- convergence

def test_loss_residual_decays_geometrically_on_a_strongly_convex_problem():
    """Theorem 1 (qualitative): linear convergence with far fewer uploads than GD."""
    prob = LeastSquares(seed=10, M=8)
    alpha = np.float32(0.5 / prob.Lsmooth)
    st, hist = _run_laq(prob, 4, 0.08, alpha, 400, D=10, t_bar=50)
    f_star = prob.loss(prob.theta_star)
    res = np.array([prob.loss(r["theta"]) - f_star for r in hist])
    assert res[100] < 1e-2 * res[0]
    assert res[399] < 1e-2 * res[100] or res[399] < 1e-10
    assert int(st.uploads.sum()) < 0.8 * prob.M * 400
