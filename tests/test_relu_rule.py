"""The comparison rule for network gradients (tests/relu_rule.py), pinned on the CPU.

A pre-activation that is zero to within binary32 rounding is planted (a bias chosen so that one
sample's z cancels to a fraction of an ulp).  The "other side" is made here, deterministically: the
same gradient with the decision of planted units taken the other way, computed by a separate
binary64 backward pass with explicit masks.  The rule must accept exactly those results, report the
flips it found, and still reject a flipped decision of a unit that is NOT near zero and a plain
numerical error."""
import numpy as np
import pytest

import laq_synth
import oracle
import relu_rule


def _manual_grad(theta, Xm, ym, dims, lam, N_total, flip=()):
    """Binary64 gradient share of one worker with ReLU decisions z > 0, except that the units in
    `flip` (tuples (sample, hidden layer l >= 1, unit)) take the other decision."""
    a, z, W, b = relu_rule.forward64(theta, Xm, dims)
    L = len(dims) - 1
    masks = [zz > 0.0 for zz in z[:L - 1]]
    for (n, l, j) in flip:
        masks[l - 1][n, j] = ~masks[l - 1][n, j]
    zl = z[L - 1] - z[L - 1].max(axis=1, keepdims=True)
    P = np.exp(zl)
    P /= P.sum(axis=1, keepdims=True)
    dz = P
    dz[np.arange(len(ym)), ym] -= 1.0
    parts = [None] * (2 * L)
    for l in range(L, 0, -1):
        parts[2 * (l - 1)] = (a[l - 1].T @ dz).reshape(-1)
        parts[2 * (l - 1) + 1] = dz.sum(axis=0)
        if l > 1:
            dz = np.where(masks[l - 2], dz @ W[l - 1].T, 0.0)
    g = np.concatenate(parts) / N_total
    return g + (len(ym) / N_total) * lam * np.asarray(theta, np.float64)


def _planted_case(dims=(20, 16, 12, 5), N_m=40, seed=5, twin=None):
    """A one-worker network whose units (l = 1, j = 0..3) and (l = 2, j = 0..2) have a pre-activation
    within a fraction of a binary32 ulp of zero for one sample each.  twin = (n_src, n_dst): sample n_dst
    becomes sample n_src scaled by 1 + 2^-22, a second near-zero unit wherever n_src has one in layer 1."""
    w = laq_synth.Workload("t", 3, laq_synth.KIND_MLP, 1, N_m, dims, laq_synth.mlp_param_count(dims), 8)
    X, y, theta0 = laq_synth.model_inputs(w)
    if twin is not None:
        X = X.copy()
        X[0, twin[1]] = X[0, twin[0]] * np.float32(1.0 + 2.0 ** -22)
    rng = np.random.default_rng(seed)
    theta = (theta0 + 0.05 * rng.standard_normal(w.p)).astype(np.float32)
    offW, offB, _ = relu_rule._layout(dims)
    planted = []
    for j in range(4):                                   # layer 1: z = x.W[:, j] + b_j
        n = 3 + 5 * j
        Wj = theta[offW[0]:offW[0] + dims[0] * dims[1]].reshape(dims[0], dims[1])[:, j].astype(np.float64)
        theta[offB[0] + j] = np.float32(-(X[0, n, :dims[0]].astype(np.float64) @ Wj))
        planted.append((n, 1, j))
    a, z, W, b = relu_rule.forward64(theta, X[0], dims)
    for j in range(3):                                   # layer 2, on the activations of the edited layer 1
        n = 4 + 7 * j
        theta[offB[1] + j] = np.float32(-(a[1][n] @ W[1][:, j]))
        planted.append((n, 2, j))
    return w, X[0], y[0], theta, planted


def test_planted_preactivations_are_the_candidates():
    w, Xm, ym, theta, planted = _planted_case()
    a, z, W, b = relu_rule.forward64(theta, Xm, w.dims)
    cands = relu_rule.candidate_units(a, z, W, b, w.dims)
    found = {(int(n), l + 1, int(j)) for l, c in enumerate(cands) for n, j in zip(*np.nonzero(c))}
    assert found == set(planted)
    for (n, l, j) in planted:                            # zero to a fraction of an ulp of the cancelled terms
        assert abs(z[l - 1][n, j]) <= 2.0 ** -24 * np.abs(b[l - 1][j])


def test_manual_backward_agrees_with_the_oracle():
    w, Xm, ym, theta, _ = _planted_case()
    g_ref = oracle.grad_worker(w.kind, theta, Xm, ym, w.dims, w.lam, w.N_m)
    g = _manual_grad(theta, Xm, ym, w.dims, w.lam, w.N_m)
    assert np.abs(g - g_ref).max() <= 1e-6 * np.abs(g_ref).max()    # (g_ref is rounded to binary32)


@pytest.mark.parametrize("subset", [(0,), (5,), (0, 1, 2, 3), (4, 5, 6), (0, 2, 4, 6), (0, 1, 2, 3, 4, 5, 6)])
def test_other_decision_on_planted_units_fails_naively_and_passes_under_the_rule(subset):
    w, Xm, ym, theta, planted = _planted_case()
    g_ref = oracle.grad_worker(w.kind, theta, Xm, ym, w.dims, w.lam, w.N_m)
    flip = [planted[i] for i in subset]
    g_other = _manual_grad(theta, Xm, ym, w.dims, w.lam, w.N_m, flip).astype(np.float32)
    naive = np.abs(g_other - g_ref).max() / np.abs(g_ref).max()
    assert naive > 1e-4                                   # far outside the tolerance: the naive comparison fails
    report = []
    n_cand, n_flip = relu_rule.assert_network_gradients_close(g_other, g_ref, theta, Xm, ym, w.dims, w.N_m,
                                                              report=report)
    assert n_cand == len(planted) and n_flip == len(flip) and report == [("", n_cand, n_flip)]


def test_no_flip_is_reported_when_the_decisions_agree():
    w, Xm, ym, theta, planted = _planted_case()
    g_ref = oracle.grad_worker(w.kind, theta, Xm, ym, w.dims, w.lam, w.N_m)
    g_same = _manual_grad(theta, Xm, ym, w.dims, w.lam, w.N_m).astype(np.float32)
    assert relu_rule.assert_network_gradients_close(g_same, g_ref, theta, Xm, ym, w.dims, w.N_m) == (len(planted), 0)


def test_nearly_parallel_candidates_do_not_turn_noise_into_a_flip():
    """Two candidates of one column whose samples are equal up to a factor 1 + 2^-22: their effect vectors
    are parallel to 2e-7, and a difference of the size of that gap (far inside the tolerance) is fitted
    by coefficients of order one (1 and minus the ratio of the two vectors).  Rounded and clipped that reads as one flip, which would move the
    reference by a whole sample's contribution; the rule must see that the subset does not bring the
    reference closer and compare with the oracle's gradient as it is."""
    w, Xm, ym, theta, planted = _planted_case(twin=(3, 30))
    a, z, W, b = relu_rule.forward64(theta, Xm, w.dims)
    cands = relu_rule.candidate_units(a, z, W, b, w.dims)
    assert cands[0][3, 0] and cands[0][30, 0]            # both samples are candidates of unit 0 in layer 1
    g0 = _manual_grad(theta, Xm, ym, w.dims, w.lam, w.N_m)
    V1 = _manual_grad(theta, Xm, ym, w.dims, w.lam, w.N_m, [(3, 1, 0)]) - g0
    V2 = _manual_grad(theta, Xm, ym, w.dims, w.lam, w.N_m, [(30, 1, 0)]) - g0
    s = (V1 @ V2) / (V2 @ V2)                            # V1 = s V2 up to the gap
    g = g0 + (V1 - s * V2)                               # a gap of 2e-7 |V1|, nothing more
    g_ref = g0.copy()
    assert np.abs(g - g_ref).max() <= 1e-6 * np.abs(g_ref).max() < 1e-2 * np.abs(V1).max()
    n_cand, n_flip = relu_rule.assert_network_gradients_close(g, g_ref, theta, Xm, ym, w.dims, w.N_m)
    assert n_flip == 0


def test_a_flipped_decision_away_from_zero_is_rejected():
    w, Xm, ym, theta, planted = _planted_case()
    g_ref = oracle.grad_worker(w.kind, theta, Xm, ym, w.dims, w.lam, w.N_m)
    a, z, W, b = relu_rule.forward64(theta, Xm, w.dims)
    n, j = np.unravel_index(np.argmax(np.abs(z[0])), z[0].shape)          # the unit farthest from zero
    g_bad = _manual_grad(theta, Xm, ym, w.dims, w.lam, w.N_m, [(int(n), 1, int(j))]).astype(np.float32)
    with pytest.raises(AssertionError):
        relu_rule.assert_network_gradients_close(g_bad, g_ref, theta, Xm, ym, w.dims, w.N_m)
    # also in a column that does hold a candidate: the fit must not absorb it
    n2 = int(np.argmax(np.abs(z[0][:, 0])))
    g_bad = _manual_grad(theta, Xm, ym, w.dims, w.lam, w.N_m, [(n2, 1, 0)]).astype(np.float32)
    with pytest.raises(AssertionError):
        relu_rule.assert_network_gradients_close(g_bad, g_ref, theta, Xm, ym, w.dims, w.N_m)


def test_a_numerical_error_is_rejected():
    w, Xm, ym, theta, planted = _planted_case()
    g_ref = oracle.grad_worker(w.kind, theta, Xm, ym, w.dims, w.lam, w.N_m)
    for at in (0, w.p // 2, w.p - 1):
        g_bad = g_ref.copy()
        g_bad[at] += np.float32(5e-5) * np.abs(g_ref).max()
        with pytest.raises(AssertionError):
            relu_rule.assert_network_gradients_close(g_bad, g_ref, theta, Xm, ym, w.dims, w.N_m)


def test_networks_without_candidates_reduce_to_the_plain_comparison():
    dims = (30, 24, 7)
    w = laq_synth.Workload("t", 3, laq_synth.KIND_MLP, 1, 50, dims, laq_synth.mlp_param_count(dims), 8)
    X, y, theta = laq_synth.model_inputs(w)
    g_ref = oracle.grad_worker(w.kind, theta, X[0], y[0], dims, w.lam, 50)
    assert relu_rule.assert_network_gradients_close(g_ref, g_ref, theta, X[0], y[0], dims, 50) == (0, 0)
    g_bad = g_ref.copy()
    g_bad[7] *= np.float32(1.001)
    if abs(g_bad[7] - g_ref[7]) > 2e-5 * np.abs(g_ref).max():
        with pytest.raises(AssertionError):
            relu_rule.assert_network_gradients_close(g_bad, g_ref, theta, X[0], y[0], dims, 50)
