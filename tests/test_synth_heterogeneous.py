"""The heterogeneity knob of the input generator (a stand-in for the sweep announced at the end of
Sec. 4) and what the oracle's Algorithm 2 loop does on it: per-worker behaviour that follows from the
skip rule (7a), checked on the CPU."""
import numpy as np
import pytest

import laq_synth
import oracle


def test_level_zero_returns_the_inputs_and_level_one_spreads_the_shards():
    w = laq_synth.workload(2, 0.02)
    X, y, _ = laq_synth.model_inputs(w)
    X0, y0 = laq_synth.heterogeneous(w, X, y, 0.0)
    assert X0 is X and y0 is y
    Xh, yh = laq_synth.heterogeneous(w, X, y, 1.0)
    F = w.dims[0] - 1
    for m in range(w.M):
        s = np.float32(10.0 ** (-m / (w.M - 1)))
        assert np.array_equal(Xh[m, :, :F], X[m, :, :F] * s)
        assert np.array_equal(Xh[m, :, F], X[m, :, F])              # the bias column stays 1
        assert np.all(yh[m] == m % w.dims[1])                       # level 1: one class per worker
    assert np.array_equal(X, laq_synth.model_inputs(w)[0])          # the inputs were not written to
    Xq, yq = laq_synth.heterogeneous(w, X, y, 0.5)
    frac = np.mean(yq != y)
    assert 0.35 < frac < 0.55                                        # about level * (1 - 1/C)
    with pytest.raises(ValueError):
        laq_synth.heterogeneous(w, X, y, 1.5)


def test_workers_with_small_smoothness_constants_upload_less():
    """With features scaled down a worker's gradient moves less per step, so the left side of (7a)
    shrinks against the same right side: over a run, the worker with the smallest features uploads no
    more often than the one with the largest, and the whole run uploads less than M per iteration."""
    w = laq_synth.workload(1)
    X, y, theta0 = laq_synth.model_inputs(w)
    Xh, yh = laq_synth.heterogeneous(w, X, y, 1.0)
    st = oracle.State(w.M, w.p, w.b, w.D, w.xi, w.t_bar, w.alpha, theta0)
    for _ in range(w.iterations):
        G, _ = oracle.grads_all(w.kind, st.theta, Xh, yh, w.dims, w.lam)
        out = st.iteration(G, want_codes=False)
        assert out["status"] == 0
    up = np.asarray(st.uploads)
    assert up[-1] <= up[0]
    assert up.sum() < w.M * w.iterations
    assert st.bits == up.sum() * (32 + w.b * w.p)
