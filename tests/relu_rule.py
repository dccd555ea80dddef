"""Comparison rule for the gradients of the ReLU network (supplement, "Simulation details").

The paper's ReLU is a function of a real pre-activation z.  The oracle decides z > 0 on its binary64
sums, the HIP kernels on their binary32 ones, and no two summation orders agree on the sign of a z
that is zero to within rounding.  For such a unit both decisions are valid evaluations of the
paper's formula, and each moves that sample's contribution to the gradient by far more than the
1e-5 the gradients are compared at.  The rule used by every network parity test:

  * recompute the hidden pre-activations of the worker in binary64 (numpy, this file only);
  * a unit (sample n, layer l, unit j) is a CANDIDATE iff |z| <= margin, with
        margin = 16 l 2^-24 sqrt(K_l) (||a_{l-1}(n) o W_l[:, j]||_2 + |b_l[j]|)
    (about twenty standard deviations of a length-K_l binary32 dot product's rounding error, the
    factor l for the error the inputs of layer l carry);
  * the result under test must equal the oracle's gradient within the tolerance after the
    decisions of SOME subset of the candidates are flipped.  The subset is found, not guessed:
    flipping (n, l, j) changes column j of dW_l and db_l[j] by a known vector (a_{l-1}(n), 1) times the
    back-propagated value at that unit, so per column a small least-squares fit of the observed
    difference gives each candidate's coefficient, which must round to 0 or 1; layers are taken
    from the top down and the decided flips' effect on the layers below (a rank-one term each) is
    added to the reference before those layers are fitted.
  * a fitted subset is taken only if it brings the reference closer to the result under test (a fit on
    nearly parallel or vanishing effect vectors can round noise to a flip), per column and overall: the
    empty subset, i.e. the oracle's gradient as it is, is always among the subsets tried;
  * non-candidates are never flipped, and the final comparison is the ordinary one, so a kernel
    error cannot hide behind the rule unless it equals a sum of candidate flips.

Returns how many candidates there were and how many were flipped; the tests print both.
"""
import numpy as np

U32 = 2.0 ** -24


def _layout(dims):
    offW, offB, off = [], [], 0
    for l in range(len(dims) - 1):
        offW.append(off)
        off += dims[l] * dims[l + 1]
        offB.append(off)
        off += dims[l + 1]
    return offW, offB, off


def forward64(theta, Xm, dims):
    """Binary64 forward pass of one worker's shard: activations a[0..L-1] entering each layer,
    pre-activations z[0..L-1] (z[L-1] = logits), weights W[l], biases b[l]."""
    offW, offB, p = _layout(dims)
    th = np.asarray(theta, np.float64)
    L = len(dims) - 1
    W = [th[offW[l]:offW[l] + dims[l] * dims[l + 1]].reshape(dims[l], dims[l + 1]) for l in range(L)]
    b = [th[offB[l]:offB[l] + dims[l + 1]] for l in range(L)]
    a = [np.asarray(Xm[:, :dims[0]], np.float64)]
    z = []
    for l in range(L):
        z.append(a[l] @ W[l] + b[l])
        if l + 1 < L:
            a.append(np.maximum(z[l], 0.0))
    return a, z, W, b


def candidate_units(a, z, W, b, dims):
    """Boolean [N_m][d_l] per hidden layer l = 1..L-1 (index l - 1): |z| <= margin."""
    out = []
    for l in range(1, len(dims) - 1):
        K = dims[l - 1]
        spread = np.sqrt((a[l - 1] ** 2) @ (W[l - 1] ** 2)) + np.abs(b[l - 1])
        margin = 16.0 * l * U32 * np.sqrt(K) * spread
        out.append(np.abs(z[l - 1]) <= margin)
    return out


def reconcile(g, g_ref, theta, Xm, ym, dims, N_total):
    """g: gradient under test, g_ref: the oracle's, both [p] for one worker whose shard is (Xm, ym).
    Returns (g_adj, n_candidates, n_flipped): the oracle's gradient with the decisions of the
    candidates that the result under test took the other way flipped."""
    dims = tuple(int(d) for d in dims)
    offW, offB, p = _layout(dims)
    L = len(dims) - 1
    g = np.asarray(g, np.float64)
    g_adj = np.asarray(g_ref, np.float64).copy()
    if L < 2:
        return g_adj, 0, 0
    a, z, W, b = forward64(theta, Xm, dims)
    cands = candidate_units(a, z, W, b, dims)
    n_cand = int(sum(c.sum() for c in cands))
    if n_cand == 0:
        return g_adj, 0, 0
    # residuals of the class layer
    zl = z[L - 1] - z[L - 1].max(axis=1, keepdims=True)
    P = np.exp(zl)
    P /= P.sum(axis=1, keepdims=True)
    dz_next = P
    dz_next[np.arange(len(ym)), np.asarray(ym)] -= 1.0          # dZ_L
    inv_N = 1.0 / float(N_total)
    n_flip = 0
    masks = [zz > 0.0 for zz in z[:L - 1]]                      # the oracle's decisions
    # extra[l] (sparse rows): change of dZ_l caused by flips decided in the layers above
    for l in range(L - 1, 0, -1):                               # hidden layer l, weights W[l-1]
        da = dz_next @ W[l].T                                   # [N_m][d_l], with the flips above applied
        cand = cands[l - 1]
        flips = []
        for j in np.unique(np.nonzero(cand)[1]):
            rows = np.nonzero(cand[:, j])[0]
            # effect of flipping (n, j): +-(a_{l-1}(n), 1) da[n][j] / N on (dW_l[:, j], db_l[j])
            sign = np.where(masks[l - 1][rows, j], -1.0, 1.0)
            coef = sign * da[rows, j] * inv_N
            V = np.concatenate([a[l - 1][rows].T, np.ones((1, len(rows)))], axis=0) * coef     # [K+1][k]
            colW = offW[l - 1] + np.arange(dims[l - 1]) * dims[l] + j
            idx = np.concatenate([colW, [offB[l - 1] + j]])
            delta = g[idx] - g_adj[idx]
            c, *_ = np.linalg.lstsq(V, delta, rcond=None)
            take = np.rint(np.clip(c, 0.0, 1.0)).astype(bool)
            # a fit on nearly parallel or vanishing effect vectors can round noise to a flip: a subset is
            # taken only if it brings the column closer to the result under test
            if take.any() and np.abs(delta - V[:, take].sum(axis=1)).max() >= np.abs(delta).max():
                take[:] = False
            for r, t in zip(rows, take):
                if t:
                    flips.append((int(r), int(j)))
            g_adj[idx] += V[:, take].sum(axis=1)
        # apply the decided flips of this layer, then pass dZ_l down
        m = masks[l - 1].copy()
        for (n, j) in flips:
            m[n, j] = ~m[n, j]
        n_flip += len(flips)
        dz_l = np.where(m, da, 0.0)
        # effect of this layer's flips on every layer below: rank-one terms per flipped sample
        if flips and l > 1:
            dz_old = np.where(masks[l - 1], da, 0.0)
            ddz = {}                                            # sample -> change of dZ_l row
            for (n, j) in flips:
                ddz.setdefault(n, np.zeros(dims[l]))[j] = dz_l[n, j] - dz_old[n, j]
            for n, row in ddz.items():
                d = row
                for ll in range(l - 1, 0, -1):                  # layer ll's pre-activation gradient
                    d = np.where(masks[ll - 1][n], W[ll] @ d, 0.0)
                    sl = slice(offW[ll - 1], offW[ll - 1] + dims[ll - 1] * dims[ll])
                    g_adj[sl] += (np.outer(a[ll - 1][n], d) * inv_N).reshape(-1)
                    g_adj[offB[ll - 1]:offB[ll - 1] + dims[ll]] += d * inv_N
            # the fits below must see the flips too: they use dz_next -> da of the lower layer
        masks[l - 1] = m
        dz_next = dz_l
    return g_adj, n_cand, n_flip


def assert_network_gradients_close(g, g_ref, theta, Xm, ym, dims, N_total, tag="", rtol=1e-5,
                                   layer_rtol=2e-5, report=None):
    """The network comparison of every parity test: g against the oracle's g_ref for one worker,
    ||g - g_adj||_inf <= rtol ||g_ref||_inf overall and layer_rtol per parameter block, where g_adj
    is g_ref with the candidate decisions reconciled (see the module docstring)."""
    g = np.asarray(g, np.float64)
    scale = np.abs(g_ref).max()
    g_adj, n_cand, n_flip = reconcile(g, g_ref, theta, Xm, ym, dims, N_total)
    if n_flip and np.abs(g - np.asarray(g_ref, np.float64)).max() <= np.abs(g - g_adj).max():
        # the empty subset is at least as close as the fitted one: compare with the oracle as it is
        g_adj, n_flip = np.asarray(g_ref, np.float64), 0
    if report is not None:
        report.append((tag, n_cand, n_flip))
    err = np.abs(g - g_adj).max()
    assert err <= rtol * scale, (tag, "overall", err / scale, n_cand, n_flip)
    off = 0
    for i in range(len(dims) - 1):
        for n in (dims[i] * dims[i + 1], dims[i + 1]):
            seg, ref = g[off:off + n], g_adj[off:off + n]
            sc = np.abs(np.asarray(g_ref)[off:off + n]).max()
            assert np.abs(seg - ref).max() <= layer_rtol * sc, (tag, "block", i, n, n_cand, n_flip)
            off += n
    return n_cand, n_flip
