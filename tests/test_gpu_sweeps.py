"""Parity of the whole loop along the two sweeps announced at the end of Sec. 4: bits per coordinate
and heterogeneity between the workers' shards (laq_synth.heterogeneous).  Teacher-forced as in the
other whole-loop tests: the oracle quantizes the GPU's gradients (within 1e-5 of its own) from the same
state, and codes, masks, radii, stored gradients, nabla and theta are compared bit for bit."""
import numpy as np
import pytest
import torch

import laq_synth
import oracle
from gpu_common import DEV, check_quantize, check_server, make_pair, push_state

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg,scale,level,b,iters", [
    (1, 1.0, 1.0, 1, 60), (1, 1.0, 1.0, 3, 60), (1, 1.0, 0.5, 6, 60), (1, 1.0, 0.25, 12, 60), (1, 1.0, 1.0, 16, 60),
    (2, 0.03, 1.0, 3, 25), (2, 0.03, 0.5, 1, 25), (2, 0.03, 0.25, 8, 25), (2, 0.011, 1.0, 16, 25)])
def test_whole_loop_along_the_bit_and_heterogeneity_sweeps(cfg, scale, level, b, iters):
    w = laq_synth.workload(cfg, scale)
    X, y, theta0 = laq_synth.model_inputs(w)
    X, y = laq_synth.heterogeneous(w, X, y, level)
    ctx, st, theta = make_pair(w.M, w.p, b, D=w.D, xi=w.xi, t_bar=w.t_bar, alpha=w.alpha, theta0=theta0)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    ctx.laq_set_data(torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV))
    if ctx.laq_tiled_data_bytes() > 0:
        ctx.laq_tile_data()
    Gd = ctx.alloc_G()
    msgs = ctx.alloc_messages()
    uploads = np.zeros(w.M, np.int64)
    for it in range(iters):
        ctx.laq_worker_grads(theta, Gd)
        torch.cuda.synchronize()
        G = Gd[:, :w.p].cpu().numpy()
        G_ref, _ = oracle.grads_all(w.kind, st.theta, X, y, w.dims, w.lam)
        err = np.abs(G - G_ref).max() / np.abs(G_ref).max()
        assert err <= 1e-5, (it, err)
        msgs, _ = check_quantize(ctx, st, Gd, G, msgs)
        out = check_server(ctx, st, theta, msgs, G)
        uploads += out["upload"].astype(np.int64)
        push_state(ctx, st)
    got, bits, status = ctx.laq_get_counters()
    assert status == 0
    assert np.array_equal(got.astype(np.int64), uploads)
    assert int(bits) == int(uploads.sum()) * (32 + b * w.p)
    ctx.close()
