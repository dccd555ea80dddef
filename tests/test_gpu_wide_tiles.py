"""Layers between 129 and 224 units wide take block tiles that span the whole layer width.  Which
GEMM of the network uses them depends on the number of samples and workers (the forward and
activation-gradient products need enough rows of tiles to occupy the chip, the weight gradients
either many workers or shards long enough to split), so these cases choose M, N_m and the widths to
reach every one of those launches, with and without 16-byte aligned operands, and compare the
gradients with the oracle (all workers where that takes seconds, sampled workers otherwise)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
import laq_synth
import oracle
from gpu_common import DEV, check_model_grads, make_pair

pytestmark = pytest.mark.gpu


def _gradients(w, seed):
    X, y, theta0 = laq_synth.model_inputs(w)
    rng = np.random.default_rng(seed)
    theta = (theta0 + 0.05 * rng.standard_normal(w.p)).astype(np.float32)
    ctx, _, _ = make_pair(w.M, w.p, w.b, D=w.D, xi=w.xi, t_bar=w.t_bar, alpha=w.alpha, theta0=theta)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    ctx.laq_set_data(torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV))
    Gd = ctx.alloc_G()
    ctx.laq_worker_grads(torch.from_numpy(theta).to(DEV), Gd)
    torch.cuda.synchronize()
    return Gd[:, :w.p].cpu().numpy(), theta, X, y


@pytest.mark.parametrize("dims,M,N_m", [((36, 200, 160, 10), 8, 4100),     # aligned: fast loaders; tiles 208 and 160 wide
                                        ((37, 190, 150, 7), 8, 4099),      # ragged: generic loaders
                                        ((48, 224, 176, 10), 8, 2100)])    # tiles 224 and 192 wide, no column past the edge / 16 past it
def test_many_samples_forward_backward_and_split_weight_gradients(dims, M, N_m):
    w = laq_synth.Workload("t", 3, laq_synth.KIND_MLP, M, N_m, dims, laq_synth.mlp_param_count(dims), 8)
    G, theta, X, y = _gradients(w, 21)
    ref = {m: oracle.grad_worker(w.kind, theta, X[m], y[m], w.dims, w.lam, M * N_m) for m in (0, M - 1)}
    check_model_grads(w, G, ref, theta, X, y, workers=(0, M - 1))       # overall and per parameter block


@pytest.mark.parametrize("dims,M,N_m", [((1024, 200, 10), 96, 16), ((1022, 190, 10), 96, 15)])
def test_many_workers_unsplit_weight_gradients(dims, M, N_m):
    w = laq_synth.Workload("t", 3, laq_synth.KIND_MLP, M, N_m, dims, laq_synth.mlp_param_count(dims), 8)
    G, theta, X, y = _gradients(w, 22)
    G_ref, _ = oracle.grads_all(w.kind, theta, X, y, w.dims, w.lam)
    check_model_grads(w, G, G_ref, theta, X, y)
