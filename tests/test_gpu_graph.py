"""The three hot calls enqueue kernels only (no allocation, no host synchronisation, no memset),
so one LAQ iteration can be captured into a HIP graph on the context's stream and replayed.
Every replay is compared with the oracle, with eager work and synchronisations in between."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
import laq_synth
import oracle
import paper_1909_07588_amd as laq
from gpu_common import DEV, bits_equal

pytestmark = pytest.mark.gpu


def test_one_iteration_captured_and_replayed():
    w = laq_synth.workload(1)
    X, y, theta0 = laq_synth.model_inputs(w)
    side = torch.cuda.Stream(device=DEV)            # default priority
    ctx = laq.Laq(w.M, w.p, w.b, w.D, w.xi, w.t_bar, w.alpha, device=DEV, stream=side)
    st = oracle.State(w.M, w.p, w.b, w.D, w.xi, w.t_bar, w.alpha, theta0)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        ctx.laq_set_model(w.kind, w.dims, w.lam)
        ctx.laq_set_data(torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV))
        theta = torch.from_numpy(theta0.copy()).to(DEV)
        G = ctx.alloc_G()
        codes, R, up = ctx.alloc_messages()
        # one eager iteration first (loads the kernels), checked like the replays below
        def eager():
            ctx.laq_worker_grads(theta, G)
            ctx.laq_quantize_skip(G, codes, R, up)
            ctx.laq_server_step(codes, R, up, theta)
        eager()
    side.synchronize()

    def oracle_step():
        Gh = G[:, :w.p].cpu().numpy()                 # the GPU's own gradients (compared separately)
        G_ref, _ = oracle.grads_all(w.kind, st.theta, X, y, w.dims, w.lam)
        assert np.abs(Gh - G_ref).max() <= 1e-5 * np.abs(G_ref).max()
        out = st.iteration(Gh)
        assert np.array_equal(up.cpu().numpy(), out["upload"])
        assert bits_equal(theta.cpu().numpy(), st.theta)
        s = ctx.state()
        assert bits_equal(s["H"][:, :w.p].cpu().numpy(), st.H)
        # the order-free history entry is re-imposed so that both sides keep the same state
        s["dtheta2"].copy_(torch.from_numpy(st.dtheta2))
        torch.cuda.synchronize()

    oracle_step()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        ctx.laq_worker_grads(theta, G)
        ctx.laq_quantize_skip(G, codes, R, up)
        ctx.laq_server_step(codes, R, up, theta)
    # capture does not execute: state unchanged so far
    for it in range(12):
        graph.replay()
        torch.cuda.synchronize()
        oracle_step()
        if it % 4 == 3:                               # eager iterations between the replays
            with torch.cuda.stream(side):
                eager()
            side.synchronize()
            oracle_step()
    up_cnt, bits, status = ctx.laq_get_counters()
    assert status == 0 and np.array_equal(up_cnt, st.uploads) and bits == st.bits.value
