"""Parity of the HIP path (through the C ABI binding) with the CPU oracle.

Bar: radii, codes, upload masks, the two integer sums, both sides of (7a),
stored quantized gradients, nabla and theta bit-exact when both sides are fed
the same gradients and state; the binary64 history entry alpha^2||nabla||^2
within 4 p 2^-53 relative (its summation order is free); model gradients within 1e-5 of
the largest gradient entry.
"""
import os

import numpy as np
import pytest
import torch

import laq_synth
import oracle
from paper_1909_07588_amd import LaqError
from gpu_common import (DEV, bits_equal, check_model_grads, check_quantize, check_server, make_pair,
                        push_state, to_dev_G)

pytestmark = pytest.mark.gpu


def _random_state(st, rng, scale=1.0):
    """A mid-run state: stored gradients, clocks, error norms, history."""
    M, p = st.M, st.p
    st.H[:] = (rng.standard_normal((M, p)) * scale).astype(np.float32)
    st.nabla[:] = st.H.sum(0)
    st.theta[:] = rng.standard_normal(p).astype(np.float32)
    st.Ehat2[:] = rng.random(M) * 1e-3 * scale ** 2
    st.t[:] = rng.integers(0, st.t_bar + 1, M)
    st.dtheta2[:] = rng.random(st.D) * 1e-4 * scale ** 2


@pytest.mark.parametrize("b", [1, 2, 3, 4, 5, 7, 8, 11, 16])
@pytest.mark.parametrize("M,p", [(1, 1), (2, 7), (3, 8), (2, 9), (10, 50), (4, 2049), (10, 7850)])
def test_one_iteration_from_a_random_state(b, M, p):
    rng = np.random.default_rng(1000 * b + p)
    ctx, st, theta = make_pair(M, p, b, D=4, t_bar=6, alpha=0.05)
    _random_state(st, rng)
    push_state(ctx, st)
    theta.copy_(torch.from_numpy(st.theta))
    # innovations of very different sizes: some workers skip, some upload
    G = (st.H + rng.standard_normal((M, p)).astype(np.float32)
         * (10.0 ** rng.uniform(-4, 0, (M, 1))).astype(np.float32)).astype(np.float32)
    Gd = to_dev_G(ctx, G)
    msgs, _ = check_quantize(ctx, st, Gd, G)
    # repeated call: same answer (the call leaves the state untouched)
    msgs2, _ = check_quantize(ctx, st, Gd, G)
    check_server(ctx, st, theta, msgs, G)


@pytest.mark.parametrize("b,p", [(2, 300_007), (4, (1 << 20) + 5), (8, 1_000_003), (3, 524_288),
                                 # 4096 tiles per worker: thousands of block partials per sum
                                 (4, (1 << 23) + 13), (5, (1 << 23))])
def test_many_tiles_and_ragged_tail(b, p):
    rng = np.random.default_rng(b * 7 + p)
    M = 5
    ctx, st, theta = make_pair(M, p, b, D=10, t_bar=50, alpha=0.01)
    scales = laq_synth.worker_scales(M)
    G = laq_synth.host_gradients(M, p, scales=scales)
    Gd = to_dev_G(ctx, G)
    for it in range(3):
        msgs, _ = check_quantize(ctx, st, Gd, G)
        check_server(ctx, st, theta, msgs, G)
        push_state(ctx, st)            # impose the oracle's history entry (its order-free part)
        G = laq_synth.host_drift(G, it, scales=scales)
        Gd[:, :p].copy_(torch.from_numpy(G))


@pytest.mark.parametrize("M,p,b,D", [(300, 100, 4, 4), (1500, 37, 2, 3), (70, 5000, 8, 300), (257, 4100, 3, 257),
                                     (4096, 21, 3, 2), (4097, 21, 3, 2), (9001, 19, 4, 2), (65535, 9, 1, 1)])
def test_many_workers_and_long_history(M, p, b, D):
    """More workers than one block's threads (the server's list of uploaders is built in several
    passes), more workers than 64 (fewer partial slots each), a history longer than the part of it
    that is staged in LDS; more workers than one round of the server step lists (4096: the sums go
    on across rounds, in ascending worker order), up to the largest M the library accepts."""
    rng = np.random.default_rng(M + p)
    ctx, st, theta = make_pair(M, p, b, D=D, xi=0.5 / D, t_bar=D + 2, alpha=0.05)
    for it in range(3):
        _random_state(st, rng, scale=0.5)
        st.dtheta2[:] = rng.random(D) * 1e-3
        theta.copy_(torch.from_numpy(st.theta))
        push_state(ctx, st)
        scale = (10.0 ** rng.uniform(-3, 0, (M, 1))).astype(np.float32)
        G = (st.H + scale * rng.standard_normal((M, p))).astype(np.float32)
        Gd = to_dev_G(ctx, G)
        msgs, _ = check_quantize(ctx, st, Gd, G)
        check_server(ctx, st, theta, msgs, G)


def test_teacher_forced_run_skips_and_uploads():
    """30 iterations of drifting synthetic gradients: every mask, code and iterate equal."""
    M, p, b = 12, 40_000, 4
    ctx, st, theta = make_pair(M, p, b, D=5, t_bar=8, alpha=0.01)
    scales = laq_synth.worker_scales(M)
    G = laq_synth.host_gradients(M, p, scales=scales)
    Gd = to_dev_G(ctx, G)
    n_up = 0
    for it in range(30):
        msgs, _ = check_quantize(ctx, st, Gd, G)
        out = check_server(ctx, st, theta, msgs, G)
        n_up += int(out["upload"].sum())
        push_state(ctx, st)
        G = laq_synth.host_drift(G, it, scales=scales)
        Gd[:, :p].copy_(torch.from_numpy(G))
    assert M < n_up < 30 * M            # the run exercised both branches
    up, bits, status = ctx.laq_get_counters()
    assert status == 0 and int(up.sum()) == n_up and bits == n_up * (32 + b * p)


def test_free_running_run_stays_on_the_oracle_trajectory():
    """No state is copied: iterates within 1e-5 per iteration; masks reported."""
    M, p, b = 8, 20_000, 8
    ctx, st, theta = make_pair(M, p, b, D=5, t_bar=8, alpha=0.01)
    scales = laq_synth.worker_scales(M)
    G = laq_synth.host_gradients(M, p, scales=scales)
    Gd = to_dev_G(ctx, G)
    msgs = ctx.alloc_messages()
    agree = 0
    for it in range(25):
        ctx.laq_quantize_skip(Gd, *msgs)
        ctx.laq_server_step(*msgs, theta)
        out = st.iteration(G)
        th = theta.cpu().numpy()
        assert np.abs(th - st.theta).max() <= 1e-5 * np.abs(st.theta).max(), it
        agree += int(np.array_equal(msgs[2].cpu().numpy(), out["upload"]))
        G = laq_synth.host_drift(G, it, scales=scales)
        Gd[:, :p].copy_(torch.from_numpy(G))
    assert agree == 25


def test_zero_innovation_and_forced_upload_clock():
    M, p, b = 4, 1000, 4
    rng = np.random.default_rng(3)
    ctx, st, theta = make_pair(M, p, b, D=2, t_bar=3, alpha=0.1)
    _random_state(st, rng)
    st.t[:] = [0, 3, 1, 3]                      # workers 1 and 3 have reached t_bar
    push_state(ctx, st)
    theta.copy_(torch.from_numpy(st.theta))
    G = st.H.copy()                             # zero innovation everywhere
    G[2] += rng.standard_normal(p).astype(np.float32)
    Gd = to_dev_G(ctx, G)
    msgs, ref = check_quantize(ctx, st, Gd, G)
    up = msgs[2].cpu().numpy()
    assert list(up) == [0, 1, 1, 1]
    assert msgs[1].cpu().numpy()[0] == 0.0 and not msgs[0][0].any()
    check_server(ctx, st, theta, msgs, G)


def test_force_upload_mode_is_algorithm_1():
    M, p, b = 6, 3001, 3
    rng = np.random.default_rng(4)
    ctx, st, theta = make_pair(M, p, b, D=3, t_bar=9, alpha=0.02)
    ctx.laq_set_mode(1)
    G = rng.standard_normal((M, p)).astype(np.float32)
    Gd = to_dev_G(ctx, G)
    for it in range(4):
        msgs, _ = check_quantize(ctx, st, Gd, G, force=True)
        assert msgs[2].cpu().numpy().all()
        check_server(ctx, st, theta, msgs, G, force=True)
        push_state(ctx, st)
        G = (G + 1e-3 * rng.standard_normal((M, p))).astype(np.float32)
        Gd[:, :p].copy_(torch.from_numpy(G))


def test_nonfinite_radius_sets_the_status_word():
    M, p, b = 3, 100, 4
    ctx, st, theta = make_pair(M, p, b)
    G = np.ones((M, p), np.float32)
    G[1, 17] = np.inf
    Gd = to_dev_G(ctx, G)
    msgs = ctx.alloc_messages()
    ctx.laq_quantize_skip(Gd, *msgs)
    _, _, status = ctx.laq_get_counters()
    assert status == 4
    assert msgs[2].cpu().numpy()[1] == 0         # the faulty worker is not aggregated


def test_more_tiles_than_blocks_per_worker():
    """p large enough that every block sweeps several tiles of each worker and
    several workers in turn (the launch shape of the full-size workloads)."""
    M, p, b = 3, 5_000_003, 4
    ctx, st, theta = make_pair(M, p, b, D=5, t_bar=10)
    scales = laq_synth.worker_scales(M)
    G = laq_synth.host_gradients(M, p, scales=scales)
    Gd = to_dev_G(ctx, G)
    for it in range(2):
        msgs, _ = check_quantize(ctx, st, Gd, G)
        check_server(ctx, st, theta, msgs, G)
        push_state(ctx, st)
        G = laq_synth.host_drift(G, it, scales=scales)
        Gd[:, :p].copy_(torch.from_numpy(G))


def test_bad_arguments_are_rejected():
    import ctypes as C
    import paper_1909_07588_amd as laq
    L = laq.lib()
    h = C.c_void_p()
    xi = (C.c_float * 2)(0.1, 0.1)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)
    args = lambda **k: [C.byref(h), k.get("M", 2), k.get("p", 100), k.get("b", 4), k.get("D", 2), xi,
                        k.get("t_bar", 5), C.c_float(k.get("alpha", 0.1)),
                        C.c_void_p(ws.data_ptr() + k.get("mis", 0)), k.get("bytes", 1 << 20), None]
    assert L.laq_create(*args(b=0)) == 1
    assert L.laq_create(*args(b=17)) == 1
    assert L.laq_create(*args(M=0)) == 1
    assert L.laq_create(*args(D=6)) == 1        # D <= t_bar
    assert L.laq_create(*args(alpha=0.0)) == 1
    assert L.laq_create(*args(bytes=16)) == 1
    assert L.laq_create(*args(mis=4)) == 1
    assert L.laq_create(*args()) == 0
    assert L.laq_worker_grads(h, None, None) == 2      # no model bound
    assert L.laq_quantize_skip(h, None, None, None, None) == 1
    assert L.laq_destroy(h) == 0


# --------------------------------------------------------------------------- model gradients

def _grad_case(w):
    X, y, theta0 = laq_synth.model_inputs(w)
    rng = np.random.default_rng(w.cfg)
    theta = (theta0 + 0.05 * rng.standard_normal(w.p)).astype(np.float32)
    ctx, st, _ = make_pair(w.M, w.p, w.b, D=w.D, xi=w.xi, t_bar=w.t_bar, alpha=w.alpha, theta0=theta)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    ctx.laq_set_data(torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV))
    th_d = torch.from_numpy(theta).to(DEV)
    Gd = ctx.alloc_G()
    ctx.laq_worker_grads(th_d, Gd)
    torch.cuda.synchronize()
    G_ref, _ = oracle.grads_all(w.kind, theta, X, y, w.dims, w.lam)
    return Gd[:, :w.p].cpu().numpy(), G_ref, (theta, X, y)


@pytest.mark.parametrize("cfg,scale", [(1, 1.0), (2, 0.05), (2, 0.011)])
def test_logistic_gradients_match_the_oracle(cfg, scale):
    w = laq_synth.workload(cfg, scale)
    G, G_ref, _ = _grad_case(w)
    err = np.abs(G - G_ref).max(axis=1) / np.abs(G_ref).max(axis=1)
    assert err.max() <= 1e-5, err


@pytest.mark.parametrize("F,C,N_m,M", [(3, 2, 5, 2), (64, 4, 33, 3), (65, 10, 100, 2), (513, 16, 47, 2),
                                       (1000, 7, 19, 1)])
def test_softmax_gradient_shapes(F, C, N_m, M):
    w = laq_synth.Workload("t", 2, laq_synth.KIND_SOFTMAX, M, N_m, (F, C), F * C, 4)
    G, G_ref, _ = _grad_case(w)
    err = np.abs(G - G_ref).max(axis=1) / np.abs(G_ref).max(axis=1)
    assert err.max() <= 1e-5, err


@pytest.mark.parametrize("F,C", [(100, 3), (256, 10), (300, 16), (512, 5), (600, 10), (785, 10), (1000, 4), (1024, 2)])
def test_softmax_gradient_every_chunk_layout_full_batch_and_minibatch(F, C):
    """Feature counts on both sides of every boundary of the matrix-core kernel's chunk bookkeeping
    (16 waves x 16 columns: 256, 512, 768; 1000 columns fill the 160 KB of LDS to the byte), several tiles
    per block with a ragged last tile, and the
    same shapes through the index list of the stochastic variant (with an out-of-order draw)."""
    M, N_m, B = 8, 1100, 700
    w = laq_synth.Workload("t", 2, laq_synth.KIND_SOFTMAX, M, N_m, (F, C), F * C, 4)
    X, y, theta0 = laq_synth.model_inputs(w)
    rng = np.random.default_rng(F * 31 + C)
    theta_h = (theta0 + 0.05 * rng.standard_normal(w.p)).astype(np.float32)
    ctx, st, _ = make_pair(w.M, w.p, w.b, D=w.D, xi=w.xi, t_bar=w.t_bar, alpha=w.alpha, theta0=theta_h)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    ctx.laq_set_data(torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV))
    theta = torch.from_numpy(theta_h).to(DEV)
    Gd = ctx.alloc_G()
    ctx.laq_worker_grads(theta, Gd)
    torch.cuda.synchronize()
    G_ref, _ = oracle.grads_all(w.kind, theta_h, X, y, w.dims, w.lam)
    G = Gd[:, :w.p].cpu().numpy()
    assert (np.abs(G - G_ref).max(axis=1) / np.abs(G_ref).max(axis=1)).max() <= 1e-5
    idx = laq_synth.minibatch_indices(w, B, 3)
    ctx.laq_worker_grads_minibatch(theta, torch.from_numpy(idx).to(DEV), Gd)
    torch.cuda.synchronize()
    G_ref = oracle.grads_minibatch(w.kind, theta_h, X, y, w.dims, w.lam, idx)
    G = Gd[:, :w.p].cpu().numpy()
    assert (np.abs(G - G_ref).max(axis=1) / np.abs(G_ref).max(axis=1)).max() <= 1e-5
    assert ctx.laq_get_counters()[2] == 0
    # the tiled copy of the same rows: same arithmetic in the same order, so the same bits as the
    # row-major read; the minibatch call still goes through the index list
    ctx.laq_worker_grads(theta, Gd)
    torch.cuda.synchronize()
    G_rows = Gd[:, :w.p].cpu().numpy().copy()
    if ctx.laq_tiled_data_bytes() == 0:              # (F = 1024 does not fit the matrix-core kernel's LDS)
        assert F == 1024
        return
    ctx.laq_tile_data()
    Gd.zero_()
    ctx.laq_worker_grads(theta, Gd)
    torch.cuda.synchronize()
    G_tiled = Gd[:, :w.p].cpu().numpy().copy()
    assert np.array_equal(G_tiled, G_rows)
    G_full, _ = oracle.grads_all(w.kind, theta_h, X, y, w.dims, w.lam)
    assert (np.abs(G_tiled - G_full).max(axis=1) / np.abs(G_full).max(axis=1)).max() <= 1e-5
    ctx.laq_worker_grads_minibatch(theta, torch.from_numpy(idx).to(DEV), Gd)
    torch.cuda.synchronize()
    G = Gd[:, :w.p].cpu().numpy()
    assert (np.abs(G - G_ref).max(axis=1) / np.abs(G_ref).max(axis=1)).max() <= 1e-5


@pytest.mark.parametrize("N_m", [1, 15, 16, 17, 257])
def test_tiled_data_small_and_ragged_shards(N_m):
    """Shards of less than a tile, exactly one tile, and a ragged last tile: the tiled copy pads
    with zero rows, which must not reach the gradient."""
    F, C, M = 785, 10, 3
    w = laq_synth.Workload("t", 2, laq_synth.KIND_SOFTMAX, M, N_m, (F, C), F * C, 3)
    X, y, theta0 = laq_synth.model_inputs(w)
    rng = np.random.default_rng(N_m)
    theta_h = (theta0 + 0.05 * rng.standard_normal(w.p)).astype(np.float32)
    ctx, st, _ = make_pair(w.M, w.p, w.b, D=w.D, xi=w.xi, t_bar=w.t_bar, alpha=w.alpha, theta0=theta_h)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    ctx.laq_set_data(torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV))
    assert ctx.laq_tiled_data_bytes() == M * ((N_m + 15) // 16) * ((F + 15) // 16) * 1024
    ctx.laq_tile_data()
    theta = torch.from_numpy(theta_h).to(DEV)
    Gd = ctx.alloc_G()
    ctx.laq_worker_grads(theta, Gd)
    torch.cuda.synchronize()
    G_ref, _ = oracle.grads_all(w.kind, theta_h, X, y, w.dims, w.lam)
    G = Gd[:, :w.p].cpu().numpy()
    assert (np.abs(G - G_ref).max(axis=1) / np.abs(G_ref).max(axis=1)).max() <= 1e-5


def test_tiled_data_is_a_snapshot_and_set_data_drops_it():
    """After laq_tile_data the gradient kernel reads the copy: a later change of X is seen only after
    the next laq_tile_data, and binding other data drops the copy."""
    M, N_m, F, C = 2, 100, 300, 7
    w = laq_synth.Workload("t", 2, laq_synth.KIND_SOFTMAX, M, N_m, (F, C), F * C, 3)
    X, y, theta0 = laq_synth.model_inputs(w)
    theta_h = (theta0 + 0.05 * np.random.default_rng(5).standard_normal(w.p)).astype(np.float32)
    ctx, st, _ = make_pair(w.M, w.p, w.b, D=w.D, xi=w.xi, t_bar=w.t_bar, alpha=w.alpha, theta0=theta_h)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    Xd, yd = torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV)
    ctx.laq_set_data(Xd, yd)
    ctx.laq_tile_data()
    theta = torch.from_numpy(theta_h).to(DEV)
    Gd = ctx.alloc_G()
    G1, _ = oracle.grads_all(w.kind, theta_h, X, y, w.dims, w.lam)
    X2 = (X * np.float32(0.5)).astype(np.float32)
    G2, _ = oracle.grads_all(w.kind, theta_h, X2, y, w.dims, w.lam)

    def close(Gref):
        ctx.laq_worker_grads(theta, Gd)
        torch.cuda.synchronize()
        G = Gd[:, :w.p].cpu().numpy()
        return (np.abs(G - Gref).max(axis=1) / np.abs(Gref).max(axis=1)).max() <= 1e-5

    Xd.copy_(torch.from_numpy(X2).to(DEV))
    assert close(G1) and not close(G2)              # still the snapshot
    ctx.laq_tile_data()
    assert close(G2)
    Xd.copy_(torch.from_numpy(X).to(DEV))
    ctx.laq_set_data(Xd, yd)                        # drops the copy: reads X again
    assert close(G1)


def test_tile_data_refused_where_no_kernel_reads_tiles():
    w = laq_synth.workload(1)                       # binary logistic regression
    X, y, theta0 = laq_synth.model_inputs(w)
    ctx, st, theta = make_pair(w.M, w.p, w.b, D=w.D, xi=w.xi, t_bar=w.t_bar, alpha=w.alpha, theta0=theta0)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    ctx.laq_set_data(torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV))
    assert ctx.laq_tiled_data_bytes() == 0
    with pytest.raises(LaqError):
        ctx.laq_tile_data()


def test_full_loop_on_the_smallest_workload():
    """Config 1, all four steps on the GPU, teacher-forced: the oracle quantizes
    the GPU's gradients (compared to its own within 1e-5) from the same state."""
    w = laq_synth.workload(1)
    X, y, theta0 = laq_synth.model_inputs(w)
    ctx, st, theta = make_pair(w.M, w.p, w.b, D=w.D, xi=w.xi, t_bar=w.t_bar, alpha=w.alpha, theta0=theta0)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    ctx.laq_set_data(torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV))
    Gd = ctx.alloc_G()
    msgs = ctx.alloc_messages()
    skipped = 0
    for it in range(w.iterations):
        ctx.laq_worker_grads(theta, Gd)
        torch.cuda.synchronize()
        G = Gd[:, :w.p].cpu().numpy()
        G_ref, _ = oracle.grads_all(w.kind, st.theta, X, y, w.dims, w.lam)
        err = np.abs(G - G_ref).max() / np.abs(G_ref).max()
        assert err <= 1e-5, (it, err)
        msgs, _ = check_quantize(ctx, st, Gd, G, msgs)
        out = check_server(ctx, st, theta, msgs, G)
        skipped += int((out["upload"] == 0).sum())
        push_state(ctx, st)
    assert skipped > w.iterations          # lazy aggregation is active on this problem


@pytest.mark.parametrize("dims,N_m,M", [((20, 16, 12, 5), 33, 2), ((30, 7), 50, 3), ((784, 200, 10), 300, 3),
                                        ((130, 257, 129, 10), 259, 2), ((64, 128, 16), 128, 1),
                                        ((784, 512, 256, 10), 512, 2),
                                        # widths of 4, 8 and 12 on the aligned loaders: a contraction shorter
                                        # than one K tile of the matrix kernel
                                        ((8, 12, 4, 5), 64, 2), ((4, 8, 3), 32, 1), ((12, 16, 8, 4, 2), 100, 3)])
def test_mlp_gradients_match_the_oracle(dims, N_m, M):
    w = laq_synth.Workload("t", 3, laq_synth.KIND_MLP, M, N_m, dims, laq_synth.mlp_param_count(dims), 8)
    G, G_ref, (theta, X, y) = _grad_case(w)
    # per worker, overall and every parameter block separately (a small layer cannot hide behind a
    # large one); near-zero pre-activations handled as relu_rule documents
    report = []
    check_model_grads(w, G, G_ref, theta, X, y, report=report)
    print("relu candidates / flips:", sum(r[1] for r in report), sum(r[2] for r in report))


def test_full_loop_on_a_scaled_network_workload():
    """Config 3 at reduced N_m: gradients -> quantize/skip -> server step on the GPU,
    teacher-forced against the oracle for a few iterations."""
    w = laq_synth.workload(3, scale=0.02)
    X, y, theta0 = laq_synth.model_inputs(w)
    ctx, st, theta = make_pair(w.M, w.p, w.b, D=w.D, xi=w.xi, t_bar=w.t_bar, alpha=w.alpha, theta0=theta0)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    ctx.laq_set_data(torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV))
    Gd = ctx.alloc_G()
    msgs = ctx.alloc_messages()
    for it in range(6):
        ctx.laq_worker_grads(theta, Gd)
        torch.cuda.synchronize()
        G = Gd[:, :w.p].cpu().numpy()
        G_ref, _ = oracle.grads_all(w.kind, st.theta, X, y, w.dims, w.lam)
        check_model_grads(w, G, G_ref, st.theta, X, y, tag=f"iteration {it}")
        msgs, _ = check_quantize(ctx, st, Gd, G, msgs)
        check_server(ctx, st, theta, msgs, G)
        push_state(ctx, st)


@pytest.mark.parametrize("b,iters", [(4, 3), (2, 1), (8, 1)])
def test_full_size_stress_shape_all_workers(b, iters):
    """The bandwidth-stress workload at its full size (M = 64, p = 2^24, b = 4, 2, 8), in the launch
    configuration bench.py times: radii, both integer sums, both sides of (7a) and the masks
    of all 64 workers, the packed codes of 6 sampled workers, and one whole server step; the
    third iteration (b = 4) with the radius handed over by the caller (a single pass)."""
    w = laq_synth.workload(4)
    M, p = w.M, w.p
    ctx, st, theta = make_pair(M, p, b, D=w.D, xi=w.xi, t_bar=w.t_bar, alpha=w.alpha)
    Gd, s, gen = laq_synth.device_gradients(M, p, ctx.p_stride, DEV)
    codes, R, up = ctx.alloc_messages()
    rmax = torch.zeros((M, 1), dtype=torch.float32, device=DEV)
    for it in range(iters):
        G = Gd[:, :p].cpu().numpy()
        if it == 2:           # the fourth stress line: the producer of the gradients hands the radius over
            Hd = ctx.state()["H"]
            for m in range(M):
                rmax[m, 0] = (Gd[m] - Hd[m]).abs_().max()
            ctx.laq_radius_handover(Gd, rmax.view(torch.int32))
        ctx.laq_quantize_skip(Gd, codes, R, up)
        torch.cuda.synchronize()
        sview = ctx.state()
        R_h, up_h = R.cpu().numpy(), up.cpu().numpy()
        Sq_h, E2_h = sview["Sq"].cpu().numpy(), sview["E2"].cpu().numpy()
        lhs_h, rhs_h = sview["lhs"].cpu().numpy(), sview["rhs"].cpu().numpy()
        nw = oracle.code_words(p, b)
        sampled = {0, 7, 21, 40, 62, 63}
        for m in range(M):
            o = oracle.quantize(G[m], st.H[m], b, want_vectors=(m in sampled))
            skip, rhs = oracle.skip(o["lhs"], o["E2"], st.Ehat2[m], st.xi, st.dtheta2, st.alpha, M,
                                    st.t[m], st.t_bar)
            assert bits_equal(np.float32(R_h[m]), np.float32(o["R"])), m
            assert int(Sq_h[m]) == o["Sq"] and bits_equal(np.float64(E2_h[m]), np.float64(o["E2"])), m
            assert bits_equal(np.float64(lhs_h[m]), np.float64(o["lhs"])), m
            assert bits_equal(np.float64(rhs_h[m]), np.float64(rhs)), m
            assert int(up_h[m]) == int(not skip), m
            if m in sampled:
                got = codes[m, :nw].cpu().numpy().view(np.uint32)
                assert np.array_equal(got, oracle.pack(o["q"], b)), m
        out = st.iteration(G, want_codes=False)
        ctx.laq_server_step(codes, R, up, theta)
        torch.cuda.synchronize()
        assert np.array_equal(up_h, out["upload"])
        assert bits_equal(theta.cpu().numpy(), st.theta)
        assert bits_equal(sview["nabla"][:p].cpu().numpy(), st.nabla)
        for m in (0, 21, 63):
            assert bits_equal(sview["H"][m, :p].cpu().numpy(), st.H[m]), m
        assert np.allclose(sview["dtheta2"].cpu().numpy(), st.dtheta2, rtol=4.0 * p * 2.0 ** -53, atol=0)
        push_state(ctx, st)
        laq_synth.device_drift_(Gd, s, gen)


def test_largest_network_widths_at_reduced_batch():
    """The 784-2048-2048-10 network of the largest workload at its full layer widths with few samples
    per worker: the class-layer kernels at their real shapes; the matrix kernels on 64 x 64 block tiles
    (so few rows do not fill the chip with 128 x 128 ones; those are reached by the tests below)."""
    dims = (784, 2048, 2048, 10)
    w = laq_synth.Workload("t", 5, laq_synth.KIND_MLP, 2, 192, dims, laq_synth.mlp_param_count(dims), 4)
    G, G_ref, (theta, X, y) = _grad_case(w)
    check_model_grads(w, G, G_ref, theta, X, y)


def _network_case_with_state(w, seed):
    """Gradients of a network workload from a random mid-run state (so the radius the weight-gradient
    epilogues hand over is max |g - h| against non-trivial stored gradients), the oracle's gradients,
    then quantizer + skip rule + server step on the GPU's own gradients against the oracle."""
    X, y, theta0 = laq_synth.model_inputs(w)
    rng = np.random.default_rng(seed)
    theta_h = (theta0 + 0.02 * rng.standard_normal(w.p)).astype(np.float32)
    ctx, st, theta = make_pair(w.M, w.p, w.b, D=w.D, xi=w.xi, t_bar=w.t_bar, alpha=w.alpha, theta0=theta_h)
    st.H[:] = (1e-4 * rng.standard_normal((w.M, w.p))).astype(np.float32)
    st.nabla[:] = st.H.sum(0)
    st.Ehat2[:] = rng.random(w.M) * 1e-9
    st.t[:] = rng.integers(0, w.t_bar + 1, w.M)
    st.dtheta2[:] = rng.random(w.D) * 1e-9
    push_state(ctx, st)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    ctx.laq_set_data(torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV))
    Gd = ctx.alloc_G()
    ctx.laq_worker_grads(theta, Gd)
    torch.cuda.synchronize()
    G = Gd[:, :w.p].cpu().numpy()
    return ctx, st, theta, Gd, G, theta_h, X, y


def test_large_tiles_forward_and_activation_gradient_against_the_oracle():
    """16 384 samples through 768-wide layers: 128 x 6 = 768 block tiles of 128 x 128, the count from which
    the forward products (bias + ReLU epilogue) and the activation-gradient product (ReLU-mask epilogue) of
    the largest workload take their 128 x 128 instantiation; every worker against the oracle, then the
    quantizer on the radius these launches hand over."""
    dims = (64, 768, 768, 10)
    w = laq_synth.Workload("t", 5, laq_synth.KIND_MLP, 2, 8192, dims, laq_synth.mlp_param_count(dims), 4)
    ctx, st, theta, Gd, G, theta_h, X, y = _network_case_with_state(w, 51)
    G_ref, _ = oracle.grads_all(w.kind, theta_h, X, y, w.dims, w.lam)
    report = []
    check_model_grads(w, G, G_ref, theta_h, X, y, report=report)
    print("relu candidates / flips:", sum(r[1] for r in report), sum(r[2] for r in report))
    msgs, _ = check_quantize(ctx, st, Gd, G)
    check_server(ctx, st, theta, msgs, G)


def test_large_tiles_unsplit_weight_gradient_against_the_oracle():
    """1024 x 1024 weights, 12 workers: 8 x 8 x 12 = 768 block tiles of 128 x 128, the count from which the
    per-worker weight-gradient product is not split over the samples and writes its rows of G itself
    (scale, regulariser and block maxima of |g - h| in its epilogue) with the 128 x 128 instantiation, as
    both hidden layers of the largest workload do.  Every worker against the oracle; then the codes, radii
    and decisions from the handed-over radius, bit for bit."""
    dims = (1024, 1024, 10)
    w = laq_synth.Workload("t", 5, laq_synth.KIND_MLP, 12, 128, dims, laq_synth.mlp_param_count(dims), 4)
    ctx, st, theta, Gd, G, theta_h, X, y = _network_case_with_state(w, 52)
    G_ref, _ = oracle.grads_all(w.kind, theta_h, X, y, w.dims, w.lam)
    report = []
    check_model_grads(w, G, G_ref, theta_h, X, y, report=report)
    print("relu candidates / flips:", sum(r[1] for r in report), sum(r[2] for r in report))
    msgs, _ = check_quantize(ctx, st, Gd, G)
    check_server(ctx, st, theta, msgs, G)


def test_ragged_row_tile_of_the_unsplit_weight_gradient_against_the_oracle():
    """784 x 1024 weights, 16 workers: 7 x 8 x 16 = 896 tiles of 128 x 128, so the product is not split over
    the samples and the seventh row tile holds 16 rows of the 128 (three of its four 32-row sub-tiles lie
    wholly outside the output and take no matrix instructions), as in the first layer of the largest
    workload.  N_m = 136 leaves a ragged last K tile.  Every worker against the oracle; then codes, radii
    and decisions from the handed-over block maxima, bit for bit."""
    dims = (784, 1024, 10)
    w = laq_synth.Workload("t", 5, laq_synth.KIND_MLP, 16, 136, dims, laq_synth.mlp_param_count(dims), 4)
    ctx, st, theta, Gd, G, theta_h, X, y = _network_case_with_state(w, 53)
    G_ref, _ = oracle.grads_all(w.kind, theta_h, X, y, w.dims, w.lam)
    report = []
    check_model_grads(w, G, G_ref, theta_h, X, y, report=report)
    print("relu candidates / flips:", sum(r[1] for r in report), sum(r[2] for r in report))
    msgs, _ = check_quantize(ctx, st, Gd, G)
    check_server(ctx, st, theta, msgs, G)


def test_planted_near_zero_preactivations_pass_under_the_relu_rule():
    """Twelve hidden units get a bias that cancels one sample's pre-activation to a fraction of a binary32
    ulp: the sign the kernels' binary32 sums give it is arbitrary, and every disagreement with the oracle's
    binary64 decision moves the gradient far beyond 1e-5.  Under the rule of tests/relu_rule.py (flip a
    subset of the near-zero candidates) the comparison must still pass; the flips found are printed."""
    import relu_rule
    dims = (784, 200, 10)
    w = laq_synth.Workload("t", 3, laq_synth.KIND_MLP, 3, 300, dims, laq_synth.mlp_param_count(dims), 8)
    X, y, theta0 = laq_synth.model_inputs(w)
    rng = np.random.default_rng(77)
    theta_h = (theta0 + 0.02 * rng.standard_normal(w.p)).astype(np.float32)
    W1 = theta_h[:784 * 200].reshape(784, 200).astype(np.float64)
    planted = []
    for j in range(12):
        m, n = j % w.M, 7 + 11 * j
        theta_h[784 * 200 + j] = np.float32(-(X[m, n, :784].astype(np.float64) @ W1[:, j]))
        planted.append((m, n, j))
    ctx, st, theta = make_pair(w.M, w.p, w.b, D=w.D, xi=w.xi, t_bar=w.t_bar, alpha=w.alpha, theta0=theta_h)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    ctx.laq_set_data(torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV))
    Gd = ctx.alloc_G()
    ctx.laq_worker_grads(theta, Gd)
    torch.cuda.synchronize()
    G = Gd[:, :w.p].cpu().numpy()
    G_ref, _ = oracle.grads_all(w.kind, theta_h, X, y, w.dims, w.lam)
    report = []
    check_model_grads(w, G, G_ref, theta_h, X, y, report=report)
    n_cand, n_flip = sum(r[1] for r in report), sum(r[2] for r in report)
    naive = (np.abs(G - G_ref).max(axis=1) / np.abs(G_ref).max(axis=1)).max()
    print(f"planted 12 near-zero pre-activations: {n_cand} candidates, {n_flip} decided the other way by the "
          f"kernels; naive relative error {naive:.2e}")
    assert n_cand >= 12
    if n_flip == 0:                                         # only a flip may break the naive comparison
        assert naive <= 1e-5


@pytest.mark.parametrize("M,p,b,count", [(5, 300_007, 4, 37), (3, 4100, 3, 1), (4, 70_001, 8, 200), (10, 7850, 3, 64),
                                         (3, 700_001, 4, 256), (3, 700_001, 4, 257), (2, 50_000, 2, 1000)])
def test_radius_handed_over_by_the_caller(M, p, b, count):
    """A caller's own producer of gradients leaves block maxima of |g - h| (here: torch ops on the
    library's stored gradients, over an uneven partition of the coordinates); laq_quantize_skip then
    runs without its radius pass and must still give the oracle's codes, radii and decisions."""
    rng = np.random.default_rng(M * 31 + p)
    ctx, st, theta = make_pair(M, p, b, D=5, t_bar=8, alpha=0.02)
    _random_state(st, rng)
    push_state(ctx, st)
    theta.copy_(torch.from_numpy(st.theta))
    G = (st.H + rng.standard_normal((M, p)).astype(np.float32)
         * (10.0 ** rng.uniform(-4, 0, (M, 1))).astype(np.float32)).astype(np.float32)
    Gd = to_dev_G(ctx, G)
    Hd = ctx.state()["H"]
    cuts = np.unique(np.concatenate([[0, p], rng.integers(0, p + 1, count - 1)]))
    while len(cuts) < count + 1:                       # empty parts are fine: their maximum is 0
        cuts = np.sort(np.concatenate([cuts, [p]]))
    d = (Gd[:, :p] - Hd[:, :p]).abs()
    rmax = torch.zeros((M, count), dtype=torch.float32, device=DEV)
    for i in range(count):
        lo, hi = int(cuts[i]), int(cuts[i + 1])
        if hi > lo:
            rmax[:, i] = d[:, lo:hi].amax(dim=1)
    rbits = rmax.view(torch.int32).contiguous()
    ctx.laq_radius_handover(Gd, rbits)
    msgs, _ = check_quantize(ctx, st, Gd, G)
    # the declaration survives a repeated call, and is withdrawn by the server step
    ctx.laq_radius_handover(Gd, rbits)
    msgs, _ = check_quantize(ctx, st, Gd, G, msgs)
    check_server(ctx, st, theta, msgs, G)
    push_state(ctx, st)
    rbits.zero_()                                      # stale values: must not be read any more
    G2 = (st.H + 0.01 * rng.standard_normal((M, p))).astype(np.float32)
    Gd[:, :p].copy_(torch.from_numpy(G2))
    check_quantize(ctx, st, Gd, G2)


def test_radius_handed_over_by_the_gradient_kernels_is_dropped_when_the_state_changes():
    """laq_worker_grads leaves the radius for laq_quantize_skip; overwriting the stored
    gradients through the state view in between must fall back to the radius pass."""
    w = laq_synth.workload(2, scale=0.02)
    X, y, theta0 = laq_synth.model_inputs(w)
    ctx, st, theta = make_pair(w.M, w.p, w.b, D=w.D, xi=w.xi, t_bar=w.t_bar, alpha=w.alpha, theta0=theta0)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    ctx.laq_set_data(torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV))
    Gd = ctx.alloc_G()
    rng = np.random.default_rng(12)
    ctx.laq_worker_grads(theta, Gd)
    torch.cuda.synchronize()
    G = Gd[:, :w.p].cpu().numpy()
    msgs, _ = check_quantize(ctx, st, Gd, G)               # radius from the producer
    st.H[:] = (G + 1e-3 * rng.standard_normal(G.shape)).astype(np.float32)
    st.nabla[:] = st.H.sum(0)
    push_state(ctx, st)                                    # state overwritten behind the library
    msgs, _ = check_quantize(ctx, st, Gd, G)               # must see the new stored gradients
    check_server(ctx, st, theta, msgs, G)
    push_state(ctx, st)                                    # order-free part of the history entry
    # a copy of G at another address: no hand-over either
    G2 = Gd.clone()
    ctx.laq_worker_grads(theta, Gd)
    torch.cuda.synchronize()
    Gn = Gd[:, :w.p].cpu().numpy()
    G2.copy_(Gd)
    check_quantize(ctx, st, G2, Gn)


def test_radius_of_the_gradient_kernels_survives_a_quantizer_call_on_other_gradients():
    """laq_worker_grads(G1), laq_quantize_skip(G2), laq_quantize_skip(G1), at a size where both the
    producer's block maxima and the radius pass's (each more than 256 per worker) are finished into
    a per-worker radius: the call on G2 must not disturb the radius handed over for G1."""
    dims = (784, 700, 10)                               # p = 556 510: 272 blocks per worker in the radius pass
    w = laq_synth.Workload("t", 3, laq_synth.KIND_MLP, 4, 96, dims, laq_synth.mlp_param_count(dims), 8)
    X, y, theta0 = laq_synth.model_inputs(w)
    ctx, st, theta = make_pair(w.M, w.p, w.b, D=w.D, xi=w.xi, t_bar=w.t_bar, alpha=w.alpha, theta0=theta0)
    rng = np.random.default_rng(31)
    st.H[:] = (1e-3 * rng.standard_normal((w.M, w.p))).astype(np.float32)
    st.nabla[:] = st.H.sum(0)
    push_state(ctx, st)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    ctx.laq_set_data(torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV))
    G1d = ctx.alloc_G()
    ctx.laq_worker_grads(theta, G1d)
    torch.cuda.synchronize()
    G1 = G1d[:, :w.p].cpu().numpy()
    G2 = (st.H + 100.0 * rng.standard_normal((w.M, w.p)).astype(np.float32)).astype(np.float32)   # far larger radii
    G2d = to_dev_G(ctx, G2)
    check_quantize(ctx, st, G2d, G2)
    msgs, _ = check_quantize(ctx, st, G1d, G1)           # still the radius of G1
    check_quantize(ctx, st, G2d, G2)
    msgs, _ = check_quantize(ctx, st, G1d, G1, msgs)
    check_server(ctx, st, theta, msgs, G1)


def test_withdrawn_handover_after_an_edit_of_the_gradients_in_place():
    """A caller that changes G after laq_worker_grads (here: clipping) withdraws the hand-over with
    count = 0; the quantizer then takes the radius of the gradients as they are."""
    w = laq_synth.workload(2, scale=0.02)
    X, y, theta0 = laq_synth.model_inputs(w)
    ctx, st, theta = make_pair(w.M, w.p, w.b, D=w.D, xi=w.xi, t_bar=w.t_bar, alpha=w.alpha, theta0=theta0)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    ctx.laq_set_data(torch.from_numpy(X).to(DEV), torch.from_numpy(y).to(DEV))
    Gd = ctx.alloc_G()
    ctx.laq_worker_grads(theta, Gd)
    clip = float(Gd.abs().max().item()) * 0.25
    Gd.clamp_(-clip, clip)
    ctx.laq_radius_handover(Gd, None)
    torch.cuda.synchronize()
    G = Gd[:, :w.p].cpu().numpy()
    msgs, _ = check_quantize(ctx, st, Gd, G)
    assert float(msgs[1].max().item()) <= clip
    check_server(ctx, st, theta, msgs, G)
