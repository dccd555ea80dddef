#!/usr/bin/env python3
"""LAQ benchmark on one MI355X.

A step is one LAQ iteration: laq_worker_grads -> laq_quantize_skip ->
laq_server_step (Algorithm 2's loop body for all M workers), on synthetic
inputs already resident in HBM.  The headline line is measured on the largest
single-GPU workload (ReLU network 784-2048-2048-10, M = 32 workers x 8192
samples, p = 5 824 522, b = 4); the other workloads of the study (binary and
multinomial logistic regression, network 784-200-10, their stochastic
variants, Algorithm 1 on the network shapes, and the quantize/skip/aggregate
bandwidth stress with M = 64 x 2^24 synthetic gradients) are timed in the same
run and reported under "workloads" in the same JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--primary-only]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_F32_PEAK_TFLOPS = 157.3   # dense fp32 matrix


def _events(torch, n):
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def _roofline(bound, achieved, peak, unit, traffic=None, kernel=None, note=None):
    d = {"bound": bound, "achieved": round(achieved, 3), "peak": peak, "unit": unit,
         "frac": round(achieved / peak, 4), "traffic": traffic}
    if kernel:
        d["kernel"] = kernel
    if note:
        d["note"] = note
    return d


def kernel_sources_sha():
    """Hash of the HIP sources: counter-measured traffic is only quoted for the kernels it was measured on."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_1909_07588_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            with open(os.path.join(csrc, name), "rb") as f:
                h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def _traffic_table():
    """Counter-measured HBM bytes per launch, written into profiles/ from rocprofv3 --pmc runs
    (FETCH_SIZE, WRITE_SIZE).  The table names the sources it was measured on; after a change of the
    kernels it is not quoted (traffic: null) until it has been measured again."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(path):
        with open(path) as f:
            t = json.load(f)
        if t.get("kernel_sources_sha") == kernel_sources_sha():
            return t
    return {}


def run_model_workload(w, steps, warmup, phase_steps=100, minibatch=0, force=False, min_timed_ms=0.0,
                       inputs=None):
    """Whole-loop rate and per-phase times of a model workload (cfg 1, 2, 3, 5).  minibatch = B > 0
    runs the stochastic variant: every iteration's gradients come from B drawn samples per worker
    (64 index sets, drawn beforehand and resident on the device, used in turn).  force: every worker
    uploads in every round (Algorithm 1, QGD), so the server step aggregates M rows per iteration.
    min_timed_ms: the step count is raised until the timed region is at least that long."""
    import torch
    import laq_synth
    import paper_1909_07588_amd as laq
    dev = "cuda:0"
    X, y, theta0 = inputs if inputs is not None else laq_synth.model_inputs(w)
    ctx = laq.Laq(w.M, w.p, w.b, w.D, w.xi, w.t_bar, w.alpha, device=dev)
    if force:
        ctx.laq_set_mode(laq.MODE_FORCE_UPLOAD)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    Xd, yd = torch.from_numpy(X).to(dev), torch.from_numpy(y).to(dev)
    ctx.laq_set_data(Xd, yd)
    # the samples are fixed for the whole run: laid out once (untimed, like the upload of X itself)
    # for the kernel that reads them in every iteration, where the library has such a layout
    tiled = not minibatch and ctx.laq_tiled_data_bytes() > 0
    if tiled:
        ctx.laq_tile_data()
    theta = torch.from_numpy(theta0.copy()).to(dev)
    G = ctx.alloc_G()
    codes, R, up = ctx.alloc_messages()
    idx_sets = [torch.from_numpy(laq_synth.minibatch_indices(w, minibatch, i)).to(dev)
                for i in range(64)] if minibatch else []
    count = [0]

    def grads():
        if minibatch:
            ctx.laq_worker_grads_minibatch(theta, idx_sets[count[0] % 64], G)
            count[0] += 1
        else:
            ctx.laq_worker_grads(theta, G)

    def step():
        grads()
        ctx.laq_quantize_skip(G, codes, R, up)
        ctx.laq_server_step(codes, R, up, theta)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    if min_timed_ms > 0.0:                           # short iterations: enough of them to time
        e0, e1 = _events(torch, 2)
        e0.record()
        for _ in range(10):
            step()
        e1.record()
        torch.cuda.synchronize()
        warmup += 10
        steps = max(steps, int(min_timed_ms / max(e0.elapsed_time(e1) / 10, 1e-4)) + 1)
    e0, e1 = _events(torch, 2)
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    total_ms = e0.elapsed_time(e1)
    uploads, bits, status = ctx.laq_get_counters()
    assert status == 0, "non-finite radius during the benchmark"

    # per-phase durations (separate, shorter loop with events between the calls)
    n = max(1, min(phase_steps, steps))
    ev = [_events(torch, 4) for _ in range(n)]
    for i in range(n):
        ev[i][0].record()
        grads()
        ev[i][1].record()
        ctx.laq_quantize_skip(G, codes, R, up)
        ev[i][2].record()
        ctx.laq_server_step(codes, R, up, theta)
        ev[i][3].record()
    torch.cuda.synchronize()
    ph = [sum(e[k].elapsed_time(e[k + 1]) for e in ev) / n for k in range(3)]
    uploads_ph, _, _ = ctx.laq_get_counters()
    ph.append(float(uploads_ph.sum() - uploads.sum()) / n)      # uploading workers per iteration of the phase loop
    it_total = warmup + steps
    res = {
        "workload": w.name + (f"_slaq_B{minibatch}" if minibatch else "") + ("_every_worker_uploads" if force else ""),
        "M": w.M, "N_m": w.N_m, "p": w.p,
        "b": w.b, "steps": steps, "x_layout": "tiles of 16 rows (laq_tile_data)" if tiled else "row-major",
        "iterations_per_s": round(steps / (total_ms * 1e-3), 2), "ms_per_step": round(total_ms / steps, 5),
        "phase_ms": {"worker_grads": round(ph[0], 5), "quantize_skip": round(ph[1], 5),
                     "server_step": round(ph[2], 5)},
        "upload_fraction": round(float(uploads.sum()) / (w.M * it_total), 4),
        "uploads_per_iteration_in_phase_loop": round(ph[3], 3),
        "bits_total": int(bits),
        "quantized_gradient_GBps": round(w.M * w.p * 4 / 1e9 / (ph[1] * 1e-3), 1),
    }
    ctx.close()
    return res, ph


def model_rooflines(w, ph, traffic):
    """Rooflines of the three launch groups of a model workload from their measured times; the kernel
    names are the ones the library launches for this model kind and size."""
    out = {}
    elems = w.M * w.p
    x_bytes = w.M * w.N_m * ((w.dims[0] + 3) // 4 * 4) * 4
    if w.kind == 3:
        S = w.M * w.N_m
        d = w.dims
        fwd = sum(2 * S * d[i] * d[i + 1] for i in range(len(d) - 1))
        dA = sum(2 * S * d[i] * d[i + 1] for i in range(1, len(d) - 1))
        flops = 2 * fwd + dA                      # forward + weight gradients + activation gradients
        out["worker_grads"] = _roofline("mfma", flops / (ph[0] * 1e-3) / 1e12, MFMA_F32_PEAK_TFLOPS, "TFLOP/s",
                                        traffic.get(w.name + ":worker_grads"),
                                        "gemm_kernel (v_mfma_f32_32x32x2_f32) / gemm_narrow_kernel (v_mfma_f32_16x16x4_f32) + class_forward_kernel, "
                                        "class_grads_kernel, slab_finish_kernel")
    else:
        gb = (x_bytes + 4 * elems + 4 * w.p) / 1e9   # read X once, read theta, write G
        name = "binlog_grad_kernel" if w.kind == 1 else "softmax_grad_mfma_kernel"
        out["worker_grads"] = _roofline("hbm", gb / (ph[0] * 1e-3), HBM_PEAK_GBS, "GB/s",
                                        traffic.get(w.name + ":worker_grads"), name + " + finish_grad_kernel")
    # after laq_worker_grads the radius is handed over by the gradient kernels: one pass over g and h
    tiles = max(1, -(-(w.p // 8) // 256))
    qk = (f"codes_kernel<{w.b}, solo> (one block per worker, skip rule fused)" if tiles <= 4
          else f"codes_kernel<{w.b}> + decide_kernel") + "; radius from the gradient kernels' epilogues"
    gq = elems * (8 + w.b / 8) / 1e9
    out["quantize_skip"] = _roofline("hbm", gq / (ph[1] * 1e-3), HBM_PEAK_GBS, "GB/s",
                                     traffic.get(w.name + ":quantize_skip"), qk)
    if len(ph) > 3:
        sblocks_small = tiles <= 4
        gs = (ph[3] * w.p * (8 + w.b / 8) + 16 * w.p) / 1e9
        out["server_step"] = _roofline("hbm", gs / (ph[2] * 1e-3), HBM_PEAK_GBS, "GB/s", None,
                                       f"server_kernel<{w.b}, solo>" if sblocks_small
                                       else f"server_kernel<{w.b}> (+ server_finish_kernel on large grids)",
                                       f"{ph[3]:.2f} uploading workers per iteration")
    return out


def run_stress(b, steps, warmup, handover=False):
    """Quantize/skip/aggregate bandwidth stress (synthetic gradients, no model).
    handover: the untimed generator of the gradients also leaves max |g - h| per worker, as a
    gradient kernel's epilogue would (laq_radius_handover); laq_quantize_skip is then one pass."""
    import torch
    import laq_synth
    import paper_1909_07588_amd as laq
    dev = "cuda:0"
    w = laq_synth.workload(4)
    M, p = w.M, w.p
    ctx = laq.Laq(M, p, b, w.D, w.xi, w.t_bar, w.alpha, device=dev)
    G, s, gen = laq_synth.device_gradients(M, p, ctx.p_stride, dev)
    tmp = torch.empty_like(G[0])
    theta = torch.zeros(p, dtype=torch.float32, device=dev)
    codes, R, up = ctx.alloc_messages()
    tq = ts = 0.0
    n_up = 0
    ups = []
    H = ctx.state()["H"] if handover else None
    rmax = torch.zeros((M, 1), dtype=torch.float32, device=dev)
    for it in range(warmup + steps):
        if handover:                                   # part of producing the gradients: not timed
            for m in range(M):
                torch.sub(G[m], H[m], out=tmp)
                rmax[m, 0] = tmp.abs_().max()
            ctx.laq_radius_handover(G, rmax.view(torch.int32))
        ev = _events(torch, 3)
        ev[0].record()
        ctx.laq_quantize_skip(G, codes, R, up)
        ev[1].record()
        ctx.laq_server_step(codes, R, up, theta)
        ev[2].record()
        torch.cuda.synchronize()
        if it >= warmup:
            tq += ev[0].elapsed_time(ev[1])
            ts += ev[1].elapsed_time(ev[2])
            ups.append(int(up.sum().item()))
        laq_synth.device_drift_(G, s, gen, tmp)     # next iteration's gradients (not timed)
    torch.cuda.synchronize()
    tq /= steps
    ts /= steps
    n_up = sum(ups)
    elems = M * p
    alg_q = elems * (8 + b / 8) / 1e9
    alg_s = (n_up / steps) * p * (8 + b / 8) / 1e9 + 16 * p / 1e9
    res = {
        "workload": f"{w.name}_b{b}" + ("_radius_handover" if handover else ""), "M": M, "p": p, "b": b,
        "steps": steps,
        "iterations_per_s": round(1e3 / (tq + ts), 2), "ms_per_step": round(tq + ts, 4),
        "phase_ms": {"quantize_skip": round(tq, 4), "server_step": round(ts, 4)},
        "upload_fraction": round(n_up / (steps * M), 4),
        "quantized_gradient_GBps": round(elems * 4 / 1e9 / (tq * 1e-3), 1),
    }
    ctx.close()
    return res, (alg_q, tq, alg_s, ts)


def pmc_probe():
    """Short fixed sequence for counter collection under `rocprofv3 --pmc`: a 1 GiB device
    copy (calibrates FETCH_SIZE / WRITE_SIZE against a known size), three iterations of the
    bandwidth-stress workload at b = 4, twenty iterations of the multinomial-logistic workload, three of
    the 784-2048-2048-10 network, five of the 784-200-10 network and of its minibatch variant."""
    import torch
    import laq_synth
    import paper_1909_07588_amd as laq
    dev = "cuda:0"
    a = torch.ones(1 << 28, dtype=torch.float32, device=dev)
    c = torch.empty_like(a)
    for _ in range(3):
        c.copy_(a)
    torch.cuda.synchronize()
    del a, c
    w = laq_synth.workload(4)
    ctx = laq.Laq(w.M, w.p, 4, w.D, w.xi, w.t_bar, w.alpha, device=dev)
    G, s, gen = laq_synth.device_gradients(w.M, w.p, ctx.p_stride, dev)
    theta = torch.zeros(w.p, dtype=torch.float32, device=dev)
    codes, R, up = ctx.alloc_messages()
    for _ in range(3):
        ctx.laq_quantize_skip(G, codes, R, up)
        ctx.laq_server_step(codes, R, up, theta)
        laq_synth.device_drift_(G, s, gen)
    torch.cuda.synchronize()
    ctx.close()
    del G
    run_model_workload(laq_synth.workload(2), 20, 2, phase_steps=1)
    run_model_workload(laq_synth.workload(5), 1, 1, phase_steps=1)
    torch.cuda.empty_cache()
    run_model_workload(laq_synth.workload(3), 3, 1, phase_steps=1)                  # 784-200-10: wide tiles, split weight gradient
    ws = laq_synth.workload(3)
    ws.alpha = 0.008
    run_model_workload(ws, 3, 1, phase_steps=1, minibatch=500)                     # its minibatch variant: 64 x 64 tiles
    print("pmc probe done", flush=True)


def _run_fixed_iterations(w, Xd, yd, theta0, b, force, iters):
    """iters whole iterations with b-bit (or exact) messages, skip rule on or off; the counters."""
    import torch
    import paper_1909_07588_amd as laq
    dev = "cuda:0"
    ctx = laq.Laq(w.M, w.p, b, w.D, w.xi, w.t_bar, w.alpha, device=dev)
    if force:
        ctx.laq_set_mode(laq.MODE_FORCE_UPLOAD)
    ctx.laq_set_model(w.kind, w.dims, w.lam)
    ctx.laq_set_data(Xd, yd)
    if ctx.laq_tiled_data_bytes() > 0:
        ctx.laq_tile_data()
    theta = torch.from_numpy(theta0.copy()).to(dev)
    G = ctx.alloc_G()
    codes, R, up = ctx.alloc_messages()
    e0, e1 = _events(torch, 2)
    e0.record()
    for _ in range(iters):
        ctx.laq_worker_grads(theta, G)
        ctx.laq_quantize_skip(G, codes, R, up)
        ctx.laq_server_step(codes, R, up, theta)
    e1.record()
    torch.cuda.synchronize()
    uploads, bits, status = ctx.laq_get_counters()
    row = {"b": int(b), "alpha": w.alpha, "status": int(status), "iterations": iters, "uploads": int(uploads.sum()),
           "uploads_per_worker": [int(u) for u in uploads],
           "upload_fraction": round(float(uploads.sum()) / (iters * w.M), 4),
           "bits": int(bits), "last_dtheta2": float(ctx.state()["dtheta2"][0].item()),
           "ms_per_iteration": round(e0.elapsed_time(e1) / iters, 5)}
    ctx.close()
    return row


def modes_table(iters=500):
    """Table-2-style rows on the multinomial-logistic shapes (synthetic data): the same kernels run as GD
    (exact messages, every worker uploads), QGD (Algorithm 1: b-bit messages, every worker
    uploads), LAG (exact messages, skip rule) and LAQ (Algorithm 2), for a fixed number of
    iterations; uploads, transmitted bits and the final alpha^2 ||nabla||^2."""
    import torch
    import laq_synth
    import paper_1909_07588_amd as laq
    dev = "cuda:0"
    w = laq_synth.workload(2)
    X, y, theta0 = laq_synth.model_inputs(w)
    Xd, yd = torch.from_numpy(X).to(dev), torch.from_numpy(y).to(dev)
    rows = []
    for name, b, force in (("GD", laq.B_EXACT, True), ("QGD", w.b, True), ("LAG", laq.B_EXACT, False),
                           ("LAQ", w.b, False)):
        rows.append(dict({"mode": name}, **_run_fixed_iterations(w, Xd, yd, theta0, b, force, iters)))
    print(json.dumps({"workload": w.name, "alpha": w.alpha, "table": rows}), flush=True)


def sweeps_table(iters=500):
    """The two sweeps announced at the end of Sec. 4, on the smallest workload and the multinomial-logistic shapes (synthetic data):
    LAQ over the number of bits per coordinate, and LAQ beside GD over the level of heterogeneity
    between the workers' shards (laq_synth.heterogeneous); uploads, bits and the final
    alpha^2 ||nabla||^2 after a fixed number of iterations."""
    import torch
    import laq_synth
    import paper_1909_07588_amd as laq
    dev = "cuda:0"
    out = []
    # planted labels and the multinomial-logistic shapes, each at its own step size and at ten times that (the
    # larger steps move the gradients enough for rule (7a) to fire between the forced uploads)
    for cfg, scale_alpha in ((1, 1.0), (1, 10.0), (2, 1.0), (2, 10.0)):
        w = laq_synth.workload(cfg)
        w.alpha = w.alpha * scale_alpha
        X, y, theta0 = laq_synth.model_inputs(w)
        Xd, yd = torch.from_numpy(X).to(dev), torch.from_numpy(y).to(dev)
        bits_rows = [dict({"mode": "LAQ"}, **_run_fixed_iterations(w, Xd, yd, theta0, b, False, iters))
                     for b in (1, 2, 3, 4, 6, 8, 12, 16)]
        het_rows = []
        for level in (0.0, 0.25, 0.5, 1.0):
            Xh, yh = laq_synth.heterogeneous(w, X, y, level)
            Xd, yd = torch.from_numpy(Xh).to(dev), torch.from_numpy(yh).to(dev)
            for name, b, force in (("GD", laq.B_EXACT, True), ("LAQ", w.b, False)):
                het_rows.append(dict({"mode": name, "level": level},
                                     **_run_fixed_iterations(w, Xd, yd, theta0, b, force, iters)))
        out.append({"workload": w.name, "alpha": w.alpha, "bits_sweep": bits_rows,
                    "heterogeneity_sweep": het_rows})
    print(json.dumps({"sweeps": out}), flush=True)


def graph_rate(w, steps):
    """One iteration (the three hot calls) captured into a HIP graph on the context's stream and
    replayed: what the small workloads, whose iterations are chains of launch latencies, gain from it."""
    import torch
    import laq_synth
    import paper_1909_07588_amd as laq
    dev = "cuda:0"
    X, y, theta0 = laq_synth.model_inputs(w)
    side = torch.cuda.Stream(device=dev)             # default priority
    ctx = laq.Laq(w.M, w.p, w.b, w.D, w.xi, w.t_bar, w.alpha, device=dev, stream=side)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        ctx.laq_set_model(w.kind, w.dims, w.lam)
        ctx.laq_set_data(torch.from_numpy(X).to(dev), torch.from_numpy(y).to(dev))
        if ctx.laq_tiled_data_bytes() > 0:
            ctx.laq_tile_data()
        theta = torch.from_numpy(theta0.copy()).to(dev)
        G = ctx.alloc_G()
        codes, R, up = ctx.alloc_messages()
        for _ in range(3):                           # eager first: loads the kernels
            ctx.laq_worker_grads(theta, G)
            ctx.laq_quantize_skip(G, codes, R, up)
            ctx.laq_server_step(codes, R, up, theta)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        ctx.laq_worker_grads(theta, G)
        ctx.laq_quantize_skip(G, codes, R, up)
        ctx.laq_server_step(codes, R, up, theta)
    for _ in range(5):
        graph.replay()
    torch.cuda.synchronize()
    e0, e1 = _events(torch, 2)
    e0.record()
    for _ in range(steps):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    _, _, status = ctx.laq_get_counters()
    assert status == 0
    ctx.close()
    return ms


def _omp_threads():
    return int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))


def cpu_baseline(w, budget_s=12.0, max_iters=1000):
    """The oracle, as it stands, on the host cores.  Small workloads: whole LAQ iterations at full size.
    The large network: the oracle's plain loops need minutes per iteration (8.3 TFLOP in binary64), so
    a bounded part of one iteration is timed and scaled: the gradient of worker 0 on the first
    `rows` samples of its shard (OpenMP over samples; cost is linear in the samples), and one whole
    quantize / skip / aggregate pass of all M workers at full p (every worker uploads, as in the
    first iteration of Algorithm 2)."""
    import numpy as np
    import laq_synth
    import oracle
    oracle.lib()
    host = os.cpu_count() or 1
    if w.kind == 3 and w.M * w.N_m * w.p > 1e12:
        rows = min(w.N_m, 1024)
        w1 = laq_synth.Workload(w.name, w.cfg, w.kind, 1, rows, w.dims, w.p, w.b)
        X, y, theta0 = laq_synth.model_inputs(w1)
        N = w.M * w.N_m
        t0 = time.perf_counter()
        g = oracle.grad_worker(w.kind, theta0, X[0], y[0], w.dims, w.lam, N)
        t_grad = time.perf_counter() - t0
        st = oracle.State(w.M, w.p, w.b, w.D, w.xi, w.t_bar, w.alpha, theta0)
        G = np.empty((w.M, w.p), np.float32)
        for m in range(w.M):                          # stand-ins for the other workers' gradients
            G[m] = g * np.float32(1.0 + 0.01 * m)
        t0 = time.perf_counter()
        out = st.iteration(G, want_codes=False)
        t_rest = time.perf_counter() - t0
        assert out["status"] == 0 and int(out["upload"].sum()) == w.M
        est = t_grad * (w.N_m / rows) * w.M + t_rest
        return {"value": round(1.0 / est, 6), "unit": "iterations/s", "cores": _omp_threads(), "host_cores": host,
                "kind": "oracle",
                "sample": f"{w.name}: gradient of worker 0 on the first {rows} of its {w.N_m} samples "
                          f"({t_grad:.2f} s, scaled by {w.N_m // rows} x {w.M} workers) + one quantize/skip/aggregate "
                          f"pass of all {w.M} workers at p = {w.p}, every worker uploading ({t_rest:.2f} s): "
                          f"estimated {est:.0f} s per iteration; gcc -O2 -ffp-contract=off, OpenMP over samples "
                          f"(gradient) and workers (quantizer)"}
    X, y, theta0 = laq_synth.model_inputs(w)
    st = oracle.State(w.M, w.p, w.b, w.D, w.xi, w.t_bar, w.alpha, theta0)
    t0 = time.perf_counter()
    n = 0
    while n < max_iters and (time.perf_counter() - t0) < budget_s:
        G, _ = oracle.grads_all(w.kind, st.theta, X, y, w.dims, w.lam)
        out = st.iteration(G, want_codes=False)
        assert out["status"] == 0
        n += 1
    dt = time.perf_counter() - t0
    threads = _omp_threads()
    used = min(threads, w.M) if w.kind != 3 else threads
    return {"value": round(n / dt, 4), "unit": "iterations/s", "cores": used, "host_cores": host, "kind": "oracle",
            "sample": f"first {n} iterations of {w.name} (full size, all {w.M} workers), "
                      f"gcc -O2 -ffp-contract=off, OpenMP over workers"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--primary-only", action="store_true", help="skip the other workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU baseline")
    ap.add_argument("--workload", type=int, default=5, choices=[1, 2, 3, 5], help="headline workload")
    ap.add_argument("--pmc-probe", action="store_true", help="short run for rocprofv3 --pmc (no timing)")
    ap.add_argument("--modes-table", action="store_true",
                    help="GD / QGD / LAG / LAQ on the multinomial-logistic shapes: uploads and bits after --steps iterations")
    ap.add_argument("--sweeps-table", action="store_true",
                    help="LAQ over b, and LAQ beside GD over the heterogeneity level, on the logistic shapes")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (all M workers are simulated on one MI355X); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    import laq_synth
    import paper_1909_07588_amd as laq
    laq.lib()                                   # fails loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    if args.pmc_probe:
        pmc_probe()
        return
    if args.modes_table:
        modes_table(args.steps)
        return
    if args.sweeps_table:
        sweeps_table(args.steps)
        return
    traffic = _traffic_table()

    w = laq_synth.workload(args.workload)
    inputs = laq_synth.model_inputs(w)
    res, ph = run_model_workload(w, args.steps, args.warmup, phase_steps=min(args.steps, 100), inputs=inputs)
    roofs = model_rooflines(w, ph, traffic)
    dominant = max(("worker_grads", "quantize_skip", "server_step"), key=lambda k: res["phase_ms"][k])
    workloads = [dict(res, rooflines=roofs)]

    if not args.primary_only:
        if w.kind == 3:
            # the same workload as Algorithm 1 (every worker uploads): the server step with M rows to aggregate
            r, p3 = run_model_workload(w, 4, 1, phase_steps=4, force=True, inputs=inputs)
            workloads.append(dict(r, rooflines=model_rooflines(w, p3, traffic)))
        del inputs
        torch.cuda.empty_cache()
        for cfg in (1, 2, 3, 5):
            if cfg == args.workload:
                continue
            wk = laq_synth.workload(cfg)
            k, wu = (6, 2) if cfg == 5 else (50, 10)
            r, p3 = run_model_workload(wk, k, wu, phase_steps=min(k, 50) if cfg == 5 else 100,
                                       min_timed_ms=0.0 if cfg == 5 else 60.0)
            if cfg != 5:
                # launch-bound iterations: the same three calls replayed from a HIP graph
                r["ms_per_step_hip_graph"] = round(graph_rate(wk, max(200, r["steps"])), 5)
            workloads.append(dict(r, rooflines=model_rooflines(wk, p3, traffic)))
            torch.cuda.empty_cache()
        # Algorithm 1 on the small network
        wk = laq_synth.workload(3)
        r, p3 = run_model_workload(wk, 50, 5, phase_steps=50, force=True, min_timed_ms=60.0)
        workloads.append(dict(r, rooflines=model_rooflines(wk, p3, traffic)))
        # stochastic variant on the multinomial-logistic shapes (Sec. 4: minibatch 500, alpha = 0.008, b = 3)
        ws = laq_synth.workload(2)
        ws.alpha = 0.008
        r, _ = run_model_workload(ws, 500, 10, phase_steps=100, minibatch=500, min_timed_ms=60.0)
        workloads.append(r)
        # ... and on the small network (Sec. 4: minibatch 500, alpha = 0.008, b = 8)
        ws = laq_synth.workload(3)
        ws.alpha = 0.008
        r, _ = run_model_workload(ws, 300, 10, phase_steps=100, minibatch=500, min_timed_ms=60.0)
        workloads.append(r)
        torch.cuda.empty_cache()
        two_pass = "radius_kernel + radius_final_kernel + codes_kernel<%d> + decide_kernel"
        for b in (2, 4, 8):
            r, (alg_q, tq, alg_s, ts) = run_stress(b, 50, 3)
            name = r["workload"]
            r["rooflines"] = {
                "quantize_skip": _roofline("hbm", alg_q / (tq * 1e-3), HBM_PEAK_GBS, "GB/s",
                                           traffic.get(name + ":quantize_skip"), two_pass % b,
                                           "algorithmic bytes 8 + b/8 per worker-element; the radius needs a "
                                           "first full read of g and h, so HBM traffic is about twice that"),
                "server_step": _roofline("hbm", alg_s / (ts * 1e-3), HBM_PEAK_GBS, "GB/s",
                                         traffic.get(name + ":server_step"), "server_kernel<%d> + server_finish_kernel" % b),
            }
            workloads.append(r)
            torch.cuda.empty_cache()
        # the same stress with the radius handed over by the (untimed) producer of the gradients
        r, (alg_q, tq, alg_s, ts) = run_stress(4, 30, 3, handover=True)
        r["rooflines"] = {
            "quantize_skip": _roofline("hbm", alg_q / (tq * 1e-3), HBM_PEAK_GBS, "GB/s", None,
                                       "codes_kernel<4> + decide_kernel",
                                       "single pass: max |g - h| per worker comes with the gradients "
                                       "(laq_radius_handover), as from laq_worker_grads' epilogues; forming it "
                                       "is the producer's work and is not in this figure"),
            "server_step": _roofline("hbm", alg_s / (ts * 1e-3), HBM_PEAK_GBS, "GB/s", None,
                                     "server_kernel<4> + server_finish_kernel"),
        }
        workloads.append(r)
        torch.cuda.empty_cache()

    line = {
        "metric": "LAQ iterations/sec and worker-gradient GB/s quantized (fraction of HBM peak)",
        "value": res["iterations_per_s"], "unit": "iterations/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": res["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "M": w.M, "N_m": w.N_m, "p": w.p, "b": w.b, "D": w.D,
                   "xi": w.xi, "t_bar": w.t_bar, "alpha": w.alpha, "lambda": w.lam},
        "quantized_gradient_GBps": res["quantized_gradient_GBps"],
        "roofline": roofs[dominant],
        "rooflines": roofs,
        "workloads": workloads,
    }
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
