"""Host-side behaviour of bench.py and of the workload table that needs no GPU."""
import os
import subprocess
import sys

import laq_synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_workload_table_matches_the_stated_shapes():
    w2 = laq_synth.workload(2)
    assert (w2.M, w2.N_m, w2.dims, w2.p, w2.b, w2.alpha) == (10, 6000, (785, 10), 7850, 3, 0.02)
    w3 = laq_synth.workload(3)
    assert w3.p == 784 * 200 + 200 + 200 * 10 + 10 == 159010 and w3.b == 8
    w5 = laq_synth.workload(5)
    assert w5.p == 5824522 and (w5.M, w5.N_m, w5.b) == (32, 8192, 4)
    w4 = laq_synth.workload(4)
    assert (w4.M, w4.p, w4.t_bar) == (64, 1 << 24, 50)
    for cfg in (1, 2, 3, 4, 5):
        w = laq_synth.workload(cfg)
        assert w.D == 10 and abs(w.xi * w.D - 0.8) < 1e-12       # xi_d = 0.8 / D (supplement, "Parameters")


def test_inputs_are_a_function_of_the_seed_only():
    w = laq_synth.workload(2, 0.01)
    a, b = laq_synth.model_inputs(w), laq_synth.model_inputs(w)
    assert all((x == y).all() for x, y in zip(a, b))
    i0, i1 = laq_synth.minibatch_indices(w, 7, 3), laq_synth.minibatch_indices(w, 7, 3)
    assert (i0 == i1).all() and i0.shape == (w.M, 7)
    assert all(len(set(row)) == 7 and row.min() >= 0 and row.max() < w.N_m for row in i0)
    zero_share = (a[0][:, :, :784] == 0).mean()
    assert 0.78 < zero_share < 0.82                                # about 80 % zero features
