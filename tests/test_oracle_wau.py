"""Pins of the workload-analysis oracle (Eq. 1) against what the mathematics fixes: closed forms, limiting
cases and a hand-worked table (tests/golden/wau_hand_example.txt)."""
import math
import os

import numpy as np

from oracle import wau

HERE = os.path.dirname(os.path.abspath(__file__))


def test_single_gpu_has_no_aggregation_cost():
    assert wau.t_s(1e9, 1, 1e9, 1e-3) == 0.0
    est, best = wau.estimate([[3.0], [4.0]], [1e6, 2e6], 1e9, 1e-5)
    assert est == [7.0] and best == 1


def test_ring_allreduce_closed_form():
    # d = 2: each GPU moves exactly the gradient once each way (2 * 1/2 * bytes), two latency steps
    assert math.isclose(wau.t_s(8e6, 2, 4e6, 0.25), 2.0 + 0.5, rel_tol=0, abs_tol=1e-15)
    # d -> large: traffic tends to 2 * bytes / bandwidth
    assert math.isclose(wau.t_s(1e9, 1000, 1e9, 0.0), 2.0 * 999 / 1000, rel_tol=1e-15)
    # traffic term is monotone in d, bounded by 2 * bytes / bw
    prev = 0.0
    for d in range(2, 64):
        cur = wau.t_s(1.0, d, 1.0, 0.0)
        assert prev < cur < 2.0
        prev = cur


def test_perfect_scaling_without_communication_takes_every_gpu():
    G = 8
    t_c = [[10.0 / d for d in range(1, G + 1)], [6.0 / d for d in range(1, G + 1)]]
    est, best = wau.estimate(t_c, [0.0, 0.0], 1e9, 0.0)
    assert best == G
    assert all(math.isclose(est[d - 1], 16.0 / d, rel_tol=1e-15) for d in range(1, G + 1))


def test_no_compute_speedup_keeps_one_gpu():
    # the paper's small-workload case: dividing the minibatch does not shorten the layers, aggregation only adds
    G = 4
    est, best = wau.estimate([[5.0] * G, [1.0] * G], [4e6, 4e6], 1e9, 1e-6)
    assert best == 1
    assert est[0] == 6.0 and all(est[d] > 6.0 for d in range(1, G))


def test_exact_tie_prefers_fewer_gpus_and_disallowed_counts_are_skipped():
    est, best = wau.estimate([[4.0, 4.0, 1.0, 4.0]], [0.0], 1e9, 0.0, allowed=[1, 1, 0, 1])
    assert best == 1 and est[2] == math.inf
    est, best = wau.estimate([[4.0, 3.0, 1.0, 3.0]], [0.0], 1e9, 0.0, allowed=[1, 1, 0, 1])
    assert best == 2


def test_interior_optimum_matches_calculus():
    # t(d) = A / d + 2 (d - 1) c  (latency-dominated aggregation): the continuous minimum is sqrt(A / (2 c))
    A, c, G = 1.0, 0.01, 16
    est, best = wau.estimate([[A / d for d in range(1, G + 1)]], [0.0], 1e9, c)
    d_star = math.sqrt(A / (2 * c))   # 7.07
    assert best in (math.floor(d_star), math.ceil(d_star))
    assert best == min(range(1, G + 1), key=lambda d: A / d + 2 * (d - 1) * c)


def test_hand_worked_example():
    """Two layers, four GPUs, numbers small enough to add by hand (see the golden file for the sums)."""
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "wau_hand_example.txt")) if l.strip() and l[0] != "#"]
    vals = {r[0]: [float(v) for v in r[1:]] for r in rows}
    t_c = [vals["t_c_layer0"], vals["t_c_layer1"]]
    est, best = wau.estimate(t_c, vals["grad_bytes"], vals["link"][0], vals["link"][1])
    assert np.allclose(est, vals["t_estimate"], rtol=0, atol=1e-12)
    assert best == int(vals["best_d"][0])
