"""The workload analysis unit's decision through the C ABI (host arithmetic, no GPU needed) against the
fp64 oracle: random tables, the oracle's hand-worked example, ties, masks and the error paths."""
import math
import os

import numpy as np
import pytest

from oracle import wau as orc_wau

HERE = os.path.dirname(os.path.abspath(__file__))


def _wap():
    import paper_1811_01532_amd as wap
    wap.lib()
    return wap


def test_matches_oracle_on_random_tables():
    wap = _wap()
    rng = np.random.default_rng([181101532, 900])
    for case in range(200):
        L, G = int(rng.integers(1, 20)), int(rng.integers(1, 17))
        base = rng.uniform(1e-5, 1e-2, L)
        # compute time shrinks with d at a random efficiency, never below a launch floor
        t_c = [[max(base[l] / d ** rng.uniform(0.0, 1.0), 5e-6) for d in range(1, G + 1)] for l in range(L)]
        gb = rng.uniform(0, 4e8, L)
        bw, lat = float(rng.uniform(1e9, 2e11)), float(rng.uniform(0, 5e-5))
        allowed = None if case % 3 else [1] + [int(v) for v in rng.integers(0, 2, G - 1)]
        est_o, best_o = orc_wau.estimate(t_c, gb, bw, lat, allowed)
        best, est = wap.wap_choose_gpus(t_c, gb, bw, lat, allowed)
        assert best == best_o
        for a, b in zip(est, est_o):
            assert (math.isinf(a) and math.isinf(b)) or abs(a - b) <= 1e-12 * max(abs(b), 1e-30)


def test_hand_worked_example_and_tie():
    wap = _wap()
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "wau_hand_example.txt")) if l.strip() and l[0] != "#"]
    vals = {r[0]: [float(v) for v in r[1:]] for r in rows}
    best, est = wap.wap_choose_gpus([vals["t_c_layer0"], vals["t_c_layer1"]], vals["grad_bytes"], *vals["link"])
    assert best == int(vals["best_d"][0]) and np.allclose(est, vals["t_estimate"], rtol=0, atol=1e-12)
    best, est = wap.wap_choose_gpus([[4.0, 4.0, 1.0, 4.0]], [0.0], 1e9, 0.0, allowed=[1, 1, 0, 1])
    assert best == 1 and math.isinf(est[2])


def test_rejects_bad_arguments():
    wap = _wap()
    ok = ([[1.0, 0.5]], [1e6], 1e9, 1e-6)
    for bad in (([[1.0, -0.5]], [1e6], 1e9, 1e-6), ([[1.0, float("nan")]], [1e6], 1e9, 1e-6),
                ([[1.0, 0.5]], [-1.0], 1e9, 1e-6), ([[1.0, 0.5]], [1e6], 0.0, 1e-6),
                ([[1.0, 0.5]], [1e6], 1e9, -1e-6)):
        with pytest.raises(wap.WapError):
            wap.wap_choose_gpus(*bad)
    with pytest.raises(wap.WapError):
        wap.wap_choose_gpus(*ok, allowed=[0, 0])
    assert wap.wap_choose_gpus(*ok)[0] in (1, 2)
