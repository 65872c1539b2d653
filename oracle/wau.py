"""Plain fp64 model of the workload analysis unit's decision (Eq. 1, Section 3.2.1), with the ring
all-reduce cost of Section 3.2.3 as the gradient-aggregation term.

TEST INFRASTRUCTURE: only tests/ and bench.py's cpu_baseline leg may import this module; it shares no
code with the HIP package.  Pure Python loops on purpose: every line can be checked against the
equation by eye.

    t_estimate(d) = sum over layers l of { t_c(l, d) + t_s(l, d) },      d = 1 .. G        (Eq. 1)

t_c(l, d) is an input (the measured forward + backward time of layer l at the divided workload, i.e.
at per-GPU minibatch B / d).  The paper takes t_s from the cost of a ring all-reduce, whose traffic per
GPU grows as O(W N) over all GPUs, i.e. each of the d GPUs sends and receives 2 (d - 1) / d of the
gradient's bytes in 2 (d - 1) steps (Section 3.2.3); the reading used here (the paper prints no
formula) is

    t_s(l, d) = 0                                                       for d = 1
              = 2 (d - 1) / d * bytes_l / link_bytes_per_s + 2 (d - 1) * latency_s     otherwise.

The unit picks the d with the smallest estimate among the allowed ones; on an exact tie the smaller d
wins (fewer GPUs for the same speed is the energy argument of Section 3.2.1).
"""
from __future__ import annotations

import math


def t_s(grad_bytes: float, d: int, link_bytes_per_s: float, latency_s: float) -> float:
    if d == 1:
        return 0.0
    return 2.0 * (d - 1) / d * grad_bytes / link_bytes_per_s + 2.0 * (d - 1) * latency_s


def estimate(t_c, grad_bytes, link_bytes_per_s, latency_s, allowed=None):
    """t_c[l][d-1] in seconds, grad_bytes[l]; returns (t_estimate list over d = 1..G with math.inf for
    disallowed d, best d)."""
    n_layers = len(t_c)
    G = len(t_c[0])
    est = []
    for d in range(1, G + 1):
        if allowed is not None and not allowed[d - 1]:
            est.append(math.inf)
            continue
        total = 0.0
        for l in range(n_layers):
            total += float(t_c[l][d - 1]) + t_s(float(grad_bytes[l]), d, link_bytes_per_s, latency_s)
        est.append(total)
    best, best_t = 0, math.inf
    for d in range(1, G + 1):
        if est[d - 1] < best_t:
            best, best_t = d, est[d - 1]
    return est, best
