"""CPU oracle of the analytic profile selector (test infrastructure only; numpy, float64).

KVServe section 3.1 / 3.2 (latency model, Eq. 1), section 6.1: the benefit threshold of a profile
(Eq. 5, Theorem 1) and the piecewise-optimal policy over x = 1/B (Eq. 6, Theorem 2).  Everything
here is the definition written out: no envelope construction, only direct evaluation of the
latency model and exhaustive comparison.

A profile is (cr, s_enc, s_dec): compression ratio V / V_p and the encode / decode throughputs in
bytes of uncompressed KV per second.  Profile index -1 stands for moving the KV uncompressed.
"""
import itertools

import numpy as np


def throughput(p):
    """s_p: harmonic combination of encode and decode throughput (section 3.1)."""
    cr, s_enc, s_dec = p
    return 1.0 / (1.0 / s_enc + 1.0 / s_dec)


def jct(p, V, B, t_model):
    """T_p(c) of Eq. 1; p = None is T_0."""
    if p is None:
        return t_model + V / B
    return t_model + V / throughput(p) + V / (B * p[0])


def benefit_threshold(p):
    """B*_p of Eq. 5."""
    return (1.0 - 1.0 / p[0]) * throughput(p)


def cost(p, x):
    """Linearised cost of Eq. 6 at x = 1/B; p = None is the uncompressed transfer (cost x)."""
    if p is None:
        return x
    return 1.0 / throughput(p) + x / p[0]


def best_profile(profiles, B):
    """Index of the profile with the smallest cost at bandwidth B (-1 = uncompressed).  At an
    exact tie the candidate with the larger compression ratio wins (it is the one that stays
    optimal as the bandwidth drops further); remaining ties go to the lower index."""
    x = 1.0 / B
    cands = [(-1, None)] + list(enumerate(profiles))
    best = None
    for idx, p in cands:
        key = (cost(p, x), -(p[0] if p is not None else 1.0), idx)
        if best is None or key < best[0]:
            best = (key, idx)
    return best[1]


def policy_table(profiles):
    """Piecewise policy of Theorem 2 by exhaustion: every pairwise crossing of two cost lines is a
    possible breakpoint; between consecutive crossings the optimum is constant and is found by
    evaluating all lines at the midpoint.  Returns [(x_from, profile)], x_from ascending, first
    entry at x = 0."""
    lines = [(-1, 0.0, 1.0)] + [(i, 1.0 / throughput(p), 1.0 / p[0]) for i, p in enumerate(profiles)]
    xs = {0.0}
    for (i, a1, b1), (j, a2, b2) in itertools.combinations(lines, 2):
        if b1 != b2:
            x = (a2 - a1) / (b1 - b2)
            if x > 0 and np.isfinite(x):
                xs.add(x)
    xs = sorted(xs)
    table = []
    for k, x0 in enumerate(xs):
        x1 = xs[k + 1] if k + 1 < len(xs) else x0 * 2 + 1.0
        mid = 0.5 * (x0 + x1)
        best = min(lines, key=lambda l: (l[1] + l[2] * mid, l[2], l[0]))[0]
        if not table or table[-1][1] != best:
            table.append((x0, best))
    return table
