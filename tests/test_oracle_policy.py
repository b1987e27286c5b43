"""Pins for the oracle of the analytic selector (CPU only): the statements of Theorems 1 and 2
checked against the latency model of Eq. 1 evaluated directly, plus a hand-computed table."""
import numpy as np

from oracle import policy_ref as pr


def random_profiles(rng, n):
    return [(float(rng.uniform(1.2, 9.0)), float(rng.uniform(0.5e9, 4e12)), float(rng.uniform(0.5e9, 4e12)))
            for _ in range(n)]


def test_throughput_is_total_time():
    p = (3.2, 3.7e12, 4.1e12)
    V = 10.7e9
    assert abs(V / pr.throughput(p) - (V / p[1] + V / p[2])) < 1e-15


def test_theorem_1_bandwidth_threshold():
    """T_p < T_0 exactly when B < B*_p, whatever V and T_model are (Eq. 1 against Eq. 5)."""
    rng = np.random.default_rng(0)
    for p in random_profiles(rng, 200):
        bstar = pr.benefit_threshold(p)
        V, tm = float(rng.uniform(1e6, 1e11)), float(rng.uniform(0, 5))
        for B in (bstar * 0.5, bstar * 0.99, bstar * 1.01, bstar * 3):
            assert (pr.jct(p, V, B, tm) < pr.jct(None, V, B, tm)) == (B < bstar)


def test_linearised_cost_is_the_latency_model():
    rng = np.random.default_rng(1)
    for p in random_profiles(rng, 50):
        V, tm, B = float(rng.uniform(1e6, 1e11)), float(rng.uniform(0, 5)), float(rng.uniform(1e8, 1e12))
        assert abs((pr.jct(p, V, B, tm) - tm) / V - pr.cost(p, 1.0 / B)) < 1e-9 * pr.cost(p, 1.0 / B)


def test_table_is_optimal_under_eq_1():
    """Within every interval of the table, the listed profile minimises the JCT of Eq. 1."""
    rng = np.random.default_rng(2)
    for n in (1, 2, 5, 12):
        profiles = random_profiles(rng, n)
        table = pr.policy_table(profiles)
        assert table[0][0] == 0.0 and table[0][1] == -1        # infinite bandwidth: do not compress
        for k, (x0, best) in enumerate(table):
            x1 = table[k + 1][0] if k + 1 < len(table) else x0 * 3 + 1e-9
            for x in np.linspace(x0, x1, 7)[1:-1]:
                B = 1.0 / x
                t = [pr.jct(None, 1e9, B, 0.1)] + [pr.jct(p, 1e9, B, 0.1) for p in profiles]
                assert int(np.argmin(t)) - 1 == best
                assert pr.best_profile(profiles, B) == best


def test_hand_computed_table():
    """Two profiles: cr 2 at s = 100 (a = 0.01, b = 0.5) and cr 4 at s = 50 (a = 0.02, b = 0.25).
    Uncompressed (cost x) loses to the first at x = 0.01 / 0.5 = 0.02, the first to the second at
    x = (0.02 - 0.01) / (0.5 - 0.25) = 0.04."""
    profiles = [(2.0, 200.0, 200.0), (4.0, 100.0, 100.0)]
    table = pr.policy_table(profiles)
    assert [t[1] for t in table] == [-1, 0, 1]
    assert np.allclose([t[0] for t in table], [0.0, 0.02, 0.04], rtol=1e-14)
    assert abs(pr.benefit_threshold(profiles[0]) - 50.0) < 1e-12          # (1 - 1/2) * 100 = 1 / 0.02
    assert pr.best_profile(profiles, 1.0 / 0.03) == 0 and pr.best_profile(profiles, 1.0 / 0.05) == 1


def test_dominated_profile_never_appears():
    profiles = [(3.0, 2e12, 2e12), (2.5, 1e12, 1e12)]                     # second: smaller cr and slower
    assert 1 not in [t[1] for t in pr.policy_table(profiles)]
