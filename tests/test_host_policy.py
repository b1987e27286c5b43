"""The library's analytic selector (host code, no GPU) against the oracle of the same passages
(section 6.1, Eq. 5 and 6): thresholds, policy tables and look-ups on seeded random profile sets,
degenerate sets, and the error paths."""
import numpy as np
import pytest

from oracle import policy_ref as pr
from paper_2605_13734_amd import kvc


def random_profiles(rng, n):
    return [(float(rng.uniform(1.05, 12.0)), float(rng.uniform(1e9, 5e12)), float(rng.uniform(1e9, 5e12)))
            for _ in range(n)]


def test_threshold_and_throughput():
    rng = np.random.default_rng(0)
    for p in random_profiles(rng, 100):
        assert kvc.profile_throughput(*p) == pytest.approx(pr.throughput(p), rel=1e-15)
        assert kvc.benefit_threshold(*p) == pytest.approx(pr.benefit_threshold(p), rel=1e-14)


@pytest.mark.parametrize("n", [0, 1, 2, 3, 8, 40])
def test_table_equals_exhaustive_construction(n):
    rng = np.random.default_rng(10 + n)
    for _ in range(30):
        profiles = random_profiles(rng, n)
        rc, got = kvc.policy_build(profiles)
        want = pr.policy_table(profiles)
        assert rc == 0
        assert [g[1] for g in got] == [w[1] for w in want]
        assert np.allclose([g[0] for g in got], [w[0] for w in want], rtol=1e-12, atol=0)
        # look-ups inside the intervals, and the neighbours
        for k, (x0, prof) in enumerate(got):
            x1 = got[k + 1][0] if k + 1 < len(got) else x0 * 2 + 1e-12
            B = 1.0 / (0.5 * (x0 + x1))
            rc, p, more, less = kvc.policy_lookup(got, B)
            assert rc == 0 and p == prof == pr.best_profile(profiles, B)
            assert more == (got[k - 1][1] if k > 0 else prof)
            assert less == (got[k + 1][1] if k + 1 < len(got) else prof)


def test_breakpoint_belongs_to_the_interval_on_its_right():
    profiles = [(2.0, 200.0, 200.0), (4.0, 100.0, 100.0)]        # breakpoints at x = 0.02 and 0.04
    rc, table = kvc.policy_build(profiles)
    assert rc == 0 and [t[1] for t in table] == [-1, 0, 1]
    assert kvc.policy_lookup(table, 1.0 / table[1][0])[1] == 0
    assert kvc.policy_lookup(table, 1.0 / table[2][0])[1] == 1
    assert kvc.policy_lookup(table, 1e30)[1] == -1               # unlimited bandwidth: do not compress


def test_equal_and_dominated_profiles():
    same = (3.0, 1e12, 1e12)
    rc, table = kvc.policy_build([same, same, (3.0, 0.5e12, 1e12), (2.0, 1e11, 1e11)])
    assert rc == 0 and [t[1] for t in table] == [-1, 0]          # lowest index of equals; the rest never wins
    # a profile that does not compress (cr <= 1) can never beat the uncompressed transfer
    rc, table = kvc.policy_build([(1.0, 1e12, 1e12), (0.8, 1e12, 1e12)])
    assert rc == 0 and [t[1] for t in table] == [-1]


def test_errors():
    assert kvc.policy_build([(2.0, -1.0, 1.0)])[0] != 0
    assert kvc.policy_build([(float("nan"), 1.0, 1.0)])[0] != 0
    rc, table = kvc.policy_build([(2.0, 10.0, 10.0)])
    assert kvc.policy_lookup(table, 0.0)[0] != 0
    assert kvc.policy_lookup(table, -5.0)[0] != 0
    import ctypes as C
    count = C.c_int32(0)
    arr = (kvc.Profile * 2)(kvc.Profile(2.0, 10.0, 10.0), kvc.Profile(4.0, 5.0, 5.0))
    small = (kvc.PolicySegment * 1)()
    assert kvc.load().kvc_policy_build(arr, 2, small, 1, C.byref(count)) == -3 and count.value == 3
