"""CPU checks of the inequalities behind the exact shortcuts of the GPU scan (early abandon with
remaining minima, list-level pruning): binary32 sums of non-negative table entries, evaluated the
way the kernel evaluates them, against the margins its thresholds carry."""
import numpy as np

U = np.float32(2.0 ** -24)


def seq_sum(values):
    s = np.float32(0.0)
    out = []
    for v in values:
        s = np.float32(s + v)
        out.append(s)
    return out


def test_running_sum_plus_remaining_minimum_bounds_the_finished_sum():
    """s_full >= (s_j + rest_j)(1 - 2 M u): what lets a running sum be tested against
    thr - rest_j once thr carries a relative margin of 5e-5 (M <= 256)."""
    rng = np.random.default_rng(11)
    for M in (8, 32, 120, 192):
        for scale in (1e-3, 1.0, 3e4):
            T = (rng.random((M, 256), dtype=np.float32) ** 3 * np.float32(scale)).astype(np.float32)
            rowmin = T.min(axis=1)
            rest = np.zeros(M + 1, dtype=np.float32)          # rest[j] = binary32 sum of rowmin[j:]
            for j in range(M - 1, -1, -1):
                rest[j] = np.float32(rest[j + 1] + rowmin[j])
            codes = rng.integers(0, 256, size=(200, M))
            for c in codes:
                partial = seq_sum(T[np.arange(M), c])
                full = float(partial[-1])
                for j in range(1, M):
                    lower = (float(partial[j - 1]) + float(rest[j])) * (1.0 - 2.0 * M * float(U))
                    assert full >= lower
            assert 2 * 256 * float(U) < 3.2e-5                # the share of the 5e-5 margin it may use


def test_minimum_over_the_codes_of_a_list_bounds_every_member():
    """Sum over subspaces of the smallest entry among the codes that occur in a list is a lower
    bound of every member's table sum (up to the same roundings), and never below the bound
    from the row minima over all codes."""
    rng = np.random.default_rng(12)
    M = 32
    T = (rng.random((M, 256), dtype=np.float32) * np.float32(5e4)).astype(np.float32)
    members = rng.integers(0, 256, size=(500, M))
    members[:, ::2] = members[:, ::2] % 19                    # few distinct codes in half the subspaces
    mins = np.array([T[j, np.unique(members[:, j])].min() for j in range(M)], dtype=np.float32)
    lb = float(seq_sum(mins)[-1])
    glob = float(seq_sum(T.min(axis=1))[-1])
    assert lb >= glob
    for c in members:
        assert float(seq_sum(T[np.arange(M), c])[-1]) >= lb * (1.0 - 2.0 * M * float(U))


def test_passing_over_a_list_is_implied_by_its_slack():
    """sqrt(lb)(1 - 1e-6) - c bmax (1 + 1e-6) > st  implies  lb > (c b + st)^2 for every b <= bmax,
    in binary32 as the kernel evaluates the right side (fma, then a square)."""
    rng = np.random.default_rng(13)
    c = np.float32(1.000025)
    for _ in range(20000):
        bmax = np.float32(rng.random() * 300.0)
        st = np.float32(rng.random() * 400.0 + 1e-3)
        lb = np.float32((float(bmax) * 1.00003 + float(st)) ** 2 * (1.0 + rng.random() * 1e-4))
        slack = np.float32(np.float32(np.sqrt(lb)) * np.float32(1.0 - 1e-6)
                           - np.float32(np.float32(c * bmax) * np.float32(1.0 + 1e-6)))
        if slack > st:
            b = np.float32(bmax * np.float32(rng.random()))
            r = np.float32(np.float64(b) * np.float64(c) + np.float64(st))      # one rounding: an fma
            assert lb > np.float32(r * r)


def test_abandon_threshold_implies_the_bound_exceeds_tau(oracle):
    """Once a table sum s exceeds (c b + c max(sqrt(tau), 1e-15))^2 as the kernel computes it, the
    oracle's Equation 3 at that s (and at any larger s, any gamma >= 0) is above tau: abandoning
    there prunes nobody the full evaluation would keep."""
    rng = np.random.default_rng(14)
    c = np.float32(1.000025)
    checked = 0
    for _ in range(4000):
        b = np.float32(rng.random() * 10 ** rng.uniform(-3, 3))
        tau = np.float32(rng.random() * 10 ** rng.uniform(-6, 6))
        st = np.float32(c * max(np.float32(np.sqrt(tau)), np.float32(1e-15)))
        r = np.float32(np.float64(b) * np.float64(c) + np.float64(st))
        thr = np.float32(r * r)
        for gamma in (0.0, 0.3, 1.0):
            for mult in (1.0 + 1e-7, 1.0001, 1.5, 40.0):
                s = np.nextafter(np.float32(thr * np.float32(mult)), np.float32(np.inf))
                if s > thr:
                    assert oracle.plb_from_s(s, b, gamma) > tau
                    checked += 1
    assert checked > 40000
