"""The library's Load Balancer arithmetic against the oracle's definitions (Sec. 4.3 Eq. 4-8).
Host only: no GPU call is made.

The oracle states what is aimed at -- Eq. 4, Eq. 5, the minimum of Eq. 5 over the shares
(bisection), the threshold of Eq. 6 (bisection) -- and the library is held to it: the closed
form (nz_balance, nz_balance_threshold) to 1e-9, the paper's iteration (nz_balance_iterate:
Eq. 8 start, Eq. 7 steps) to the resolution of the data-length table within 100 steps."""
import random

import numpy as np
import pytest

from paper_2405_17870_amd import nezha_sim as nz


def _random_model(rnd, R):
    ts = [rnd.choice([9e-6, 5e-5, 2e-4, 1e-3]) * rnd.uniform(0.5, 2.0) for _ in range(R)]
    bw = [rnd.choice([0.1e9, 0.4e9, 1e9, 12e9]) * rnd.uniform(0.5, 2.0) for _ in range(R)]
    return ts, bw


def test_balance_matches_oracle_iteration(orc):
    rnd = random.Random(42)
    for case in range(60):
        R = rnd.randint(1, 5)
        ts, bw = _random_model(rnd, R)
        S = 10 ** rnd.uniform(3, 9)
        got = nz.nz_balance(ts, bw, S)
        # exact statements
        tc, best = orc.t_cold(ts, bw, S)
        assert got["t_cold"] == pytest.approx(tc, rel=1e-12) and got["best_rail"] == best
        assert got["alpha"].sum() == pytest.approx(1.0, abs=1e-12) and (got["alpha"] >= 0).all()
        assert orc.t_hot(ts, bw, S, got["alpha"]) == pytest.approx(got["t_hot"], rel=1e-9)
        assert int(got["ratios"].astype(np.int64).sum()) == nz.NZ_RATIO_SCALE
        assert np.abs(got["ratios"] / nz.NZ_RATIO_SCALE - got["alpha"]).max() <= 1.0 / nz.NZ_RATIO_SCALE
        assert got["t_hot"] <= got["t_cold"] * (1 + 1e-12)
        assert got["hot"] == (np.count_nonzero(got["alpha"]) > 1)
        # against the definition: the minimum of Eq. 5 over all shares
        a, t = orc.balance_optimum(ts, bw, S)
        assert got["t_hot"] == pytest.approx(t, rel=1e-9), case
        assert np.abs(a - got["alpha"]).max() <= 1e-9, case


def test_threshold_separates_the_two_states(orc):
    rnd = random.Random(7)
    for _ in range(40):
        R = rnd.randint(2, 5)
        ts, bw = _random_model(rnd, R)
        th = nz.nz_balance_threshold(ts, bw)
        assert th >= 0
        assert th == pytest.approx(orc.threshold(ts, bw), rel=1e-9, abs=1e-3)      # Eq. 6 by its definition
        below, above = nz.nz_balance(ts, bw, th * 0.999), nz.nz_balance(ts, bw, th * 1.001 + 1.0)
        assert not below["hot"] and above["hot"]
        # Eq. 6: at the threshold both states cost the same
        at = nz.nz_balance(ts, bw, th)
        assert at["t_hot"] == pytest.approx(at["t_cold"], rel=1e-9)
    assert nz.nz_balance_threshold([1e-3], [1e9]) == float("inf")
    # hand case: (4 ms - 1 ms) * 1 GB/s = 3 MB
    assert nz.nz_balance_threshold([1e-3, 4e-3], [1e9, 4e9]) == pytest.approx(3e6, rel=1e-12)


def test_balance_special_cases_and_errors():
    r = nz.nz_balance([2e-4] * 4, [1e9] * 4, 16e6)               # homogeneous rails: equal shares
    assert np.allclose(r["alpha"], 0.25) and list(r["ratios"]) == [1 << 18] * 4 and r["hot"]
    r = nz.nz_balance([1e-3, 4e-3], [1e9, 4e9], 8e6)              # hand case: a = 1/2, T = 5 ms
    assert np.allclose(r["alpha"], [0.5, 0.5]) and r["t_hot"] == pytest.approx(5e-3)
    r = nz.nz_balance([1e-3, 4e-3], [1e9, 4e9], 1e6)              # small: cold start on rail 0
    assert list(r["ratios"]) == [1 << 20, 0] and not r["hot"] and r["best_rail"] == 0
    r = nz.nz_balance([1e-3], [1e9], 0.0)
    assert list(r["ratios"]) == [1 << 20]
    for bad in ([[-1e-3], [1e9]], [[1e-3], [0.0]], [[1e-3], [float("nan")]], [[], []]):
        with pytest.raises(nz.NezhaSimError):
            nz.nz_balance(bad[0], bad[1], 1e6)
    with pytest.raises(nz.NezhaSimError):
        nz.nz_balance([1e-3] * 9, [1e9] * 9, 1e6)


def test_ratios_feed_the_partition(orc):
    r = nz.nz_balance([9e-6, 982e-6], [0.35e9, 0.2e9], 64e6)
    b = nz.nz_rail_partition(16 * 1024 * 1024, 4, r["ratios"])
    assert b.tolist() == orc.rail_partition(16 * 1024 * 1024, r["ratios"], 4).tolist()
    share = (b[1] - b[0]) / (16 * 1024 * 1024)
    assert share == pytest.approx(r["alpha"][0], abs=1e-4)


def test_measured_launch_latencies_as_setup_times(orc):
    """Two rails whose (T_setup, B) are the fixed cost per call and the asymptotic payload rate
    measured for the two allreduce modes at 8 nodes (profiles/size_sweep.txt): a real setup
    time in the sense of Eq. 2, not an invented one."""
    ts, bw = [8.37e-6, 49.28e-6], [373.57e9, 193.24e9]
    th = nz.nz_balance_threshold(ts, bw)
    assert th == pytest.approx((49.28e-6 - 8.37e-6) * 373.57e9, rel=1e-12)     # Eq. 6: about 15.3 MB
    small = nz.nz_balance(ts, bw, 4e6)                       # below it: everything on the fast-to-start rail
    assert not small["hot"] and list(small["ratios"]) == [1 << 20, 0]
    big = nz.nz_balance(ts, bw, 256e6)
    assert big["hot"]
    # both rails finish together (Eq. 5 is a maximum: its minimum equalises the two terms)
    t = [ts[i] + big["alpha"][i] * 256e6 / bw[i] for i in range(2)]
    assert t[0] == pytest.approx(t[1], rel=1e-9) and big["t_hot"] == pytest.approx(t[0], rel=1e-9)
    a, t_opt = orc.balance_optimum(ts, bw, 256e6)
    assert big["t_hot"] == pytest.approx(t_opt, rel=1e-9) and np.abs(a - big["alpha"]).max() <= 1e-9
    assert th == pytest.approx(orc.threshold(ts, bw), rel=1e-9)


def _table1_rails():
    """(T_setup, B) of the paper's TCP and SHARP rails, fitted from the single-rail columns of its
    Table 1 at the smallest and the largest size."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "table1_latency.txt")
    tab = {}
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            v = [int(x) for x in line.split("|")]
            tab[v[0]] = v[1:]
    small, large = min(tab), max(tab)

    def fit(col):
        t1, t2 = tab[small][col] * 1e-6, tab[large][col] * 1e-6
        b = (large - small) / (t2 - t1)
        return t1 - small / b, b

    (ts_s, b_s), (ts_t, b_t) = fit(0), fit(1)
    return [ts_t, ts_s], [b_t, b_s], sorted(tab)


def _table_resolution(ts, bw, S):
    """Time one unit of the data-length table (2^-20 of the message) takes on the slowest rail:
    what an iteration that stops at table convergence may still be away from the optimum."""
    return S / nz.NZ_RATIO_SCALE / min(bw)


def test_iteration_on_the_papers_rails_converges_within_100_steps(orc):
    """Eq. 8 start + Eq. 7 steps on the rails of the paper's Table 1, over the range of its
    allreduce benchmark: the optimum of Eq. 5 is reached well inside the 100 iterations the
    paper reports for convergence."""
    ts, bw, sizes = _table1_rails()
    for S in sizes + [2.0 ** k for k in range(11, 27)]:
        got = nz.nz_balance_iterate(ts, bw, S, 100)
        a, t = orc.balance_optimum(ts, bw, S)
        assert got["iterations"] < 100
        assert got["t_hot"] >= t * (1 - 1e-12)
        assert got["t_hot"] - t <= 2 * _table_resolution(ts, bw, S) + 1e-12 * t, S
        assert np.abs(got["alpha"] - a).max() <= 2.0 / nz.NZ_RATIO_SCALE, S
        assert orc.t_hot(ts, bw, S, got["alpha"]) == pytest.approx(got["t_hot"], rel=1e-12)
        assert int(got["ratios"].astype(np.int64).sum()) == nz.NZ_RATIO_SCALE


def test_iteration_start_steps_and_monotone_descent(orc):
    # Eq. 8 by hand: uniform split of 3 MB over three 1 GB/s rails -> T_i = 2, 3, 4 ms, T = 9 ms
    ts, bw, S = [1e-3, 2e-3, 3e-3], [1e9, 1e9, 1e9], 3e6
    start = nz.nz_balance_iterate(ts, bw, S, 0)
    assert start["iterations"] == 0
    assert np.allclose(start["alpha"], [(9 - 2) / 18, (9 - 3) / 18, (9 - 4) / 18], rtol=1e-12)
    # first step by hand: times 1 + 7/6, 2 + 1, 3 + 5/6 ms -> slowest rail 2 (3.8333), first to finish
    # rail 0 (2.1667); equal bandwidths: they meet at 3 ms, rail 2's startup alone: it sits out
    one = nz.nz_balance_iterate(ts, bw, S, 1)
    assert np.allclose(one["alpha"], [7 / 18 + 5 / 18, 6 / 18, 0.0], rtol=1e-12)
    # T_hot never rises from step to step, and ends at the optimum
    rnd = random.Random(5)
    for _ in range(40):
        R = rnd.randint(2, 8)
        ts, bw = _random_model(rnd, R)
        S = 10 ** rnd.uniform(3, 9)
        prev = None
        for k in range(0, 60):
            cur = nz.nz_balance_iterate(ts, bw, S, k)
            assert abs(cur["alpha"].sum() - 1.0) <= 1e-12 and (cur["alpha"] >= 0).all()
            if prev is not None:
                assert cur["t_hot"] <= prev * (1 + 1e-12)
            prev = cur["t_hot"]
            if cur["iterations"] < k:
                break
        assert prev >= orc.balance_optimum(ts, bw, S)[1] * (1 - 1e-12)


def test_iteration_reaches_the_optimum_on_random_rails(orc):
    rng = np.random.default_rng(21)
    worst = 0.0
    for case in range(3000):
        R = int(rng.integers(1, 9))
        ts, bw = list(10 ** rng.uniform(-6, -2, R)), list(10 ** rng.uniform(7, 10.5, R))
        S = 10 ** rng.uniform(3, 9.5)
        got = nz.nz_balance_iterate(ts, bw, S, 100)
        _, t = orc.balance_optimum(ts, bw, S)
        assert got["t_hot"] >= t * (1 - 1e-12)
        worst = max(worst, got["t_hot"] / t - 1.0)
        if R <= 3:       # up to three rails the table converges within the 100 steps
            assert got["iterations"] < 100
            assert got["t_hot"] - t <= R * _table_resolution(ts, bw, S) + 1e-12 * t, case
    assert worst <= 5e-3         # eight very unequal rails after 100 steps: within half a percent
    with pytest.raises(nz.NezhaSimError):
        nz.nz_balance_iterate([1e-3], [1e9], 0.0)
    with pytest.raises(nz.NezhaSimError):
        nz.nz_balance_iterate([1e-3] * 9, [1e9] * 9, 1e6)


def test_efficiency_and_ratio_match_the_oracle(orc):
    rnd = random.Random(3)
    for _ in range(200):
        R = rnd.randint(1, 8)
        ts, bw = _random_model(rnd, R)
        S = 10 ** rnd.uniform(2, 9)
        assert nz.nz_net_efficiency(ts[0], bw[0], S) == pytest.approx(orc.net_efficiency(ts[0], bw[0], S), rel=1e-13)
        alpha = [rnd.choice([0.0, rnd.random()]) for _ in range(R)]
        if sum(alpha) == 0.0:
            alpha[rnd.randrange(R)] = 1.0
        for shares in (None, alpha):
            a = [1.0 / R] * R if shares is None else [x / sum(alpha) for x in alpha]
            live = [i for i in range(R) if a[i] > 0]
            want = max([orc.efficiency_ratio(ts[i], bw[i], a[i] * S, ts[j], bw[j], a[j] * S)
                        for i in live for j in live if i != j], default=1.0)
            assert nz.nz_efficiency_ratio(ts, bw, S, shares) == pytest.approx(want, rel=1e-12)
    assert nz.nz_efficiency_ratio([2e-4] * 3, [1e9] * 3, 6e6) == 1.0        # homogeneous rails
    assert nz.NZ_TOLERANCE_TAU == 5.0
    for bad in (lambda: nz.nz_net_efficiency(1e-3, 1e9, 0.0), lambda: nz.nz_net_efficiency(1e-3, 0.0, 1e6),
                lambda: nz.nz_efficiency_ratio([1e-3, 1e-3], [1e9, 1e9], 1e6, [0.0, 0.0]),
                lambda: nz.nz_efficiency_ratio([1e-3, 1e-3], [1e9, 1e9], 1e6, [-1.0, 2.0]),
                lambda: nz.nz_efficiency_ratio([1e-3], [1e9], float("inf"))):
        with pytest.raises(nz.NezhaSimError):
            bad()
