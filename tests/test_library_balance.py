"""The library's Load Balancer arithmetic (closed form) against the oracle's (the paper's
iteration, Sec. 4.3 Eq. 4-8).  Host only: no GPU call is made.

The oracle reaches the optimum by a subgradient iteration; the bar is therefore the iteration's
own accuracy: T_hot within 5e-3 relative, shares within 1e-2 absolute.  What is exact is checked
exactly: Eq. 4 and Eq. 5 evaluated by the oracle on the library's shares, sums, and the state."""
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
        # against the paper's iteration
        a, t = orc.balance_iterate(ts, bw, S, 30000)
        assert got["t_hot"] <= t * (1 + 1e-9)                    # the closed form is the minimum
        assert got["t_hot"] == pytest.approx(t, rel=5e-3), case
        assert np.abs(a - got["alpha"]).max() <= 1e-2, case


def test_threshold_separates_the_two_states(orc):
    rnd = random.Random(7)
    for _ in range(40):
        R = rnd.randint(2, 5)
        ts, bw = _random_model(rnd, R)
        th = nz.nz_balance_threshold(ts, bw)
        assert th >= 0
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
    a, t_iter = orc.balance_iterate(ts, bw, 256e6, 30000)
    assert big["t_hot"] == pytest.approx(t_iter, rel=5e-3) and np.abs(a - big["alpha"]).max() <= 1e-2


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
