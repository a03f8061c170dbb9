"""Pins for the oracle's data-allocation arithmetic (Nezha Sec. 4.3, Eq. 4-8), CPU only.

Pinned by hand-worked two-rail cases, by brute force over a fine grid of the simplex, by the
special cases the paper states (homogeneous rails share equally; small messages go to the best
single rail) and by the equal-finish-time property of the optimum."""
import itertools

import numpy as np
import pytest


def test_eq4_and_eq5_by_hand(orc):
    ts, bw = [1e-3, 4e-3], [1e9, 4e9]
    # 8 MB: rail 0 -> 1 ms + 8 ms = 9 ms, rail 1 -> 4 ms + 2 ms = 6 ms
    t, best = orc.t_cold(ts, bw, 8e6)
    assert best == 1 and t == pytest.approx(6e-3, rel=1e-12)
    # 1 MB: 2 ms vs 4.25 ms
    t, best = orc.t_cold(ts, bw, 1e6)
    assert best == 0 and t == pytest.approx(2e-3, rel=1e-12)
    # Eq. 5 with shares 1/4, 3/4 of 8 MB: max(1 + 2, 4 + 1.5) ms
    assert orc.t_hot(ts, bw, 8e6, [0.25, 0.75]) == pytest.approx(5.5e-3, rel=1e-12)
    # a rail given nothing sits out: all on rail 0
    assert orc.t_hot(ts, bw, 8e6, [1.0, 0.0]) == pytest.approx(9e-3, rel=1e-12)
    # the optimum equalises: 1 + 8a = 4 + 2(1-a) -> a = 0.5, T = 5 ms
    assert orc.t_hot(ts, bw, 8e6, [0.5, 0.5]) == pytest.approx(5e-3, rel=1e-12)


def _grid_best(orc, ts, bw, S, steps):
    R = len(ts)
    best = (np.inf, None)
    for c in itertools.product(range(steps + 1), repeat=R - 1):
        if sum(c) > steps:
            continue
        a = [x / steps for x in c] + [1 - sum(c) / steps]
        t = orc.t_hot(ts, bw, S, a)
        if t < best[0]:
            best = (t, a)
    return best


@pytest.mark.parametrize("ts,bw,S", [
    ([1e-3, 4e-3], [1e9, 4e9], 8e6),
    ([1e-3, 4e-3], [1e9, 4e9], 1e6),            # small: everything on rail 0
    ([9e-6, 982e-6], [0.35e9, 0.2e9], 64e6),    # an RDMA-like and a TCP-like rail
    ([1e-4, 1e-4, 1e-4], [1e9, 1e9, 1e9], 3e6),
    ([1e-4, 2e-4, 5e-3], [1e9, 3e9, 2e9], 2e6),
])
def test_iteration_reaches_the_brute_force_optimum(orc, ts, bw, S):
    a, t = orc.balance_iterate(ts, bw, S, 40000)
    assert a.sum() == pytest.approx(1.0, abs=1e-9) and (a >= 0).all()
    assert orc.t_hot(ts, bw, S, a) == pytest.approx(t, rel=1e-12)
    steps = 2000 if len(ts) == 2 else 120
    tg, ag = _grid_best(orc, ts, bw, S, steps)
    assert t <= tg * (1 + 1e-9) + 0 or t == pytest.approx(tg, rel=5e-3)
    assert t == pytest.approx(tg, rel=2e-2)            # the grid itself is coarse for three rails
    tc, _ = orc.t_cold(ts, bw, S)
    assert t <= tc * (1 + 1e-12)                        # never worse than the best single rail


def _zoom_best(orc, ts, bw, S, rounds=9, steps=20):
    """Brute force over the simplex with Eq. 5 alone: a grid over the whole simplex (vertices and
    faces included: rails given nothing sit out), then ever finer grids around the best point."""
    R = len(ts)
    best_t, best_a = np.inf, None
    centre, width = np.full(R - 1, 0.5), 0.5
    for _ in range(rounds):
        axes = [np.unique(np.clip(np.linspace(c - width, c + width, steps + 1), 0.0, 1.0)) for c in centre]
        for head in itertools.product(*axes):
            last = 1.0 - sum(head)
            if last < -1e-15:
                continue
            a = list(head) + [max(last, 0.0)]
            t = orc.t_hot(ts, bw, S, a)
            if t < best_t:
                best_t, best_a = t, a
        centre, width = np.array(best_a[:-1]), width * 2.5 / steps
    return best_t, best_a


_MODELS = [
    ([1e-3, 4e-3], [1e9, 4e9], 8e6),
    ([1e-3, 4e-3], [1e9, 4e9], 1e6),            # small: everything on rail 0
    ([9e-6, 982e-6], [0.35e9, 0.2e9], 64e6),    # an RDMA-like and a TCP-like rail
    ([1e-4, 1e-4, 1e-4], [1e9, 1e9, 1e9], 3e6),
    ([1e-4, 2e-4, 5e-3], [1e9, 3e9, 2e9], 2e6),  # the third rail starts too late to help
    ([3e-4, 1e-4, 2e-4], [2e9, 1e9, 5e8], 9e6),
]


@pytest.mark.parametrize("ts,bw,S", _MODELS)
def test_optimum_is_the_brute_force_minimum_of_eq5(orc, ts, bw, S):
    a, t = orc.balance_optimum(ts, bw, S)
    assert a.sum() == pytest.approx(1.0, abs=1e-12) and (a >= 0).all()
    assert orc.t_hot(ts, bw, S, a) == pytest.approx(t, rel=1e-12)       # the shares do reach it
    tg, ag = _zoom_best(orc, ts, bw, S, steps=40 if len(ts) == 2 else 20)
    assert t == pytest.approx(tg, rel=1e-6)
    assert t <= tg * (1 + 1e-12)                                         # nothing on the grid beats it
    assert np.abs(a - np.array(ag)).max() <= 1e-5


def test_optimum_hand_cases_and_its_characterisation(orc):
    # 8 MB over (1 ms, 1 GB/s) and (4 ms, 4 GB/s): 1 + 8a = 4 + 2(1 - a) ms -> a = 1/2, T = 5 ms
    a, t = orc.balance_optimum([1e-3, 4e-3], [1e9, 4e9], 8e6)
    assert np.allclose(a, [0.5, 0.5], atol=1e-12) and t == pytest.approx(5e-3, rel=1e-12)
    # equal startup latencies: shares proportional to bandwidth, T = T_setup + S / sum B
    a, t = orc.balance_optimum([2e-4] * 3, [1e9, 2e9, 5e9], 4e7)
    assert np.allclose(a, np.array([1, 2, 5]) / 8, atol=1e-12) and t == pytest.approx(2e-4 + 4e7 / 8e9, rel=1e-12)
    # homogeneous rails share equally
    a, _ = orc.balance_optimum([2e-4] * 4, [1e9] * 4, 16e6)
    assert np.allclose(a, 0.25, atol=1e-12)
    # a message the first rail finishes before the second could start stays on the first
    a, t = orc.balance_optimum([1e-3, 4e-3], [1e9, 4e9], 1e6)
    assert list(a) == [1.0, 0.0] and t == pytest.approx(2e-3, rel=1e-12)
    # what characterises the minimum of a maximum: rails that take part finish together, the
    # others could not even have started by then
    rng = np.random.default_rng(11)
    for _ in range(200):
        R = int(rng.integers(1, 9))
        ts, bw, S = 10 ** rng.uniform(-6, -2, R), 10 ** rng.uniform(7, 10.5, R), 10 ** rng.uniform(3, 9.5)
        a, t = orc.balance_optimum(ts, bw, S)
        assert a.sum() == pytest.approx(1.0, abs=1e-9)
        for i in range(R):
            if a[i] > 0:
                assert ts[i] + a[i] * S / bw[i] == pytest.approx(t, rel=1e-9)
            else:
                assert ts[i] >= t * (1 - 1e-12)
        assert t <= orc.t_cold(ts, bw, S)[0] * (1 + 1e-12)
        # any other allocation is no better: perturb the shares
        for _ in range(5):
            b = np.clip(a + rng.normal(0, 0.05, R), 0, None)
            if b.sum() > 0:
                assert orc.t_hot(ts, bw, S, b / b.sum()) >= t * (1 - 1e-9)


def test_eq6_threshold_by_hand_and_by_its_definition(orc):
    # (4 ms - 1 ms) * 1 GB/s = 3 MB: up to there the first rail is done before the second starts
    assert orc.threshold([1e-3, 4e-3], [1e9, 4e9]) == pytest.approx(3e6, rel=1e-9)
    assert orc.threshold([1e-3], [1e9]) == float("inf")
    assert orc.threshold([1e-3, 1e-3], [1e9, 2e9]) == pytest.approx(0.0, abs=1e-3)   # equal start: always share
    rng = np.random.default_rng(12)
    for _ in range(100):
        R = int(rng.integers(2, 7))
        ts, bw = 10 ** rng.uniform(-6, -2, R), 10 ** rng.uniform(7, 10.5, R)
        th = orc.threshold(ts, bw)
        # Eq. 6 holds at the threshold and below it, and fails above it
        for S, equal in ((0.5 * th, True), (th, True), (1.01 * th + 1.0, False)):
            if S > 0:
                cold, hot = orc.t_cold(ts, bw, S)[0], orc.balance_optimum(ts, bw, S)[1]
                assert (hot == pytest.approx(cold, rel=1e-11)) == equal, (S, th)
                assert hot <= cold * (1 + 1e-12)
    # the paper's Table 1 rails (fitted as in the Eq. 5 test): 1 KB lies below the threshold (no
    # split helps there), 8 MB and 64 MB above it (the 1:1 split beats both single rails)
    tab = _table1()
    small, large = min(tab), max(tab)

    def fit(col):
        t1, t2 = tab[small][col] * 1e-6, tab[large][col] * 1e-6
        b = (large - small) / (t2 - t1)
        return t1 - small / b, b

    (ts_s, b_s), (ts_t, b_t) = fit(0), fit(1)
    th = orc.threshold([ts_t, ts_s], [b_t, b_s])
    for S, row in tab.items():
        assert (S > th) == (row[2] < min(row[0], row[1])), (S, th)


def test_homogeneous_rails_share_equally_and_bandwidth_proportional(orc):
    a, _ = orc.balance_iterate([2e-4] * 4, [1e9] * 4, 16e6)
    assert np.allclose(a, 0.25, atol=2e-3)
    # equal startup, different bandwidth: shares proportional to bandwidth once setup is negligible
    a, _ = orc.balance_iterate([1e-6] * 3, [1e9, 2e9, 5e9], 1e9, 40000)
    assert np.allclose(a, np.array([1, 2, 5]) / 8, atol=3e-3)


def test_small_message_goes_to_one_rail(orc):
    # below (Ts_2 - Ts_1) * B_1 = 3 ms * 1 GB/s = 3 MB the second rail cannot help
    a, t = orc.balance_iterate([1e-3, 4e-3], [1e9, 4e9], 1e6, 40000)
    assert a[0] == pytest.approx(1.0, abs=1e-6) and a[1] == pytest.approx(0.0, abs=1e-6)
    assert t == pytest.approx(orc.t_cold([1e-3, 4e-3], [1e9, 4e9], 1e6)[0], rel=1e-9)


def test_eq8_starting_shares_sum_to_one(orc):
    # zero iterations returns Eq. 8's shares: (T - T_i) / (T (R - 1))
    ts, bw, S = [1e-3, 2e-3, 3e-3], [1e9, 1e9, 1e9], 3e6
    a, _ = orc.balance_iterate(ts, bw, S, 0)
    Ti = np.array([2e-3, 3e-3, 4e-3])
    assert np.allclose(a, (Ti.sum() - Ti) / (Ti.sum() * 2), rtol=1e-12)
    assert a.sum() == pytest.approx(1.0, abs=1e-12)


def _table1():
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "table1_latency.txt")
    rows = {}
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            v = [int(x) for x in line.split("|")]
            rows[v[0]] = v[1:]
    return rows


def test_eq5_reproduces_the_printed_split_latencies_of_table1(orc):
    """The paper's own measurements (Table 1): each rail's (T_setup, B) is fitted from its
    single-rail column at the smallest and the largest size; Eq. 5 with the printed shares must
    then land near every printed two-rail latency (the model is linear, the measurements are not
    quite: 12 % covers all nine entries), and Eq. 4 must pick the rail the table shows as best.
    A sum or a minimum in place of the maximum, or shares given to the wrong rail, miss by 40 %
    or more."""
    tab = _table1()
    small, large = min(tab), max(tab)

    def fit(col):
        t1, t2 = tab[small][col] * 1e-6, tab[large][col] * 1e-6
        b = (large - small) / (t2 - t1)
        return t1 - small / b, b

    (ts_s, b_s), (ts_t, b_t) = fit(0), fit(1)
    ts, bw = [ts_t, ts_s], [b_t, b_s]                       # rail 0 = TCP, rail 1 = SHARP
    for S, row in tab.items():
        for shares, printed in (((0.5, 0.5), row[2]), ((0.99, 0.01), row[3]), ((0.01, 0.99), row[4])):
            assert orc.t_hot(ts, bw, S, shares) * 1e6 == pytest.approx(printed, rel=0.12), (S, shares)
        t, best = orc.t_cold(ts, bw, S)
        assert best == 1 and row[0] < row[1]                 # SHARP is the better single rail at every size
        assert t * 1e6 == pytest.approx(row[0], rel=0.03)
    # what the table shows for small messages: no split comes near the best single rail (Eq. 4 applies)
    assert orc.t_cold(ts, bw, small)[0] * 1e6 < 0.02 * min(tab[small][2:])
    # swapping the shares of the 99:1 column gives the 1:99 column, not the 99:1 one
    assert orc.t_hot(ts, bw, large, (0.01, 0.99)) * 1e6 != pytest.approx(tab[large][3], rel=0.12)


def test_eq2_network_efficiency_closed_forms(orc):
    # T_setup equal to the transmission time halves the efficiency; three times it quarters it
    assert orc.net_efficiency(1e-3, 1e9, 1e6) == pytest.approx(0.5, rel=1e-15)
    assert orc.net_efficiency(3e-3, 1e9, 1e6) == pytest.approx(0.25, rel=1e-15)
    assert orc.net_efficiency(0.0, 1e9, 1e6) == 1.0
    # it is T_theoretical / T_actual, and grows with the message size towards one
    for ts, bw, S in [(9e-6, 0.37e9, 1024.0), (982e-6, 0.21e9, 8.0 * 2 ** 20), (5e-5, 12e9, 3e7)]:
        assert orc.net_efficiency(ts, bw, S) == pytest.approx((S / bw) / (ts + S / bw), rel=1e-14)
        assert orc.net_efficiency(ts, bw, S) < orc.net_efficiency(ts, bw, 2 * S) < 1.0
    # half efficiency exactly at S = T_setup * B
    assert orc.net_efficiency(982e-6, 0.2e9, 982e-6 * 0.2e9) == pytest.approx(0.5, rel=1e-14)


def test_eq3_efficiency_ratio_is_a_ratio_of_throughputs(orc):
    from fractions import Fraction as Fr
    cases = [((Fr(1, 1000), Fr(10 ** 9), Fr(4 * 10 ** 6)), (Fr(4, 1000), Fr(4 * 10 ** 9), Fr(12 * 10 ** 6))),
             ((Fr(9, 10 ** 6), Fr(37 * 10 ** 7), Fr(512)), (Fr(982, 10 ** 6), Fr(21 * 10 ** 7), Fr(512)))]
    for (ti, bi, si), (tj, bj, sj) in cases:
        exact = (si / (ti + si / bi)) / (sj / (tj + sj / bj))          # bytes per second over bytes per second
        got = orc.efficiency_ratio(float(ti), float(bi), float(si), float(tj), float(bj), float(sj))
        assert got == pytest.approx(float(exact), rel=1e-13)
        back = orc.efficiency_ratio(float(tj), float(bj), float(sj), float(ti), float(bi), float(si))
        assert got * back == pytest.approx(1.0, rel=1e-13)
    # hand case: 4 MB on (1 ms, 1 GB/s) takes 5 ms -> 0.8 GB/s; 12 MB on (4 ms, 4 GB/s) takes 7 ms -> 12/7 GB/s
    assert orc.efficiency_ratio(1e-3, 1e9, 4e6, 4e-3, 4e9, 12e6) == pytest.approx(0.8 / (12 / 7), rel=1e-13)
    # identical networks with equal volumes: the homogeneous case, rho = 1
    assert orc.efficiency_ratio(2e-4, 1e9, 5e6, 2e-4, 1e9, 5e6) == 1.0


def test_eq3_against_table1_and_the_tolerance_threshold(orc):
    """Table 1 again: the two single-rail columns are each network's latency on the whole
    message, so their quotient is the measured efficiency ratio.  It is far above the paper's
    tolerance threshold (tau = 5, Sec. 2.2.1) at 1 KB, where the table shows that no split
    helps, and below it at 8 MB and 64 MB, where the 1:1 split beats both single rails."""
    tab = _table1()
    small, large = min(tab), max(tab)
    tau = 5.0

    def fit(col):
        t1, t2 = tab[small][col] * 1e-6, tab[large][col] * 1e-6
        b = (large - small) / (t2 - t1)
        return t1 - small / b, b

    (ts_s, b_s), (ts_t, b_t) = fit(0), fit(1)
    for S, row in tab.items():
        measured = row[1] / row[0]                                   # SHARP's throughput over TCP's
        rho = orc.efficiency_ratio(ts_s, b_s, S, ts_t, b_t, S)
        assert rho == pytest.approx(measured, rel=0.08), S
        split_helps = row[2] < min(row[0], row[1])
        assert (rho <= tau) == split_helps, S
