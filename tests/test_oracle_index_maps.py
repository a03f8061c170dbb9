"""Pins for the oracle's rail partition and ring segment cut (CPU only).

What fixes them: the paper's statements that each rail owns one contiguous
slice, that the proportions sum to one, and that a ring cuts a message into N
pieces (Nezha Sec. 3.4, 3.5, 4.3 under Eq. 5, Eq. 1), hand-worked numbers in
tests/golden/partition_cases.txt, exact rational arithmetic, and brute force.
"""
import os
import random
from fractions import Fraction

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "partition_cases.txt")


def _golden_rows():
    rows = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        head, w, b, qr = [p.split() for p in line.split("|")]
        rows.append(dict(name=head[0], N=int(head[1]), n=int(head[2]), e=int(head[3]),
                         w=[int(x) for x in w], b=[int(x) for x in b],
                         qr=[tuple(int(v) for v in x.split(":")) for x in qr]))
    return rows


@pytest.mark.parametrize("row", _golden_rows(), ids=lambda r: r["name"])
def test_partition_and_segments_match_hand_worked_table(orc, row):
    b = orc.rail_partition(row["n"], row["w"], row["e"])
    assert [int(x) for x in b] == row["b"]
    seg = orc.segment_map(b, row["N"])
    for k, (q, r) in enumerate(row["qr"]):
        lens = np.diff(seg[k].astype(np.int64))
        assert int(seg[k, 0]) == row["b"][k] and int(seg[k, -1]) == row["b"][k + 1]
        assert list(lens[:r]) == [q + 1] * r
        assert list(lens[r:]) == [q] * (row["N"] - r)


def test_hand_case_segment_offsets(orc):
    # N = 3, n = 200, weights 3:1, 4-byte elements: worked on paper.
    b = orc.rail_partition(200, [3, 1], 4)
    seg = orc.segment_map(b, 3)
    assert seg.tolist() == [[0, 43, 86, 128], [128, 152, 176, 200]]


def test_partition_invariants_random(orc):
    rnd = random.Random(1234)
    for _ in range(400):
        e = rnd.choice([2, 4])
        align = rnd.choice([e, 16, 64, 256])
        A = align // e
        R = rnd.randint(1, 6)
        n = rnd.choice([0, 1, rnd.randint(0, 300), rnd.randint(0, 10**6), rnd.randint(0, 2**40)])
        w = [rnd.choice([0, 1, rnd.randint(0, 1000), rnd.randint(0, 2**32 - 1)]) for _ in range(R)]
        if sum(w) == 0:
            w[rnd.randrange(R)] = 7
        b = [int(x) for x in orc.rail_partition(n, w, e, align)]
        W = sum(w)
        assert b[0] == 0 and b[-1] == n and len(b) == R + 1
        assert all(b[k] <= b[k + 1] for k in range(R))
        for k in range(1, R):
            exact = Fraction(n * sum(w[:k]), W)          # the proportional point
            if sum(w[:k]) == W:                          # only zero-weight rails follow
                assert b[k] == n
                continue
            assert b[k] % A == 0
            assert 0 <= exact - b[k] < A                 # floored, never more than A away
            assert b[k] == (exact // A) * A              # exact rational floor
        for k in range(R):                               # zero weight => empty range
            if w[k] == 0:
                assert b[k] == b[k + 1]
        # scaling every weight by a constant changes nothing
        c = rnd.randint(2, 9)
        if max(w) * c < 2**32:
            assert [int(x) for x in orc.rail_partition(n, [x * c for x in w], e, align)] == b


def test_partition_brute_force_marking(orc):
    rnd = random.Random(99)
    for _ in range(60):
        n = rnd.randint(0, 4096)
        R = rnd.randint(1, 5)
        w = [rnd.randint(0, 50) for _ in range(R)]
        if sum(w) == 0:
            w[0] = 1
        b = orc.rail_partition(n, w, 4, rnd.choice([4, 64, 256]))
        marks = np.zeros(n, dtype=np.int32)
        for k in range(R):
            marks[int(b[k]):int(b[k + 1])] += 1
        assert (marks == 1).all()


def test_partition_special_cases(orc):
    # one rail: everything
    assert orc.rail_partition(12345, [9], 4).tolist() == [0, 12345]
    # all data on one rail (the cold-start state of Sec. 4.3, Eq. 4)
    assert orc.rail_partition(1000, [1, 0], 4).tolist() == [0, 1000, 1000]
    assert orc.rail_partition(1000, [0, 1], 4).tolist() == [0, 0, 1000]
    # equal weights on a size divisible by R*A: an equal split (homogeneous rails share equally)
    assert orc.rail_partition(4 * 64 * 10, [5, 5, 5, 5], 4).tolist() == [0, 640, 1280, 1920, 2560]
    assert orc.rail_partition(1000, [3, 0, 1, 0], 4).tolist() == [0, 704, 704, 1000, 1000]
    # smaller than one alignment unit: the last rail takes it all
    assert orc.rail_partition(63, [1, 1], 4).tolist() == [0, 0, 63]
    # empty message
    assert orc.rail_partition(0, [1, 2, 3], 2).tolist() == [0, 0, 0, 0]
    with pytest.raises(ValueError):
        orc.rail_partition(10, [0, 0], 4)


def test_segment_invariants_random_and_brute_force(orc):
    rnd = random.Random(7)
    for _ in range(200):
        R = rnd.randint(1, 4)
        N = rnd.choice([1, 2, 3, 8, 32, 128, rnd.randint(1, 200)])
        cuts = sorted(rnd.randint(0, 5000) for _ in range(R - 1))
        n = rnd.randint(cuts[-1] if cuts else 0, 6000)
        b = [0] + cuts + [n]
        seg = orc.segment_map(b, N).astype(np.int64)
        marks = np.zeros(n, dtype=np.int32)
        for k in range(R):
            L = b[k + 1] - b[k]
            lens = np.diff(seg[k])
            assert seg[k, 0] == b[k] and seg[k, -1] == b[k + 1]
            assert lens.sum() == L and lens.min() >= 0
            assert lens.max() - lens.min() <= 1
            assert (np.diff(lens) <= 0).all()            # longer segments first
            assert lens.max() == -(-L // N) and lens.min() == L // N
            for j in range(N):
                marks[seg[k, j]:seg[k, j + 1]] += 1
        assert (marks == 1).all()
