"""Pins for the oracle's step-by-step ring allreduce (CPU only).

Fixed by the paper: a ring over N workers moves 2(N-1)*M/N per worker in N-1
reduce-scatter and N-1 allgather steps (Nezha Sec. 2.1.1, Eq. 1), rails work on
disjoint slices without interfering (Sec. 4.1), and the result is the sum,
identical on every node.  Pinned by a pure-Python re-statement of the ring on
lists of exact integers, by Eq. 1's byte count, by the hand-worked N = 3 case
and by the summation order the schedule implies.
"""
import random

import numpy as np
import pytest

from paper_2405_17870_amd import inputs


def _python_ring(vals, rows, stop_after_rs=False):
    """Ring allreduce on python ints, written independently: message passing with queues."""
    N = len(vals)
    bufs = [list(v) for v in vals]
    sent = [0] * N
    for phase in ("rs", "ag"):
        if phase == "ag" and stop_after_rs:
            break
        for s in range(N - 1):
            inbox = []
            for r in range(N):                               # everybody sends first ...
                j = (r - s) % N if phase == "rs" else (r + 1 - s) % N
                for row in rows:
                    lo, hi = row[j], row[j + 1]
                    inbox.append(((r + 1) % N, lo, bufs[r][lo:hi]))
                    sent[r] += hi - lo
            for d, lo, payload in inbox:                     # ... then everybody receives
                for t, v in enumerate(payload):
                    bufs[d][lo + t] = bufs[d][lo + t] + v if phase == "rs" else v
    return bufs, sent


def test_hand_case_three_nodes(orc):
    # N = 3, n = 200 int32, weights 3:1; in[i][x] = 1000 (i+1) + x  =>  out = 6000 + 3x everywhere
    N, n = 3, 200
    seg = orc.segment_map(orc.rail_partition(n, [3, 1], 4), N)
    bufs = [np.arange(n, dtype=np.int32) + 1000 * (i + 1) for i in range(N)]
    out, sent = orc.ring_allreduce(orc.I32, bufs, seg)
    for o in out:
        assert (o == 6000 + 3 * np.arange(n)).all()
    assert int(sent.sum()) == 2 * (N - 1) * n * 4 == 3200      # Eq. 1 summed over nodes
    # ownership after the reduce-scatter: node r holds complete segment (r+1) mod N, per rail
    rs, _ = orc.ring_allreduce(orc.I32, bufs, seg, reduce_scatter_only=True)
    want = 6000 + 3 * np.arange(n)
    for r in range(N):
        j = (r + 1) % N
        for k in range(2):
            lo, hi = int(seg[k, j]), int(seg[k, j + 1])
            assert (rs[r][lo:hi] == want[lo:hi]).all()
    # a segment the node does not own yet is still partial: node 0 holds segment 0 untouched
    # (its own segment index is never written in the reduce-scatter) and segment 2 half done
    assert (rs[0][0:43] == bufs[0][0:43]).all()
    lo, hi = int(seg[0, 2]), int(seg[0, 3])
    assert (rs[0][lo:hi] == (bufs[2] + bufs[0])[lo:hi]).all()


@pytest.mark.parametrize("N,R", [(1, 1), (2, 2), (3, 2), (5, 3), (8, 2), (17, 4)])
def test_int32_ring_equals_python_ring_and_sum(orc, N, R):
    rnd = random.Random(N * 100 + R)
    n = rnd.randint(0, 700)
    w = [rnd.randint(1, 100) for _ in range(R)]
    seg = orc.segment_map(orc.rail_partition(n, w, 4, 16), N)
    rng = np.random.default_rng(N)
    bufs = [rng.integers(-1000, 1001, size=n, dtype=np.int32) for _ in range(N)]
    out, sent = orc.ring_allreduce(orc.I32, bufs, seg)
    pyout, pysent = _python_ring([b.tolist() for b in bufs], seg.astype(np.int64).tolist())
    total = np.sum(np.stack(bufs).astype(np.int64), axis=0) if n else np.zeros(0, np.int64)
    for i in range(N):
        assert out[i].tolist() == pyout[i] == total.tolist()
        assert int(sent[i]) == pysent[i] * 4
    assert int(sent.sum()) == 2 * (N - 1) * n * 4               # Eq. 1, all workers
    # per worker: 2(N-1)/N of the message, up to one element per rail and step
    for i in range(N):
        assert abs(int(sent[i]) - 2 * (N - 1) * n * 4 / N) <= 2 * (N - 1) * R * 4
    assert (orc.sum_i32(bufs) == out[0]).all() if N else True
    rs, _ = orc.ring_allreduce(orc.I32, bufs, seg, reduce_scatter_only=True)
    pyrs, _ = _python_ring([b.tolist() for b in bufs], seg.astype(np.int64).tolist(), True)
    for i in range(N):
        assert rs[i].tolist() == pyrs[i]


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_float_ring_follows_the_implied_summation_order(orc, dtype):
    # segment j is accumulated as ((in[j] + in[j+1]) + in[j+2]) + ..., node indices mod N,
    # each partial stored in the wire type
    N, n = 6, 257
    code = {"f32": orc.F32, "bf16": orc.BF16, "f16": orc.F16}[dtype]
    tens = [inputs.node_buffer(dtype, n, 77, i, std=1.0) for i in range(N)]
    bufs = [inputs.to_host_storage(t) for t in tens]
    seg = orc.segment_map(orc.rail_partition(n, [2, 1], bufs[0].itemsize, 16), N)
    out, _ = orc.ring_allreduce(code, bufs, seg)
    import torch
    want = torch.empty_like(tens[0])
    for k in range(seg.shape[0]):
        for j in range(N):
            lo, hi = int(seg[k, j]), int(seg[k, j + 1])
            acc = tens[j][lo:hi].clone()
            for t in range(1, N):
                acc = (acc.float() + tens[(j + t) % N][lo:hi].float()).to(tens[0].dtype)
            want[lo:hi] = acc
    w = inputs.to_host_storage(want)
    for i in range(N):
        assert (out[i] == w).all()
    # and it is a sum: close to the fp64 definition
    s, a = orc.sum_float(code, bufs)
    got = np.array([orc.bf16_to_f32(v) for v in out[0]]) if dtype == "bf16" else \
        (out[0].view(np.float16).astype(np.float64) if dtype == "f16" else out[0].astype(np.float64))
    eps = {"f32": 2.0**-24, "bf16": 2.0**-8, "f16": 2.0**-11}[dtype]
    assert (np.abs(got - s) <= (N - 1) * eps * a * 1.01 + 1e-30).all()


def test_rails_do_not_interfere(orc):
    # the result is the same whatever the rail split (int32: exactly)
    N, n = 7, 1000
    rng = np.random.default_rng(0)
    bufs = [rng.integers(-1000, 1001, size=n, dtype=np.int32) for _ in range(N)]
    ref = None
    for w in ([1], [1, 1], [100, 40], [1, 0, 5], [100, 100, 40, 10]):
        seg = orc.segment_map(orc.rail_partition(n, w, 4, 64), N)
        out, sent = orc.ring_allreduce(orc.I32, bufs, seg)
        ref = out[0] if ref is None else ref
        assert all((o == ref).all() for o in out)
        assert int(sent.sum()) == 2 * (N - 1) * n * 4


@pytest.mark.parametrize("N,R", [(1, 1), (2, 1), (3, 2), (8, 2), (13, 3)])
def test_allgather_alone_spreads_each_owner_segment(orc, N, R):
    # node r enters owning segment (r+1) mod N of every rail: mark it with the owner's id, fill
    # the rest with a canary; afterwards every buffer must read owner(x) * 1000 + x mod 1000
    rnd = random.Random(N + 10 * R)
    n = rnd.randint(N, 900)
    seg = orc.segment_map(orc.rail_partition(n, [rnd.randint(1, 9) for _ in range(R)], 4, 16), N)
    want = np.empty(n, dtype=np.int32)
    bufs = [np.full(n, -7, dtype=np.int32) for _ in range(N)]
    for k in range(R):
        for j in range(N):
            owner = (j - 1) % N
            lo, hi = int(seg[k, j]), int(seg[k, j + 1])
            vals = owner * 1000 + (np.arange(lo, hi) % 1000)
            bufs[owner][lo:hi] = vals
            want[lo:hi] = vals
    orig = [b.copy() for b in bufs]
    out, sent = orc.ring_allgather(orc.I32, bufs, seg)
    for o in out:
        assert (o == want).all()
    assert int(sent.sum()) == (N - 1) * n * 4                       # half of Eq. 1's volume
    for b, o in zip(bufs, orig):                                    # the oracle works on private copies
        assert (b == o).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16", "i32"])
def test_reduce_scatter_then_allgather_is_the_allreduce(orc, dtype):
    N, n = 7, 501
    code = {"f32": orc.F32, "bf16": orc.BF16, "i32": orc.I32}[dtype]
    bufs = [inputs.to_host_storage(inputs.node_buffer(dtype, n, 31, i, std=1.0)) for i in range(N)]
    seg = orc.segment_map(orc.rail_partition(n, [5, 2, 1], bufs[0].itemsize, 16), N)
    full, sent_full = orc.ring_allreduce(code, bufs, seg)
    rs, sent_rs = orc.ring_allreduce(code, bufs, seg, reduce_scatter_only=True)
    both, sent_ag = orc.ring_allgather(code, rs, seg)
    for a, b in zip(full, both):
        assert np.array_equal(a, b)
    assert np.array_equal(sent_full, sent_rs + sent_ag)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "i32"])
@pytest.mark.parametrize("chunk", [1, 7, 64, 1000, 10**9])
def test_chunked_ring_is_the_ring_piece_by_piece(orc, dtype, chunk):
    # splitting a transfer changes how many messages there are, not what they add up to
    N, n = 5, 803
    code = {"f32": orc.F32, "bf16": orc.BF16, "i32": orc.I32}[dtype]
    bufs = [inputs.to_host_storage(inputs.node_buffer(dtype, n, 17, i, std=1.0)) for i in range(N)]
    seg = orc.segment_map(orc.rail_partition(n, [3, 1], bufs[0].itemsize, 16), N)
    plain, sent_plain = orc.ring_allreduce(code, bufs, seg)
    out, sent, msgs = orc.ring_allreduce_chunked(code, bufs, seg, chunk)
    for a, b in zip(plain, out):
        assert np.array_equal(a, b)
    assert np.array_equal(sent, sent_plain)                          # Eq. 1's volume is unchanged
    # message count, by hand: in both phases node r sends N-1 of the N segments of every rail
    # (all but segment r+1 while reducing, all but segment r+2 while gathering)
    lens = np.diff(seg.astype(np.int64), axis=1)                     # [R, N]
    pieces = -(-lens // chunk)                                       # ceil; 0 for empty segments
    for r in range(N):
        want = int(pieces.sum() - pieces[:, (r + 1) % N].sum() + pieces.sum() - pieces[:, (r + 2) % N].sum())
        assert int(msgs[r]) == want


def test_failover_target_is_the_survivor_with_most_data(orc):
    b = [0, 100, 400, 400, 900, 1000]                                # lengths 100, 300, 0, 500, 100
    assert orc.failover_target(b, [True] * 5) == 3
    assert orc.failover_target(b, [True, True, True, False, True]) == 1      # rail 3 failed
    assert orc.failover_target(b, [True, False, True, False, True]) == 0     # tie 100/100: lowest index
    assert orc.failover_target(b, [False, False, True, False, False]) == 2   # even an empty rail survives
    with pytest.raises(ValueError):
        orc.failover_target(b, [False] * 5)
