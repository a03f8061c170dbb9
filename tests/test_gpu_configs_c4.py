"""GPU parity on the largest benchmark shape (32 nodes x 335,000,000 bf16, rails 100:25; 21 GB
of inputs), in the launch configuration the benchmark times.

Fused mode: every sum against the oracle, in element-range chunks.  Ring-stepwise: the oracle's
literal ring on sampled windows (both ends, the rail boundary, segment boundaries, random
places) under the segment table clipped to the window.  Whole-rail pack / unpack: bytes of
sampled nodes against the oracle, and the packed route gives bitwise the same sums.  Inputs are
synthetic gradients (see paper_2405_17870_amd/inputs.py)."""
import numpy as np
import pytest
import torch

from paper_2405_17870_amd import inputs
from paper_2405_17870_amd import nezha_sim as nz
from paper_2405_17870_amd import placement

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _all_equal(outs):
    return all(torch.equal(outs[0], o) for o in outs[1:])


def _points_c4(w, orc, rng):
    b = orc.rail_partition(w.n_elems, w.ratios, 2)
    seg = orc.segment_map(b, w.n_nodes)
    pts = [0, w.n_elems, int(b[1]), int(seg[0, 1]), int(seg[0, 17]), int(seg[1, 1]), int(seg[1, 5]),
           int(seg[1, 31])]
    pts += [int(x) for x in rng.integers(0, w.n_elems, size=6)]
    half = 40_000
    return seg, [(max(0, p - half), min(w.n_elems, p + half)) for p in pts]


@pytest.fixture(scope="module")
def c4():
    """The workload on the device, placed as the benchmark places it; built once for this file
    (generating it takes longer than any single check) and released at the end of the file."""
    w = inputs.WORKLOADS["c4"]
    N, n = w.n_nodes, w.n_elems
    _say("c4: generating 32 x 335M bf16")
    torch.cuda.empty_cache()
    arena = placement.try_arena(gu.DEV)
    if arena is not None:
        ins = [arena.alloc(n, torch.bfloat16, 0) for _ in range(N)]
        for i in range(N):
            ins[i].copy_(inputs.node_buffer(w.dtype, n, w.seed, i, device=gu.DEV, std=w.std))
        outs = arena.alloc_striped(N, n, torch.bfloat16)
    else:
        ins = inputs.workload_buffers(w, device=gu.DEV)
        outs = [torch.empty_like(t) for t in ins]
    state = [w, arena, ins, outs]
    yield state
    state.clear()
    del arena, ins, outs
    torch.cuda.empty_cache()


def test_c4_fused_whole_range(orc, c4):
    """Every one of the 335 M sums against the oracle, in element-range chunks (32 slices of
    16 MB at a time through pinned host memory), plus bitwise equality of all 32 outputs."""
    w, arena, ins, outs = c4[:4]
    N, n = w.n_nodes, w.n_elems
    for t in outs:
        t.zero_()
    _say("c4: fused")
    nz.nz_allreduce_sim(ins, n, w.ratios, w.dtype, "fused", outs)
    torch.cuda.synchronize()
    assert _all_equal(outs)
    C = 8 << 20
    stage = [torch.empty((N + 1, C), dtype=torch.bfloat16, pin_memory=True) for _ in range(2)]
    ready = [None, None]
    spans = [(lo, min(lo + C, n)) for lo in range(0, n, C)]

    def issue(c):
        lo, hi = spans[c]
        buf = stage[c % 2]
        for i in range(N):
            buf[i, :hi - lo].copy_(ins[i][lo:hi], non_blocking=True)
        buf[N, :hi - lo].copy_(outs[N // 2][lo:hi], non_blocking=True)
        ev = torch.cuda.Event()
        ev.record()
        ready[c % 2] = ev

    issue(0)
    escapes = checked = 0
    for c, (lo, hi) in enumerate(spans):
        ready[c % 2].synchronize()
        rows = stage[c % 2].view(torch.int16).numpy().view(np.uint16)
        host = [rows[i, :hi - lo] for i in range(N)]
        got = rows[N, :hi - lo]
        if c + 1 < len(spans):
            issue(c + 1)
        escapes += gu.check_fused_against_oracle(orc, "bf16", got, host, f"c4[{lo}:{hi}]")
        checked += hi - lo
        if c == len(spans) // 2:
            # the check does look at every element: one value of a host copy moved by four ulps
            # must be caught
            wrong = got.copy()
            wrong[12345] += 4
            with pytest.raises(AssertionError):
                gu.check_fused_against_oracle(orc, "bf16", wrong, host, "planted")
    assert checked == n
    _say(f"c4: all {n} sums checked; cancellation clause used for {escapes} elements")
    assert escapes <= n // 1_000_000


def test_c4_ring_stepwise_windows(orc, c4):
    """The 62 ring steps at full size (670 MB per step: the streaming step kernels), checked
    bit for bit on sampled windows: the oracle's literal ring runs on the 32 extracted windows
    under the segment table clipped to the window and re-based to its start."""
    w, arena, ins, outs = c4[:4]
    N, n = w.n_nodes, w.n_elems
    for t in outs:
        t.zero_()
    _say("c4: ring-stepwise")
    nz.nz_allreduce_sim(ins, n, w.ratios, w.dtype, "ring-stepwise", outs)
    torch.cuda.synchronize()
    assert _all_equal(outs)
    seg, windows = _points_c4(w, orc, np.random.default_rng(5))
    for lo, hi in windows:
        host = [inputs.to_host_storage(t[lo:hi]) for t in ins]
        local = (np.clip(seg.astype(np.int64), lo, hi) - lo).astype(np.uint64)
        want, _ = orc.ring_allreduce(orc.BF16, host, local)
        for i in (0, 1, N // 2, N - 1):
            gu.assert_same_bits(inputs.to_host_storage(outs[i][lo:hi]), want[i], "bf16",
                                f"c4 ring [{lo}:{hi}] node {i}")
        assert all(np.array_equal(want[0], x) for x in want[1:])


def _second_outputs(c4):
    """A second set of 32 result buffers, made on first use and kept for the rest of the file."""
    w, arena, ins, outs = c4[:4]
    if len(c4) == 4:
        c4.append(arena.alloc_striped(w.n_nodes, w.n_elems, torch.bfloat16, start=1) if arena is not None
                  else [torch.empty_like(t) for t in ins])
    return c4[4]


def _canary(bufs):
    for t in bufs:
        t.view(torch.uint8).fill_(0xC3)


@pytest.mark.parametrize("mode", ["fused", "ring-stepwise"])
def test_c4_phases_at_full_size(orc, c4, mode):
    """Reduce-scatter alone and allgather alone at full size (the direct allgather works through
    each rail in many cache-sized pieces here; small shapes have one).  The allreduce of the
    same mode, checked against the oracle on sampled windows, is the reference: after the
    reduce-scatter node r holds exactly its own segments of it and nothing else was written;
    after the allgather every node holds all of it."""
    w, arena, ins, outs = c4[:4]
    N, n = w.n_nodes, w.n_elems
    second = _second_outputs(c4)
    _say(f"c4 phases: {mode} allreduce as the reference")
    nz.nz_allreduce_sim(ins, n, w.ratios, w.dtype, mode, outs)
    torch.cuda.synchronize()
    assert _all_equal(outs)
    seg, windows = _points_c4(w, orc, np.random.default_rng(11))
    for lo, hi in windows[:8:2] + windows[-2:]:
        host = [inputs.to_host_storage(t[lo:hi]) for t in ins]
        got = inputs.to_host_storage(outs[N - 1][lo:hi])
        if mode == "fused":
            gu.check_fused_against_oracle(orc, "bf16", got, host, f"c4 [{lo}:{hi}]")
        else:
            local = (np.clip(seg.astype(np.int64), lo, hi) - lo).astype(np.uint64)
            want, _ = orc.ring_allreduce(orc.BF16, host, local)
            gu.assert_same_bits(got, want[N - 1], "bf16", f"c4 ring [{lo}:{hi}]")
    ref = outs[0]
    _say(f"c4 phases: {mode} reduce-scatter")
    _canary(second)
    nz.nz_reduce_scatter_sim(ins, n, w.ratios, w.dtype, mode, second)
    torch.cuda.synchronize()
    if mode == "fused":
        for r in range(N):
            j = (r + 1) % N
            edge = 0
            for k in range(seg.shape[0]):
                lo, hi = int(seg[k, j]), int(seg[k, j + 1])
                assert torch.equal(second[r][lo:hi], ref[lo:hi]), (r, k)
                assert bool((second[r][edge:lo].view(torch.uint8) == 0xC3).all()), (r, k)
                edge = hi
            assert bool((second[r][edge:].view(torch.uint8) == 0xC3).all()), r
    else:
        # the ring's reduce-scatter leaves partial sums in the other segments; the owned ones
        # are final
        for r in range(N):
            j = (r + 1) % N
            for k in range(seg.shape[0]):
                lo, hi = int(seg[k, j]), int(seg[k, j + 1])
                assert torch.equal(second[r][lo:hi], ref[lo:hi]), (r, k)
    _say(f"c4 phases: {mode} allgather")
    nz.nz_allgather_sim(second, n, w.ratios, w.dtype, mode)
    torch.cuda.synchronize()
    for r in range(N):
        assert torch.equal(second[r], ref), r


def test_c4_chunked_and_failover_at_full_size(orc, c4):
    """Ring_Chunked (pieces of 1 Mi and of 256 Ki elements, the benchmark's settings) gives the
    stepwise ring's bits, the failover allreduce the fused sums, whichever rail fails; the two
    references are checked against the oracle by the tests above."""
    w, arena, ins, outs = c4[:4]
    N, n = w.n_nodes, w.n_elems
    second = _second_outputs(c4)
    nz.nz_allreduce_sim(ins, n, w.ratios, w.dtype, "ring-stepwise", outs)
    for chunk in (1 << 20, 1 << 18):
        _say(f"c4: Ring_Chunked, pieces of {chunk} elements")
        _canary(second)
        nz.nz_allreduce_sim_chunked(ins, n, w.ratios, w.dtype, chunk, second)
        torch.cuda.synchronize()
        for r in range(N):
            assert torch.equal(second[r], outs[r]), (chunk, r)
    nz.nz_allreduce_sim(ins, n, w.ratios, w.dtype, "fused", outs)
    b = orc.rail_partition(n, w.ratios, 2)
    for failed in range(len(w.ratios)):
        _say(f"c4: failover, rail {failed} fails")
        _canary(second)
        took = nz.nz_allreduce_sim_failover(ins, n, w.ratios, w.dtype, "fused", second, failed)
        torch.cuda.synchronize()
        alive = [k != failed for k in range(len(w.ratios))]
        assert took == orc.failover_target(b, alive)
        for r in range(N):
            assert torch.equal(second[r], outs[0]), (failed, r)


def test_c4_pack_route_unpack(orc, c4):
    """Whole-rail pack and unpack at full size: packed bytes and unpacked bytes of sampled
    nodes against the oracle; the route pack -> fused allreduce of the send buffers -> unpack
    gives bitwise the sums of the direct call."""
    w, arena, ins, outs = c4[:4]
    N, n = w.n_nodes, w.n_elems
    nz.nz_allreduce_sim(ins, n, w.ratios, w.dtype, "fused", outs)
    b = nz.nz_rail_partition(n, 2, w.ratios)
    seg = nz.nz_segment_map(b, N)
    oseg = orc.segment_map(orc.rail_partition(n, w.ratios, 2), N)
    assert np.array_equal(seg, oseg)
    if arena is not None:
        routed = arena.alloc_striped(N, n, torch.bfloat16, start=1)
        for t in routed:
            t.zero_()
    else:
        routed = [torch.zeros_like(t) for t in ins]
    ids = list(range(N))
    sampled = (0, 13, N - 1)
    host = {m: inputs.to_host_storage(ins[m]) for m in sampled}
    for rail in range(len(w.ratios)):
        L = int(b[rail + 1] - b[rail])
        send = (arena.alloc_striped(N, L, torch.bfloat16, start=2) if arena is not None
                else [torch.empty(L, dtype=torch.bfloat16, device=gu.DEV) for _ in range(N)])
        assert nz.nz_pack(ins, seg, rail, ids, 2, send, L * 2) == L * 2
        torch.cuda.synchronize()
        for m in sampled:
            want, count = orc.pack(host[m], oseg, rail, ids, 2)
            assert count == L * 2
            assert np.array_equal(send[m].view(torch.uint8).cpu().numpy(), want), (rail, m)
        nz.nz_allreduce_sim(send, L, (1,), "bf16", "fused", send)
        nz.nz_unpack(send, seg, rail, ids, 2, routed)
        torch.cuda.synchronize()
        for m in sampled[:1]:
            ref = np.zeros(n * 2, dtype=np.uint8)
            orc.unpack(send[m].view(torch.uint8).cpu().numpy(), oseg, rail, ids, 2, ref)
            lo, hi = int(b[rail]), int(b[rail + 1])
            assert np.array_equal(routed[m][lo:hi].view(torch.uint8).cpu().numpy(), ref[2 * lo:2 * hi])
        del send
    for i in range(N):
        assert torch.equal(routed[i], outs[0]), i
