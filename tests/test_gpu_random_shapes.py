"""GPU parity on seeded random shapes: node count, rail count, weights (zeros included), element
count, element type and entry point are all drawn, so that combinations nobody picked by hand
get compared with the CPU oracle too.  Every case is named by its seed."""
import random

import numpy as np
import pytest
import torch

from paper_2405_17870_amd import inputs
from paper_2405_17870_amd import nezha_sim as nz

import gpu_util as gu

pytestmark = pytest.mark.gpu

N_CASES = 160


def _draw(seed):
    rng = random.Random(0x52414E44 + seed)
    N = rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 24, 31, 32, 33, 63, 64, 65, 100, 127, 128])
    R = rng.randint(1, 8)
    ratios = [rng.choice([0, 1, 1, 3, 10, 25, 40, 100, 1 << 20]) for _ in range(R)]
    if sum(ratios) == 0:
        ratios[rng.randrange(R)] = 1
    # few elements (empty segments), a few vectors, or several tiles per segment
    n = rng.choice([rng.randint(1, 200), rng.randint(200, 20_000), rng.randint(20_000, 400_000)])
    n = min(n, 3_000_000 // N)
    dtype = rng.choice(["f32", "bf16", "f16", "i32"])
    what = rng.choice(["fused", "ring", "rs-fused", "rs-ring", "ag-fused", "ag-ring", "chunked"])
    chunk = rng.choice([1, 3, 64, 1000, 4096, 1 << 40]) if what == "chunked" else None
    if what == "chunked" and chunk < 64:
        n = min(n, 2_000)           # pieces of one or three elements: keep the launch count small
    return N, tuple(ratios), n, dtype, what, chunk


@pytest.mark.parametrize("seed", range(N_CASES))
def test_random_case_matches_oracle(orc, seed):
    N, ratios, n, dtype, what, chunk = _draw(seed)
    print(f"seed={seed} N={N} ratios={ratios} n={n} dtype={dtype} what={what} chunk={chunk}", flush=True)
    e = inputs.ELEM_BYTES[dtype]
    code = gu.ORC_CODE[dtype]
    host = [inputs.node_buffer(dtype, n, 900 + seed, i, std=1.0) for i in range(N)]
    host_np = [inputs.to_host_storage(t) for t in host]
    seg = orc.segment_map(orc.rail_partition(n, ratios, e), N)
    ins = gu.device_inputs(host, dtype)
    outs = gu.fresh_outputs(N, n, dtype)
    tin, tout = [g.t for g in ins], [g.t for g in outs]

    if what == "fused":
        nz.nz_allreduce_sim(tin, n, ratios, dtype, "fused", tout)
        torch.cuda.synchronize()
        got0 = outs[0].host()
        gu.check_fused_against_oracle(orc, dtype, got0, host_np, f"seed {seed}")
        for g in outs:
            assert np.array_equal(g.host(), got0)
    elif what in ("ring", "chunked"):
        if what == "ring":
            nz.nz_allreduce_sim(tin, n, ratios, dtype, "ring-stepwise", tout)
            want, _ = orc.ring_allreduce(code, host_np, seg)
        else:
            nz.nz_allreduce_sim_chunked(tin, n, ratios, dtype, chunk, tout)
            want = orc.ring_allreduce_chunked(code, host_np, seg, chunk)[0]
        torch.cuda.synchronize()
        for i, g in enumerate(outs):
            gu.assert_same_bits(g.host(), want[i], dtype, f"seed {seed} node {i}")
    elif what in ("rs-fused", "rs-ring"):
        mode = "fused" if what == "rs-fused" else "ring-stepwise"
        nz.nz_reduce_scatter_sim(tin, n, ratios, dtype, mode, tout)
        torch.cuda.synchronize()
        want, _ = orc.ring_allreduce(code, host_np, seg, reduce_scatter_only=True)
        for r, g in enumerate(outs):
            j = (r + 1) % N                      # the segment node r owns, on every rail
            got = g.host()
            for k in range(len(ratios)):
                lo, hi = int(seg[k, j]), int(seg[k, j + 1])
                if lo == hi:
                    continue
                if what == "rs-ring":
                    gu.assert_same_bits(got[lo:hi], want[r][lo:hi], dtype, f"seed {seed} owner {r}")
                else:
                    gu.check_fused_against_oracle(orc, dtype, got[lo:hi], [h[lo:hi] for h in host_np],
                                                  f"seed {seed} owner {r}")
    else:
        # allgather: node r enters holding only its owned segments (the rest is a canary)
        mode = "fused" if what == "ag-fused" else "ring-stepwise"
        start = []
        for r in range(N):
            a = np.full_like(host_np[r], 0x5A5A if e == 2 else 0x5A5A5A5A)
            j = (r + 1) % N
            for k in range(len(ratios)):
                lo, hi = int(seg[k, j]), int(seg[k, j + 1])
                a[lo:hi] = host_np[r][lo:hi]
            start.append(a)
        bufs = gu.device_inputs([inputs.from_host_storage(a, dtype) for a in start], dtype)
        nz.nz_allgather_sim([g.t for g in bufs], n, ratios, dtype, mode)
        torch.cuda.synchronize()
        want, _ = orc.ring_allgather(code, start, seg)
        for i, g in enumerate(bufs):
            assert np.array_equal(g.host(), want[i]), f"seed {seed} node {i}"
            assert g.guards_intact()

    for g in outs:
        assert g.guards_intact()
    for i, g in enumerate(ins):
        assert g.guards_intact() and np.array_equal(g.host(), host_np[i])
