"""The harness's HBM arena hands out aligned, disjoint tensors inside the requested regions."""
import numpy as np
import pytest
import torch

from paper_2405_17870_amd import inputs
from paper_2405_17870_amd import nezha_sim as nz
from paper_2405_17870_amd import placement

import gpu_util as gu

pytestmark = pytest.mark.gpu


def test_arena_regions_alignment_and_use():
    arena = placement.try_arena("cuda:0")
    if arena is None:
        pytest.skip("not enough free HBM for a three-region arena")
    base = arena.raw.data_ptr()
    seen = []
    for region in (0, 1, 2):
        for n, dt in ((1000, torch.float32), (3, torch.bfloat16), (5_000_001, torch.int32)):
            t = arena.alloc(n, dt, region)
            off = t.data_ptr() - base
            assert t.numel() == n and t.dtype == dt
            assert t.data_ptr() % 256 == 0
            assert region * placement.REGION_BYTES <= off
            assert off + t.numel() * t.element_size() <= (region + 1) * placement.REGION_BYTES
            seen.append((off, off + t.numel() * t.element_size()))
    seen.sort()
    assert all(a[1] <= b[0] for a, b in zip(seen, seen[1:]))            # disjoint
    striped = arena.alloc_striped(7, 4096, torch.float32)
    regions = [(t.data_ptr() - base) // placement.REGION_BYTES for t in striped]
    assert regions == [0, 1, 2, 0, 1, 2, 0]
    # the tensors are ordinary device memory for the library
    ins = arena.alloc_striped(4, 4096, torch.float32)
    for i, t in enumerate(ins):
        t.fill_(float(i + 1))
    outs = arena.alloc_striped(4, 4096, torch.float32, start=1)
    nz.nz_allreduce_sim(ins, 4096, (3, 1), "f32", "fused", outs)
    torch.cuda.synchronize()
    assert all(bool((o == 10.0).all()) for o in outs)
    with pytest.raises(RuntimeError):
        arena.alloc(placement.REGION_BYTES, torch.uint8, 1)            # does not fit what is left


def test_outputs_spread_over_regions_take_the_single_launch(orc):
    """Up to 16 output buffers that span more than a region's length are written by the
    single-launch kernel however large the job (with plain allocations the same job runs as
    the pipeline); 17 spread outputs take the pipeline again.  Same bits either way, and the
    oracle's sums."""
    arena = placement.try_arena("cuda:0")
    if arena is None:
        pytest.skip("not enough free HBM for a three-region arena")
    for N, dtype, ratios in ((8, "bf16", (100, 100, 40)), (16, "f32", (100, 40)), (17, "f32", (3, 1))):
        tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        e = inputs.ELEM_BYTES[dtype]
        n = -(-(128 << 20) // (N * e)) + 77
        print(f"spread outputs N={N} {dtype} n={n}", flush=True)
        ins = [arena.alloc(n, tdt, 0) for _ in range(N)]
        for i, t in enumerate(ins):
            t.copy_(inputs.node_buffer(dtype, n, 900 + N, i, device="cuda:0", std=1e-2))
        outs = arena.alloc_striped(N, n, tdt)
        for t in outs:
            t.zero_()
        span = max(t.data_ptr() for t in outs) + n * e - min(t.data_ptr() for t in outs)
        assert span > nz.NZ_HBM_REGION_BYTES
        assert (nz.nz_allreduce_launches(N, n, ratios, dtype, "fused", N, span) == 1) == (N <= 16)
        assert nz.nz_allreduce_launches(N, n, ratios, dtype, "fused", N) > 1
        nz.nz_allreduce_sim(ins, n, ratios, dtype, "fused", outs)
        near = [torch.zeros_like(t) for t in ins]                       # plain allocations: the pipeline
        nz.nz_allreduce_sim(ins, n, ratios, dtype, "fused", near)
        torch.cuda.synchronize()
        host = [inputs.to_host_storage(t) for t in ins]
        gu.check_fused_against_oracle(orc, dtype, inputs.to_host_storage(outs[N - 1]), host, f"spread N={N}")
        for a, b in zip(outs, near):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))


def test_pack_into_send_buffers_spread_over_regions(orc):
    """Send buffers that span more than a region while the node buffers do not: the copy kernel
    then runs with the node index fastest.  Whole rail (aligned runs) and the order a node sends
    in (runs not aligned with their place in the send buffer); bytes against the oracle."""
    arena = placement.try_arena("cuda:0")
    if arena is None:
        pytest.skip("not enough free HBM for a three-region arena")
    N, ratios, n, e = 8, (100, 40), 700_001, 2
    seg = nz.nz_segment_map(nz.nz_rail_partition(n, e, ratios), N)
    rng = np.random.default_rng(5)
    host = [rng.integers(0, 256, size=n * e, dtype=np.uint8) for _ in range(N)]
    node = [arena.alloc(n, torch.bfloat16, 0) for _ in range(N)]
    for t, h in zip(node, host):
        t.view(torch.uint8).copy_(torch.from_numpy(h))
    for rail, ids in ((0, list(range(N))), (1, [(3 - s) % N for s in range(N)]), (0, [5, 2, 7])):
        total = sum(int(seg[rail, j + 1] - seg[rail, j]) for j in ids) * e
        send = arena.alloc_striped(N, total // e + 64, torch.bfloat16)
        assert max(t.data_ptr() for t in send) - min(t.data_ptr() for t in send) > nz.NZ_HBM_REGION_BYTES
        for t in send:
            t.view(torch.uint8).fill_(0xEE)
        assert nz.nz_pack(node, seg, rail, ids, e, send, total + 128) == total
        torch.cuda.synchronize()
        for m in range(N):
            want, nbytes = orc.pack(host[m], seg, rail, ids, e)
            got = send[m].view(torch.uint8).cpu().numpy()
            assert nbytes == total and np.array_equal(got[:total], want), (rail, m)
            assert (got[total:] == 0xEE).all()
