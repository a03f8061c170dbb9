"""GPU parity of nz_reduce_scatter_sim / nz_allgather_sim against the CPU oracle (C-ABI)."""
import numpy as np
import pytest
import torch

from paper_2405_17870_amd import inputs
from paper_2405_17870_amd import nezha_sim as nz

import gpu_util as gu

pytestmark = pytest.mark.gpu

SHAPES = [(1, (1,), 777), (2, (3, 1), 63), (3, (3, 1), 200), (8, (100, 40), 70_001),
          (5, (7, 0, 3), 4_097), (32, (100, 25), 100_003), (128, (100, 100, 40, 10), 33_333),
          (9, (5,), 300_000)]


def _owned(seg, N, r):
    j = (r + 1) % N
    return [(int(seg[k, j]), int(seg[k, j + 1])) for k in range(seg.shape[0])]


@pytest.mark.parametrize("mode", ["fused", "ring-stepwise"])
@pytest.mark.parametrize("dtype", ["f32", "i32", "bf16", "f16"])
@pytest.mark.parametrize("N,ratios,n", SHAPES)
def test_reduce_scatter_owned_segments(orc, mode, dtype, N, ratios, n):
    print(f"reduce-scatter mode={mode} dtype={dtype} N={N} ratios={ratios} n={n}", flush=True)
    host = [inputs.node_buffer(dtype, n, 41 + N, i, std=1.0) for i in range(N)]
    host_np = [inputs.to_host_storage(t) for t in host]
    ins = gu.device_inputs(host, dtype)
    outs = gu.fresh_outputs(N, n, dtype)
    nz.nz_reduce_scatter_sim([g.t for g in ins], n, ratios, dtype, mode, [g.t for g in outs])
    torch.cuda.synchronize()
    e = inputs.ELEM_BYTES[dtype]
    seg = orc.segment_map(orc.rail_partition(n, ratios, e), N)
    if mode == "ring-stepwise":
        want, _ = orc.ring_allreduce(gu.ORC_CODE[dtype], host_np, seg, reduce_scatter_only=True)
        for r in range(N):
            got = outs[r].host()
            for lo, hi in _owned(seg, N, r):
                gu.assert_same_bits(got[lo:hi], want[r][lo:hi], dtype, f"node {r} owned")
    else:
        # owned segments against the definitional sum; everything else untouched (canary 0xC3)
        full = gu.fresh_outputs(N, n, dtype)
        gu.allreduce(ins, full, ratios, "fused")
        ref = full[0].host()
        gu.check_fused_against_oracle(orc, dtype, ref, host_np, "allreduce reference")
        for r in range(N):
            got = outs[r].host()
            mask = np.zeros(n, dtype=bool)
            for lo, hi in _owned(seg, N, r):
                mask[lo:hi] = True
            assert np.array_equal(got[mask], ref[mask])          # bitwise the allreduce's sums
            assert (got[~mask].view(np.uint8) == 0xC3).all()
    assert all(g.guards_intact() for g in outs + ins)


@pytest.mark.parametrize("mode", ["fused", "ring-stepwise"])
@pytest.mark.parametrize("e", [2, 4])
@pytest.mark.parametrize("N,ratios,n", SHAPES)
def test_allgather_spreads_owner_segments(orc, mode, e, N, ratios, n):
    print(f"allgather mode={mode} e={e} N={N} ratios={ratios} n={n}", flush=True)
    dtype = "i32" if e == 4 else "bf16"
    seg = orc.segment_map(orc.rail_partition(n, ratios, e), N)
    rng = np.random.default_rng(N * 7 + e)
    np_dt = np.int32 if e == 4 else np.uint16
    host = [rng.integers(0, 60000, size=n).astype(np_dt) for _ in range(N)]
    want, _ = orc.ring_allgather(gu.ORC_CODE[dtype], host, seg)
    bufs = [gu.Guarded(n, dtype) for _ in range(N)]
    for g, h in zip(bufs, host):
        g.t.view(torch.uint8).copy_(torch.from_numpy(h.view(np.uint8)))
    nz.nz_allgather_sim([g.t for g in bufs], n, ratios, dtype, mode)
    torch.cuda.synchronize()
    for r in range(N):
        assert np.array_equal(bufs[r].host().view(np_dt), want[r]), r
        assert bufs[r].guards_intact()
    assert all(np.array_equal(want[0], w) for w in want[1:])


@pytest.mark.parametrize("mode", ["fused", "ring-stepwise"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_reduce_scatter_then_allgather_equals_allreduce_bitwise(orc, mode, dtype):
    N, n, ratios = 12, 200_003, (100, 100, 40)
    host = [inputs.node_buffer(dtype, n, 3, i, std=1e-2) for i in range(N)]
    ins = gu.device_inputs(host, dtype)
    ref = gu.fresh_outputs(N, n, dtype)
    gu.allreduce(ins, ref, ratios, mode)
    outs = gu.fresh_outputs(N, n, dtype)
    nz.nz_reduce_scatter_sim([g.t for g in ins], n, ratios, dtype, mode, [g.t for g in outs])
    nz.nz_allgather_sim([g.t for g in outs], n, ratios, dtype, mode)
    torch.cuda.synchronize()
    for a, b in zip(ref, outs):
        assert np.array_equal(a.host(), b.host())
    # in place reduce-scatter
    nz.nz_reduce_scatter_sim([g.t for g in ins], n, ratios, dtype, mode, [g.t for g in ins])
    nz.nz_allgather_sim([g.t for g in ins], n, ratios, dtype, mode)
    torch.cuda.synchronize()
    for a, b in zip(ref, ins):
        assert np.array_equal(a.host(), b.host())


def test_phase_argument_errors():
    N, n = 4, 1000
    bufs = [gu.Guarded(n, "f32") for _ in range(N)]
    t = [g.t for g in bufs]
    with pytest.raises(nz.NezhaSimError) as ex:
        nz.nz_allgather_sim([t[0], t[0], t[2], t[3]], n, (1,), "f32", "fused")
    assert ex.value.status == 3
    with pytest.raises(nz.NezhaSimError) as ex:
        nz.nz_reduce_scatter_sim(t, n, (1,), "f32", "fused", [t[1], t[0], t[2], t[3]])
    assert ex.value.status == 3
    with pytest.raises(nz.NezhaSimError) as ex:
        nz.nz_allgather_sim(t, n, (0,), "f32", "ring-stepwise")
    assert ex.value.status == 1
