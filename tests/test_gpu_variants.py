"""GPU parity of the Ring_Chunked allreduce and of the failover allreduce (C-ABI)."""
import numpy as np
import pytest
import torch

from paper_2405_17870_amd import inputs
from paper_2405_17870_amd import nezha_sim as nz

import gpu_util as gu

pytestmark = pytest.mark.gpu

SHAPES = [(2, (3, 1), 63), (3, (3, 1), 200), (8, (100, 40), 70_001), (5, (7, 0, 3), 4_097),
          (32, (100, 25), 100_003), (128, (100, 100, 40, 10), 33_333)]


@pytest.mark.parametrize("dtype", ["f32", "bf16", "i32", "f16"])
@pytest.mark.parametrize("N,ratios,n", SHAPES)
def test_chunked_ring_matches_oracle_bit_for_bit(orc, dtype, N, ratios, n):
    e = inputs.ELEM_BYTES[dtype]
    seg = orc.segment_map(orc.rail_partition(n, ratios, e), N)
    longest = int(np.diff(seg.astype(np.int64), axis=1).max())
    host = [inputs.node_buffer(dtype, n, 51 + N, i, std=1.0) for i in range(N)]
    host_np = [inputs.to_host_storage(t) for t in host]
    for chunk in sorted({1 if longest < 50 else max(longest // 7, 1), max(longest // 2 + 1, 1), 513, longest,
                         10 * longest + 1}):
        print(f"chunked dtype={dtype} N={N} ratios={ratios} n={n} chunk={chunk}", flush=True)
        want, _, _ = orc.ring_allreduce_chunked(gu.ORC_CODE[dtype], host_np, seg, chunk)
        ins = gu.device_inputs(host, dtype)
        outs = gu.fresh_outputs(N, n, dtype)
        nz.nz_allreduce_sim_chunked([g.t for g in ins], n, ratios, dtype, chunk, [g.t for g in outs])
        torch.cuda.synchronize()
        for i in range(N):
            gu.assert_same_bits(outs[i].host(), want[i], dtype, f"chunk {chunk} node {i}")
            assert outs[i].guards_intact() and ins[i].guards_intact()


def test_chunked_rejects_zero_chunk():
    bufs = [gu.Guarded(100, "f32") for _ in range(2)]
    with pytest.raises(nz.NezhaSimError) as ex:
        nz.nz_allreduce_sim_chunked([g.t for g in bufs], 100, (1,), "f32", 0, [g.t for g in bufs])
    assert ex.value.status == 1


@pytest.mark.parametrize("mode", ["fused", "ring-stepwise"])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "i32"])
def test_failover_gives_the_same_result_and_picks_the_oracle_target(orc, mode, dtype):
    N, n = 6, 150_001
    e = inputs.ELEM_BYTES[dtype]
    host = [inputs.node_buffer(dtype, n, 77, i, std=1e-2) for i in range(N)]
    ins = gu.device_inputs(host, dtype)
    for ratios in [(100, 40), (100, 100, 40, 10), (1, 0, 5), (0, 1), (3, 3, 3)]:
        ref = gu.fresh_outputs(N, n, dtype)
        gu.allreduce(ins, ref, ratios, mode)
        b = orc.rail_partition(n, ratios, e)
        for failed in range(len(ratios)):
            print(f"failover mode={mode} dtype={dtype} ratios={ratios} failed={failed}", flush=True)
            alive = [k != failed for k in range(len(ratios))]
            outs = gu.fresh_outputs(N, n, dtype)
            t = nz.nz_allreduce_sim_failover([g.t for g in ins], n, ratios, dtype, mode,
                                             [g.t for g in outs], failed)
            torch.cuda.synchronize()
            assert t == orc.failover_target(b, alive) == nz.nz_failover_target(b, alive)
            for a, o in zip(ref, outs):
                assert np.array_equal(a.host(), o.host())
                assert o.guards_intact()
    # oracle cross-check of the reference itself, once (last ratios)
    host_np = [inputs.to_host_storage(t) for t in host]
    if mode == "fused":
        gu.check_fused_against_oracle(orc, dtype, ref[0].host(), host_np, "ref")
    else:
        want, _ = orc.ring_allreduce(gu.ORC_CODE[dtype], host_np, orc.segment_map(b, N))
        gu.assert_same_bits(ref[0].host(), want[0], dtype, "ref ring")


def test_failover_errors(orc):
    bufs = [gu.Guarded(1000, "f32") for _ in range(2)]
    t = [g.t for g in bufs]
    with pytest.raises(nz.NezhaSimError) as ex:
        nz.nz_allreduce_sim_failover(t, 1000, (1,), "f32", "fused", t, 0)       # the only rail fails
    assert ex.value.status == 1
    with pytest.raises(nz.NezhaSimError) as ex:
        nz.nz_allreduce_sim_failover(t, 1000, (1, 1), "f32", "fused", t, 2)     # no such rail
    assert ex.value.status == 1
    with pytest.raises(nz.NezhaSimError):
        nz.nz_failover_target([0, 10, 20], [False, False])
