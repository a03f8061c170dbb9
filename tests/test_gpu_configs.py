"""GPU parity at the five benchmark shapes, in the launch configuration the benchmark times.

c1, c2, c3 and c5 are compared with the oracle element by element at full size in both modes
(the 21 GB shape has a file of its own, test_gpu_configs_c4.py).  Inputs are synthetic gradients of the shapes'
sizes (see paper_2405_17870_amd/inputs.py)."""
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


def _run(w, mode, ins):
    outs = [torch.empty_like(t) for t in ins]
    nz.nz_allreduce_sim(ins, w.n_elems, w.ratios, w.dtype, mode, outs)
    torch.cuda.synchronize()
    return outs


def _all_equal(outs):
    return all(torch.equal(outs[0], o) for o in outs[1:])


@pytest.mark.parametrize("name", ["c1", "c1_i32", "c2"])
def test_full_compare_both_modes(orc, name):
    w = inputs.WORKLOADS[name]
    _say(f"{name}: generating")
    ins = inputs.workload_buffers(w, device=gu.DEV)
    host = [inputs.to_host_storage(t) for t in ins]
    _say(f"{name}: fused")
    outs = _run(w, "fused", ins)
    assert _all_equal(outs)
    gu.check_fused_against_oracle(orc, w.dtype, inputs.to_host_storage(outs[0]), host, name)
    _say(f"{name}: ring-stepwise")
    outs = _run(w, "ring-stepwise", ins)
    seg = orc.segment_map(orc.rail_partition(w.n_elems, w.ratios, 4), w.n_nodes)
    want, sent = orc.ring_allreduce(gu.ORC_CODE[w.dtype], host, seg)
    assert int(sent.sum()) == 2 * (w.n_nodes - 1) * w.payload_bytes          # Eq. 1
    for i in range(w.n_nodes):
        gu.assert_same_bits(inputs.to_host_storage(outs[i]), want[i], w.dtype, f"{name} ring node {i}")
    gu.check_fused_against_oracle(orc, w.dtype, inputs.to_host_storage(outs[0]), host, name + " ring")


@pytest.mark.parametrize("name", ["c3", "c3_f16"])
def test_c3_16bit_outliers_full_compare(orc, name):
    """Fused and ring-stepwise at full size.  One ring step moves 277 MB here, more than the
    last-level cache keeps, so the ring runs the streaming form of the step kernels (the form
    the benchmark times on the large workloads)."""
    w = inputs.WORKLOADS[name]
    _say(f"{name}: generating")
    ins = inputs.workload_buffers(w, device=gu.DEV)
    outs = _run(w, "fused", ins)
    assert _all_equal(outs)
    _say(f"{name}: oracle sum")
    host = [inputs.to_host_storage(t) for t in ins]
    n_escape = gu.check_fused_against_oracle(orc, w.dtype, inputs.to_host_storage(outs[0]), host, name)
    _say(f"{name}: elements judged by the cancellation clause: {n_escape} of {w.n_elems}")
    assert n_escape <= w.n_elems // 1_000_000
    del outs
    _say(f"{name}: ring-stepwise")
    outs = _run(w, "ring-stepwise", ins)
    assert _all_equal(outs)
    got = inputs.to_host_storage(outs[0])
    del outs
    seg = orc.segment_map(orc.rail_partition(w.n_elems, w.ratios, 2), w.n_nodes)
    want, sent = orc.ring_allreduce(gu.ORC_CODE[w.dtype], host, seg)
    assert int(sent.sum()) == 2 * (w.n_nodes - 1) * w.payload_bytes          # Eq. 1
    gu.assert_same_bits(got, want[0], w.dtype, f"{name} ring")
    assert all(np.array_equal(want[0], x) for x in want[1:])


@pytest.mark.parametrize("dtype", ["f32", "i32"])
def test_streaming_ring_steps_32bit(orc, dtype):
    """More than 128 MiB per ring step with 4-byte elements (the streaming form of the step
    kernels), odd sizes, three rails, against the oracle's literal ring."""
    N, n, ratios = 3, 40_000_003, (3, 1, 2)
    ins = [inputs.node_buffer(dtype, n, 97, i, device=gu.DEV, std=1.0) for i in range(N)]
    host = [inputs.to_host_storage(t) for t in ins]
    outs = [torch.empty_like(t) for t in ins]
    nz.nz_allreduce_sim(ins, n, ratios, dtype, "ring-stepwise", outs)
    torch.cuda.synchronize()
    seg = orc.segment_map(orc.rail_partition(n, ratios, 4), N)
    want, sent = orc.ring_allreduce(gu.ORC_CODE[dtype], host, seg)
    assert int(sent.sum()) == 2 * (N - 1) * n * 4
    for i in range(N):
        gu.assert_same_bits(inputs.to_host_storage(outs[i]), want[i], dtype, f"{dtype} ring node {i}")
    # the two halves on their own take the same route through the step kernels
    nz.nz_reduce_scatter_sim(ins, n, ratios, dtype, "ring-stepwise", outs)
    nz.nz_allgather_sim(outs, n, ratios, dtype, "ring-stepwise")
    torch.cuda.synchronize()
    gu.assert_same_bits(inputs.to_host_storage(outs[N - 1]), want[N - 1], dtype, f"{dtype} rs+ag")


def test_c5_128_nodes_full_compare(orc):
    w = inputs.WORKLOADS["c5"]
    _say("c5: generating 128 x 16.7M fp32")
    ins = inputs.workload_buffers(w, device=gu.DEV)
    host = [inputs.to_host_storage(t) for t in ins]
    _say("c5: fused")
    outs = _run(w, "fused", ins)
    assert _all_equal(outs)
    gu.check_fused_against_oracle(orc, "f32", inputs.to_host_storage(outs[0]), host, "c5 fused")
    _say("c5: fused reduce-scatter, then the direct allgather (segments of 21 KB to 210 KB)")
    parts = [torch.full_like(t, float("nan")) for t in ins]
    nz.nz_reduce_scatter_sim(ins, w.n_elems, w.ratios, w.dtype, "fused", parts)
    nz.nz_allgather_sim(parts, w.n_elems, w.ratios, w.dtype, "fused")
    torch.cuda.synchronize()
    assert all(torch.equal(p, outs[0]) for p in parts)
    del parts
    _say("c5: ring-stepwise")
    outs = _run(w, "ring-stepwise", ins)
    assert _all_equal(outs)
    got = inputs.to_host_storage(outs[0])
    del outs
    _say("c5: oracle ring (254 steps on the host)")
    seg = orc.segment_map(orc.rail_partition(w.n_elems, w.ratios, 4), w.n_nodes)
    want, sent = orc.ring_allreduce(orc.F32, host, seg)
    assert int(sent.sum()) == 2 * (w.n_nodes - 1) * w.payload_bytes
    gu.assert_same_bits(got, want[0], "f32", "c5 ring")
    assert all(np.array_equal(want[0], x) for x in want[1:8])
    gu.check_fused_against_oracle(orc, "f32", got, host, "c5 ring vs sum")


@pytest.mark.parametrize("name", ["c2", "c3", "c5"])
def test_fused_with_buffers_placed_as_the_benchmark_places_them(orc, name):
    """With the benchmark's default placement (inputs in one region, outputs dealt out over all
    three) the 8-node shapes run as one launch of the whole-message kernel, the 128-node one as
    the pipeline: every sum against the oracle at full size, all outputs the same bits."""
    w = inputs.WORKLOADS[name]
    arena = placement.try_arena(gu.DEV)
    if arena is None:
        pytest.skip("not enough free HBM for a three-region arena")
    _say(f"{name}: generating into placed buffers")
    tdt = inputs.TORCH_DTYPE[w.dtype]
    ins = [arena.alloc(w.n_elems, tdt, 0) for _ in range(w.n_nodes)]
    for i, t in enumerate(ins):
        t.copy_(inputs.node_buffer(w.dtype, w.n_elems, w.seed, i, device=gu.DEV, std=w.std,
                                   outlier_frac=w.outlier_frac, outlier_scale=w.outlier_scale))
    outs = arena.alloc_striped(w.n_nodes, w.n_elems, tdt)
    for t in outs:
        t.zero_()
    e = inputs.ELEM_BYTES[w.dtype]
    span = max(t.data_ptr() for t in outs) + w.n_elems * e - min(t.data_ptr() for t in outs)
    launches = nz.nz_allreduce_launches(w.n_nodes, w.n_elems, w.ratios, w.dtype, "fused", w.n_nodes, span)
    assert (launches == 1) == (w.n_nodes <= 16)
    nz.nz_allreduce_sim(ins, w.n_elems, w.ratios, w.dtype, "fused", outs)
    torch.cuda.synchronize()
    assert _all_equal(outs)
    host = [inputs.to_host_storage(t) for t in ins]
    gu.check_fused_against_oracle(orc, w.dtype, inputs.to_host_storage(outs[w.n_nodes - 1]), host, name + " placed")
