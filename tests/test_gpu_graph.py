"""The library's calls can be captured in a HIP graph as they are (no allocation, no device
workspace, no host-to-device copy): every replay must give the eager result, with the
program's own eager work and synchronisations between replays."""
import numpy as np
import pytest
import torch

from paper_2405_17870_amd import inputs
from paper_2405_17870_amd import nezha_sim as nz

import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_graph_replays_match_eager(orc, dtype):
    N, n, ratios, e = 8, 300_007, (100, 100, 40), inputs.ELEM_BYTES[dtype]
    seg = nz.nz_segment_map(nz.nz_rail_partition(n, e, ratios), N)
    ids = [(3 - s) % N for s in range(N)]
    L = sum(int(seg[2, j + 1] - seg[2, j]) for j in ids)
    ins = [inputs.node_buffer(dtype, n, 61, i, device=gu.DEV, std=1e-2) for i in range(N)]
    fused = [torch.zeros_like(t) for t in ins]
    ring = [torch.zeros_like(t) for t in ins]
    send = [torch.zeros(L, dtype=ins[0].dtype, device=gu.DEV) for _ in range(N)]
    back = [torch.zeros_like(t) for t in ins]

    def work():
        nz.nz_allreduce_sim(ins, n, ratios, dtype, "fused", fused)
        nz.nz_allreduce_sim(ins, n, ratios, dtype, "ring-stepwise", ring)
        nz.nz_pack(fused, seg, 2, ids, e, send, L * e)
        nz.nz_unpack(send, seg, 2, ids, e, back)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in fused + ring + send + back]

    work()
    eager = snapshot()
    gu.check_fused_against_oracle(orc, dtype, inputs.to_host_storage(fused[0]),
                                  [inputs.to_host_storage(t) for t in ins], "eager fused")
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            work()
    for replay in range(4):
        for t in fused + ring + send:                   # eager work between replays
            t.fill_(float(replay + 1))
        for t in back:                                  # unpack writes rail 2 only: keep the rest as it was
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for a, b in zip(eager, got):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), replay
        # new inputs are picked up by a replay (the graph holds pointers, not data)
        if replay == 1:
            for t in ins:
                t.mul_(2)
            for t in back:
                t.zero_()
            work()
            eager = snapshot()


def test_graph_replays_of_the_multi_launch_forms(orc):
    """The staged fused allreduce (three launches here), Ring_Chunked (a pipeline of launches) and
    the two halves, captured together: replays equal the eager results."""
    N, n, ratios, dtype = 8, 8 * (1 << 20) + 77, (100, 40), "f32"
    assert nz.nz_allreduce_launches(N, n, ratios, dtype, "fused", N) == 3
    ins = [inputs.node_buffer(dtype, n, 62, i, device=gu.DEV, std=1e-2) for i in range(N)]
    fused = [torch.zeros_like(t) for t in ins]
    chunked = [torch.zeros_like(t) for t in ins]
    halves = [torch.zeros_like(t) for t in ins]

    def work():
        nz.nz_allreduce_sim(ins, n, ratios, dtype, "fused", fused)
        nz.nz_allreduce_sim_chunked(ins, n, ratios, dtype, 1 << 18, chunked)
        nz.nz_reduce_scatter_sim(ins, n, ratios, dtype, "fused", halves)
        nz.nz_allgather_sim(halves, n, ratios, dtype, "fused")

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in fused + chunked + halves]

    work()
    eager = snapshot()
    host = [inputs.to_host_storage(t) for t in ins]
    gu.check_fused_against_oracle(orc, dtype, inputs.to_host_storage(fused[0]), host, "eager staged")
    assert all(torch.equal(h, fused[0]) for h in halves)
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            work()
    for replay in range(3):
        for t in fused + chunked + halves:              # eager work between replays
            t.fill_(float(replay + 1))
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for a, b in zip(eager, got):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), replay
