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
