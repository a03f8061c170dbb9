"""The fused allreduce of large messages: the staged form (a pipeline of launches for jobs with
seven or more distinct outputs that together take 128 MiB or more) at the smallest sizes that
select it, and the single-launch form at those sizes for fewer nodes, where a thread works on
several vectors at once: ragged ends, every element type, node counts of all three kernel
classes, zero-weight rails, in place, repeated and cross-aliased outputs, a failed rail in the
middle (two separate spans of rails).

Each result is compared with the CPU oracle, and bitwise with the same call made with ONE shared
output buffer, which the library runs as a single launch: all forms promise the same bits."""
import numpy as np
import pytest
import torch

from paper_2405_17870_amd import inputs
from paper_2405_17870_amd import nezha_sim as nz

import gpu_util as gu

pytestmark = pytest.mark.gpu

MIB = 1 << 20


def _elems_for(N, e, extra):
    """Smallest element count whose N outputs take 128 MiB, plus a ragged remainder."""
    return -(-128 * MIB // (N * e)) + extra


CASES = [
    # (N, dtype, ratios, ragged extra elements); up to 6 nodes: one launch, 4 or 2 vectors per thread
    (2, "f32", (100, 40), 3), (3, "bf16", (3, 1, 2), 5), (4, "f16", (1,), 9), (2, "bf16", (0, 3, 1), 1),
    (4, "i32", (100, 40), 2), (6, "f32", (100, 100, 40), 3),
    (7, "f32", (100, 40), 3), (8, "bf16", (3, 1, 2), 5), (8, "f16", (100, 100, 40), 1),
    (9, "i32", (7, 0, 3), 2), (32, "bf16", (100, 25), 7), (33, "f32", (1,), 1),
    (128, "f32", (100, 100, 40, 10), 3), (17, "bf16", (0, 5, 0, 2), 6),
]


@pytest.mark.parametrize("N,dtype,ratios,extra", CASES)
def test_large_fused_matches_oracle_and_single_output_launch(orc, N, dtype, ratios, extra):
    e = inputs.ELEM_BYTES[dtype]
    n = _elems_for(N, e, extra)
    staged = nz.nz_allreduce_launches(N, n, ratios, dtype, "fused", N) > 1
    assert staged == (N >= 7)                                                  # the pipeline runs from 7 outputs on
    assert nz.nz_allreduce_launches(N, n, ratios, dtype, "fused", 1) == 1
    print(f"large fused N={N} {dtype} ratios={ratios} n={n} staged={staged}", flush=True)
    ins = [inputs.node_buffer(dtype, n, 500 + N, i, device=gu.DEV, std=1e-2) for i in range(N)]
    if dtype != "i32":                       # special values at the ragged end and at a piece boundary
        for pos in (n - 1, n - 2, 24 * MIB // e, 24 * MIB // e - 1):
            if 0 <= pos < n:
                ins[0][pos] = float("inf")
                ins[N - 1][pos] = float("-inf") if pos % 2 else 1.0
    host = [inputs.to_host_storage(t) for t in ins]
    outs = [torch.full_like(t, 7) for t in ins]
    nz.nz_allreduce_sim(ins, n, ratios, dtype, "fused", outs)
    shared = torch.full_like(ins[0], 7)
    nz.nz_allreduce_sim(ins, n, ratios, dtype, "fused", [shared] * N)
    torch.cuda.synchronize()
    got = inputs.to_host_storage(outs[0])
    gu.check_fused_against_oracle(orc, dtype, got, host, f"staged N={N}")
    gu.assert_same_bits(got, inputs.to_host_storage(shared), dtype, "staged vs single launch")
    for o in outs[1:]:
        assert torch.equal(o.view(torch.uint8), outs[0].view(torch.uint8))
    for t, h in zip(ins, host):
        assert np.array_equal(inputs.to_host_storage(t), h)                   # inputs untouched


def test_staged_in_place_repeated_and_cross_aliased_outputs(orc):
    N, dtype, ratios = 8, "f32", (100, 40)
    n = _elems_for(7, 4, 5)                  # 7 distinct outputs of 18.3 MiB still select the pipeline
    make = lambda: [inputs.node_buffer(dtype, n, 77, i, device=gu.DEV, std=1.0) for i in range(N)]
    ins = make()
    host = [inputs.to_host_storage(t) for t in ins]
    ref = torch.empty_like(ins[0])
    nz.nz_allreduce_sim(ins, n, ratios, dtype, "fused", [ref] * N)           # single launch
    # in place
    work = make()
    assert nz.nz_allreduce_launches(N, n, ratios, dtype, "fused", N) > 1
    nz.nz_allreduce_sim(work, n, ratios, dtype, "fused", work)
    torch.cuda.synchronize()
    gu.check_fused_against_oracle(orc, dtype, inputs.to_host_storage(work[3]), host, "in place")
    assert all(torch.equal(w, ref) for w in work)
    # seven distinct outputs, one of them named twice (the pipeline), then four, each named twice
    # (one launch)
    for k in (7, 4):
        some = [torch.empty_like(ref) for _ in range(k)]
        assert (nz.nz_allreduce_launches(N, n, ratios, dtype, "fused", k) > 1) == (k == 7)
        nz.nz_allreduce_sim(ins, n, ratios, dtype, "fused", [some[i % k] for i in range(N)])
        torch.cuda.synchronize()
        assert all(torch.equal(t, ref) for t in some)
    # an output that is another node's input, whole: every input of an element is read before
    # any output of it is written
    work = make()
    fresh = [torch.empty_like(ref) for _ in range(N - 2)]
    crossed = [work[5], work[2]] + fresh                                      # out[0] = in[5], out[1] = in[2]
    nz.nz_allreduce_sim(work, n, ratios, dtype, "fused", crossed)
    torch.cuda.synchronize()
    assert all(torch.equal(t, ref) for t in crossed)


@pytest.mark.parametrize("failed", [0, 1, 2])
def test_staged_failover_runs_the_surviving_spans_then_the_failed_rail(orc, failed):
    """Three rails, one fails: first or last (one span survives) or the middle one (two spans);
    the failed rail's slice follows as a second pass.  Bitwise the result without a failure."""
    N, dtype, ratios = 16, "bf16", (5, 3, 4)
    n = _elems_for(N, 2, 11) * 3             # every rail alone is big enough for the pipeline
    ins = [inputs.node_buffer(dtype, n, 31, i, device=gu.DEV, std=1e-2) for i in range(N)]
    ref = [torch.empty_like(t) for t in ins]
    nz.nz_allreduce_sim(ins, n, ratios, dtype, "fused", ref)
    outs = [torch.full_like(t, 3) for t in ins]
    took = nz.nz_allreduce_sim_failover(ins, n, ratios, dtype, "fused", outs, failed)
    torch.cuda.synchronize()
    b = orc.rail_partition(n, ratios, 2)
    alive = [k != failed for k in range(3)]
    assert took == orc.failover_target(b, alive)
    for o, r in zip(outs, ref):
        assert torch.equal(o.view(torch.uint8), r.view(torch.uint8))
    host = [inputs.to_host_storage(t[-300_000:]) for t in ins]
    gu.check_fused_against_oracle(orc, dtype, inputs.to_host_storage(outs[0][-300_000:]), host, "failover tail")


MI = 1 << 20
# (N, dtype, distinct outputs, elements): sizes the library's rule sends to the several-vectors
# form of the whole-message kernel -- at most 4 nodes, all bytes of the call within 128 MiB, and
# at least 2048 workgroups of 2 (16 MiB per node) or 4 (2 nodes, 32 MiB per node) vectors per thread
FEW_NODES_CACHED = [
    (2, "f32", 2, 4 * MI + 5),        # 16 MiB per node, two vectors per thread
    (2, "bf16", 1, 17 * MI + 3),      # 34 MiB per node, one shared output: four vectors per thread
    (2, "i32", 2, 8 * MI),            # exactly 32 MiB: four vectors per thread, no ragged end
    (3, "i32", 3, 4 * MI + MI // 2 + 7),   # 18 MiB per node, two vectors per thread
    (4, "f16", 1, 9 * MI + 1),        # 18 MiB per node, one shared output: two vectors per thread
]


@pytest.mark.parametrize("N,dtype,K,n", FEW_NODES_CACHED)
def test_cache_resident_jobs_of_few_nodes(orc, N, dtype, K, n):
    """Every sum against the oracle, inputs untouched, all outputs the same bits."""
    ratios = (100, 40)
    e = inputs.ELEM_BYTES[dtype]
    assert (N + K) * n * e <= 128 * MI and n * e >= 16 * MI
    print(f"few nodes, cache resident: N={N} {dtype} K={K} n={n}", flush=True)
    ins = [inputs.node_buffer(dtype, n, 1300 + N, i, device=gu.DEV, std=1e-2) for i in range(N)]
    if dtype not in ("i32",):
        ins[0][n - 1] = float("inf")
        ins[N - 1][n - 2] = float("nan")
    host = [inputs.to_host_storage(t) for t in ins]
    distinct = [torch.full_like(ins[0], 7) for _ in range(K)]
    nz.nz_allreduce_sim(ins, n, ratios, dtype, "fused", [distinct[i % K] for i in range(N)])
    torch.cuda.synchronize()
    got = inputs.to_host_storage(distinct[0])
    gu.check_fused_against_oracle(orc, dtype, got, host, f"few nodes N={N}")
    for o in distinct[1:]:
        assert torch.equal(o.view(torch.uint8), distinct[0].view(torch.uint8))
    for t, h in zip(ins, host):
        assert inputs.to_host_storage(t).tobytes() == h.tobytes()
