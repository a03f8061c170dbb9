"""GPU parity of nz_allreduce_sim against the CPU oracle, through the C-ABI (small shapes that
still span several tiles, every alignment class and ragged tails)."""
import random

import numpy as np
import pytest
import torch

from paper_2405_17870_amd import inputs
from paper_2405_17870_amd import nezha_sim as nz

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _host_inputs(dtype, N, n, seed, std=1e-2, outlier=0.0):
    return [inputs.node_buffer(dtype, n, seed, i, std=std, outlier_frac=outlier) for i in range(N)]


SHAPES = [
    # (N, ratios, n)
    (1, (1,), 1000), (2, (1, 1), 1), (2, (3, 1), 63), (3, (3, 1), 200), (3, (1,), 64), (2, (1, 2), 65),
    (8, (100, 40), 70_001), (8, (100, 100, 40), 12_345), (5, (7, 0, 3), 4_097),
    (32, (100, 25), 100_003), (128, (100, 100, 40, 10), 33_333), (128, (1, 1), 100),
    (7, (1, 1, 1, 1, 1, 1, 1, 1), 9_999), (9, (5,), 300_000), (17, (2, 5), 262_144 + 17),
    # segments of exactly 1, 63, 64, 65 elements; fewer elements than nodes (empty segments)
    (4, (1,), 4), (4, (1,), 4 * 63), (4, (1,), 4 * 64), (4, (1,), 4 * 65), (8, (1,), 5), (8, (3, 1), 130),
    # segment length 1001 = 1 mod 8: the 8 segment starts fall in every alignment class of a
    # 16-byte vector (0, 2, .. 14 bytes for 2-byte elements; 0, 4, 8, 12 for 4-byte elements)
    (8, (1,), 8 * 1001),
]


def test_shapes_cover_every_alignment_class(orc):
    for e in (2, 4):
        seg = orc.segment_map(orc.rail_partition(8 * 1001, (1,), e), 8)
        assert {int(x) * e % 16 for x in seg[0, :8]} == set(range(0, 16, e))


@pytest.mark.parametrize("dtype", ["f32", "i32", "bf16", "f16"])
@pytest.mark.parametrize("N,ratios,n", SHAPES)
def test_fused_matches_oracle(orc, dtype, N, ratios, n):
    _say(f"fused dtype={dtype} N={N} ratios={ratios} n={n}")
    host = _host_inputs(dtype, N, n, seed=11 + N)
    ins = gu.device_inputs(host, dtype)
    outs = gu.fresh_outputs(N, n, dtype)
    gu.allreduce(ins, outs, ratios, "fused")
    host_np = [inputs.to_host_storage(t) for t in host]
    got0 = outs[0].host()
    gu.check_fused_against_oracle(orc, dtype, got0, host_np, "fused")
    for g in outs:
        assert np.array_equal(g.host(), got0)            # every node holds identical bits
        assert g.guards_intact()
    for i, g in enumerate(ins):
        assert g.guards_intact() and np.array_equal(g.host(), host_np[i])   # inputs untouched


@pytest.mark.parametrize("dtype", ["f32", "i32", "bf16", "f16"])
@pytest.mark.parametrize("N,ratios,n", SHAPES)
def test_ring_stepwise_matches_oracle_ring_bit_for_bit(orc, dtype, N, ratios, n):
    _say(f"ring dtype={dtype} N={N} ratios={ratios} n={n}")
    host = _host_inputs(dtype, N, n, seed=23 + N, std=1.0)
    ins = gu.device_inputs(host, dtype)
    outs = gu.fresh_outputs(N, n, dtype)
    gu.allreduce(ins, outs, ratios, "ring-stepwise")
    host_np = [inputs.to_host_storage(t) for t in host]
    seg = orc.segment_map(orc.rail_partition(n, ratios, inputs.ELEM_BYTES[dtype]), N)
    want, _ = orc.ring_allreduce(gu.ORC_CODE[dtype], host_np, seg)
    for i, g in enumerate(outs):
        gu.assert_same_bits(g.host(), want[i], dtype, f"ring node {i}")
        assert g.guards_intact()
    for i, g in enumerate(ins):
        assert g.guards_intact() and np.array_equal(g.host(), host_np[i])
    # and it is the sum (tolerance for a sequential order: (N-1) roundings)
    if dtype == "i32":
        assert np.array_equal(outs[0].host(), orc.sum_i32(host_np))


@pytest.mark.parametrize("mode", ["fused", "ring-stepwise"])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "i32"])
def test_in_place(orc, mode, dtype):
    N, n, ratios = 6, 50_001, (100, 40)
    _say(f"in-place mode={mode} dtype={dtype}")
    host = _host_inputs(dtype, N, n, seed=5)
    bufs = gu.device_inputs(host, dtype)
    ref_out = gu.fresh_outputs(N, n, dtype)
    gu.allreduce(bufs, ref_out, ratios, mode)
    gu.allreduce(bufs, bufs, ratios, mode)
    for i in range(N):
        assert np.array_equal(bufs[i].host(), ref_out[i].host())
        assert bufs[i].guards_intact()


def test_fused_shared_output_and_repeated_outputs(orc):
    N, n, ratios, dtype = 8, 77_777, (100, 40), "f32"
    host = _host_inputs(dtype, N, n, seed=9)
    ins = gu.device_inputs(host, dtype)
    full = gu.fresh_outputs(N, n, dtype)
    gu.allreduce(ins, full, ratios, "fused")
    shared = gu.Guarded(n, dtype)
    nz.nz_allreduce_sim([g.t for g in ins], n, ratios, dtype, "fused", [shared.t] * N)
    two = gu.fresh_outputs(2, n, dtype)
    nz.nz_allreduce_sim([g.t for g in ins], n, ratios, dtype, "fused",
                        [two[i % 2].t for i in range(N)])
    torch.cuda.synchronize()
    assert np.array_equal(shared.host(), full[0].host()) and shared.guards_intact()
    assert np.array_equal(two[0].host(), full[0].host()) and np.array_equal(two[1].host(), full[0].host())


@pytest.mark.parametrize("dtype", ["f32", "bf16", "i32"])
def test_fused_result_does_not_depend_on_the_rail_split(orc, dtype):
    # rails work on disjoint slices and do not interfere: bitwise the same for any ratios
    N, n = 12, 123_457
    host = _host_inputs(dtype, N, n, seed=3)
    ins = gu.device_inputs(host, dtype)
    ref = None
    for ratios in [(1,), (1, 1), (100, 40), (1, 0, 5), (100, 100, 40, 10), (1, 2, 3, 4, 5, 6, 7, 8), (0, 1)]:
        out = gu.fresh_outputs(N, n, dtype)
        gu.allreduce(ins, out, ratios, "fused")
        ref = out[0].host() if ref is None else ref
        assert np.array_equal(out[0].host(), ref), ratios
        assert np.array_equal(out[N - 1].host(), ref), ratios


@pytest.mark.parametrize("mode", ["fused", "ring-stepwise"])
def test_fingerprint_and_index_inputs(orc, mode):
    # node i holds 2^i: every output bit names one (node, element)
    for dtype, N in (("i32", 31), ("f32", 24), ("bf16", 8), ("f16", 11)):
        n = 40_003
        ins = gu.device_inputs(inputs.fingerprint_buffers(dtype, N, n), dtype)
        outs = gu.fresh_outputs(N, n, dtype)
        gu.allreduce(ins, outs, (100, 100, 40, 10), mode)
        want = (torch.full((n,), 2 ** N - 1, dtype=torch.int32) if dtype == "i32"
                else torch.full((n,), float(2 ** N - 1)).to(inputs.TORCH_DTYPE[dtype]))
        for g in outs:
            assert torch.equal(g.t.cpu(), want)
    # N = 128 in passes of 31 active nodes (int32)
    N, n = 128, 20_011
    for start in range(0, N, 31):
        act = range(start, min(start + 31, N))
        ins = gu.device_inputs(inputs.fingerprint_buffers("i32", N, n, active=act), "i32")
        outs = gu.fresh_outputs(N, n, "i32")
        gu.allreduce(ins, outs, (100, 100, 40, 10), mode)
        for g in (outs[0], outs[77], outs[127]):
            assert (g.t == 2 ** len(act) - 1).all().item()
    # index inputs: closed form (x mod 2^16) * N (N+1) / 2
    N, n = 13, 200_001
    ins = gu.device_inputs(inputs.index_buffers(N, n), "i32")
    outs = gu.fresh_outputs(N, n, "i32")
    gu.allreduce(ins, outs, (100, 40), mode)
    want = (torch.arange(n, dtype=torch.int64) % 65536) * (N * (N + 1) // 2)
    for g in outs:
        assert torch.equal(g.t.cpu().to(torch.int64), want)


@pytest.mark.parametrize("mode", ["fused", "ring-stepwise"])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_two_nodes_is_a_single_ieee_add_and_special_values(orc, mode, dtype):
    n = 4_099
    a = inputs.node_buffer(dtype, n, 1, 0, std=1.0).clone()
    b = inputs.node_buffer(dtype, n, 1, 1, std=1.0).clone()
    inf, nan = float("inf"), float("nan")
    tiny = {"f32": 1e-45, "bf16": 1e-40, "f16": 6e-8}[dtype]          # subnormal in each type
    a[:8] = torch.tensor([inf, inf, nan, -0.0, tiny, 0.0, -inf, tiny]).to(a.dtype)
    b[:8] = torch.tensor([1.0, -inf, 1.0, -0.0, tiny, -0.0, -inf, -tiny]).to(b.dtype)
    ins = gu.device_inputs([a, b], dtype)
    outs = gu.fresh_outputs(2, n, dtype)
    gu.allreduce(ins, outs, (100, 40), mode)
    want = (a.float() + b.float()).to(a.dtype)               # one fp32 add, one rounding
    got = outs[0].host()
    gu.assert_same_bits(got, inputs.to_host_storage(want), dtype, "two-node add")
    s, _ = orc.sum_float(gu.ORC_CODE[dtype], [inputs.to_host_storage(a), inputs.to_host_storage(b)])
    gu.assert_same_bits(got, orc.round_to_storage(gu.ORC_CODE[dtype], s), dtype, "vs oracle")
    gu.assert_same_bits(outs[1].host(), got, dtype, "second node")


def test_bf16_rounding_of_the_kernel_matches_the_oracle_on_ties_and_carries(orc):
    # two fp... the sum of two bf16 values can need up to 16+ bits: build sums that land on
    # exact ties, just above and below them, and on mantissa carries
    rng = np.random.default_rng(12)
    n = 1 << 16
    hi = rng.integers(0x3F80, 0x4780, size=n, dtype=np.uint16)            # 1.0 .. 65536
    lo = (hi - rng.integers(8 << 7, 9 << 7, size=n).astype(np.uint16))    # 2^-8 .. 2^-9 smaller: half-ulp region
    lo[::3] = (hi[::3] & 0x7F80) - (8 << 7)                               # exactly half an ulp of hi: a tie
    sign = rng.integers(0, 2, size=n).astype(np.uint16) << 15
    a = inputs.from_host_storage(hi | sign, "bf16")
    b = inputs.from_host_storage(lo | sign, "bf16")
    for mode in ("fused", "ring-stepwise"):
        ins = gu.device_inputs([a, b], "bf16")
        outs = gu.fresh_outputs(2, n, "bf16")
        gu.allreduce(ins, outs, (1,), mode)
        s, _ = orc.sum_float(orc.BF16, [inputs.to_host_storage(a), inputs.to_host_storage(b)])
        want = orc.round_to_storage(orc.BF16, s)              # two-term sums are exact in fp32
        assert np.array_equal(outs[0].host(), want), mode


def test_fp32_error_bound_holds_for_adversarial_signs_at_128_nodes(orc):
    # all-positive values of mixed magnitude maximise accumulated rounding
    N, n = 128, 30_011
    host = [inputs.node_buffer("f32", n, 99, i, std=1.0).abs() * (10.0 ** (i % 5)) for i in range(N)]
    ins = gu.device_inputs(host, "f32")
    outs = gu.fresh_outputs(N, n, "f32")
    gu.allreduce(ins, outs, (100, 100, 40, 10), "fused")
    gu.check_fused_against_oracle(orc, "f32", outs[0].host(), [inputs.to_host_storage(t) for t in host])


def test_determinism(orc):
    N, n = 32, 250_007
    host = _host_inputs("bf16", N, n, seed=8, std=1e-3, outlier=0.01)
    ins = gu.device_inputs(host, "bf16")
    a, b = gu.fresh_outputs(N, n, "bf16"), gu.fresh_outputs(N, n, "bf16")
    gu.allreduce(ins, a, (100, 25), "fused")
    gu.allreduce(ins, b, (100, 25), "fused")
    assert all(np.array_equal(x.host(), y.host()) for x, y in zip(a, b))


def test_argument_errors_launch_nothing(orc):
    N, n = 4, 1000
    host = _host_inputs("f32", N, n, seed=2)
    ins = gu.device_inputs(host, "f32")
    outs = gu.fresh_outputs(N, n, "f32")
    before = [g.raw.clone() for g in outs]
    p_in, p_out = [g.t for g in ins], [g.t for g in outs]

    def status(*args, **kw):
        with pytest.raises(nz.NezhaSimError) as e:
            nz.nz_allreduce_sim(*args, **kw)
        return e.value.status

    assert status(p_in, n, (0, 0), "f32", "fused", p_out) == 1                   # zero weight sum
    assert status(p_in, n, (1,) * 9, "f32", "fused", p_out) == 3                  # too many rails
    mis = [p_in[0].data_ptr() + 4] + p_in[1:]
    assert status(mis, n - 1, (1,), "f32", "fused", p_out) == 2                   # misaligned base
    assert status(p_in, n, (1,), "f32", "ring-stepwise", [p_out[0]] * N) == 3     # ring needs distinct outputs
    assert status(p_in, n, (1,), "f32", "ring-stepwise", [p_in[1], p_in[0]] + p_out[2:]) == 3
    big = gu.Guarded(2 * n, "f32")
    overl = [big.t.data_ptr(), big.t.data_ptr() + 256] + p_out[2:]                # partial overlap
    assert status(p_in, n, (1,), "f32", "fused", overl) == 3
    assert status([p_in[0]] * 129, n, (1,), "f32", "fused", [p_out[0]] * 129) == 3   # too many nodes
    nz.nz_allreduce_sim(p_in, 0, (1,), "f32", "fused", p_out)                      # empty message: ok
    torch.cuda.synchronize()
    for g, b in zip(outs, before):
        assert torch.equal(g.raw, b)


def test_debug_wait_changes_nothing_but_the_timing(orc, monkeypatch):
    """NZ_DEBUG makes every call wait for its stream; results and statuses stay the same."""
    N, n, ratios, dtype = 5, 40_001, (3, 1), "bf16"
    host = _host_inputs(dtype, N, n, seed=77)
    ins = gu.device_inputs(host, dtype)
    ref, dbg = gu.fresh_outputs(N, n, dtype), gu.fresh_outputs(N, n, dtype)
    for mode in ("fused", "ring-stepwise"):
        nz.nz_allreduce_sim([g.t for g in ins], n, ratios, dtype, mode, [g.t for g in ref])
        torch.cuda.synchronize()
        monkeypatch.setenv("NZ_DEBUG", "1")
        nz.nz_allreduce_sim([g.t for g in ins], n, ratios, dtype, mode, [g.t for g in dbg])
        got = [g.host() for g in dbg]
        with pytest.raises(nz.NezhaSimError) as ex:
            nz.nz_allreduce_sim([g.t for g in ins], n, (0, 0), dtype, mode, [g.t for g in dbg])
        assert ex.value.status == 1
        monkeypatch.setenv("NZ_DEBUG", "0")
        for a, b in zip(got, ref):
            assert np.array_equal(a, b.host())


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_cold_start_ratios_equal_the_single_rail_ring(orc, dtype):
    """All data on one rail (Sec. 4.3, Eq. 4) is written as weights {1, 0, ..}: in ring mode too
    the result is bitwise the single-rail result, wherever the loaded rail sits in the list."""
    N, n = 7, 90_001
    host = _host_inputs(dtype, N, n, seed=13, std=1.0)
    ins = gu.device_inputs(host, dtype)
    single = gu.fresh_outputs(N, n, dtype)
    gu.allreduce(ins, single, (1,), "ring-stepwise")
    for ratios in [(1, 0), (0, 1), (0, 5, 0, 0)]:
        out = gu.fresh_outputs(N, n, dtype)
        gu.allreduce(ins, out, ratios, "ring-stepwise")
        for a, b in zip(out, single):
            assert np.array_equal(a.host(), b.host()), ratios
            assert a.guards_intact()
