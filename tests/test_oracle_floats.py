"""Pins for the oracle's bfloat16 / binary16 conversions (CPU only).

Pinned against the formats' definitions (exhaustive round trips, exact ties)
and against independent library conversions (torch for bfloat16, NumPy for
binary16).
"""
import numpy as np
import torch


def _bits_to_f32(u):
    return np.asarray(u, dtype=np.uint32).view(np.float32)


def test_bf16_roundtrip_all_patterns(orc):
    for h in range(1 << 16):
        f = np.float32(orc.bf16_to_f32(h))
        bits = int(np.array(f, dtype=np.float32).view(np.uint32))
        is_nan = (h & 0x7F80) == 0x7F80 and (h & 0x007F) != 0
        if not is_nan:
            assert bits == h << 16                       # widening appends 16 zero bits
            assert orc.f32_to_bf16(float(f)) == h        # and rounding it back is exact


def test_bf16_rounding_matches_torch_and_ties(orc):
    rng = np.random.default_rng(5)
    u = rng.integers(0, 2**32, size=200_000, dtype=np.uint64).astype(np.uint32)
    # exact ties (low half == 0x8000) on even and odd kept parts, near-ties, carries
    special = np.array([0x3F808000, 0x3F818000, 0x3F808001, 0x3F807FFF, 0x3FFF8000, 0x7F7F8000,
                        0x7F7FFFFF, 0x00008000, 0x00018000, 0x80008000, 0x807F8000, 0x00000001,
                        0x7F800000, 0xFF800000, 0x00000000, 0x80000000], dtype=np.uint32)
    u = np.concatenate([u, special, (u & 0xFFFF0000) | 0x8000])
    f = _bits_to_f32(u)
    finite_or_inf = ~np.isnan(f)
    with np.errstate(invalid="ignore"):                          # signalling NaNs among the patterns
        got = orc.round_to_storage(orc.BF16, f.astype(np.float64))   # f32 -> f64 -> f32 is exact
    want = torch.from_numpy(f.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (got[finite_or_inf] == want[finite_or_inf]).all()
    # NaN in, NaN out
    nan_out = got[~finite_or_inf]
    assert ((nan_out & 0x7F80) == 0x7F80).all() and ((nan_out & 0x7F) != 0).all()
    # ties go to the even neighbour, by hand
    assert orc.f32_to_bf16(float(_bits_to_f32(0x3F808000))) == 0x3F80
    assert orc.f32_to_bf16(float(_bits_to_f32(0x3F818000))) == 0x3F82
    assert orc.f32_to_bf16(float(_bits_to_f32(0x7F7F8000))) == 0x7F80   # overflows to +Inf


def test_f16_matches_numpy_exhaustively(orc):
    h = np.arange(1 << 16, dtype=np.uint16)
    want = h.view(np.float16).astype(np.float32)
    for i in range(0, 1 << 16, 1):
        got = np.float32(orc.f16_to_f32(i))
        if np.isnan(want[i]):
            assert np.isnan(got)
        else:
            assert got.tobytes() == want[i].tobytes()
            assert orc.f32_to_f16(float(got)) == i


def test_f16_rounding_matches_numpy(orc):
    rng = np.random.default_rng(6)
    u = rng.integers(0, 2**32, size=200_000, dtype=np.uint64).astype(np.uint32)
    # concentrate half of them in binary16's range, add ties at 13 dropped bits
    mid = (rng.integers(0x33000000, 0x47900000, size=200_000, dtype=np.uint64).astype(np.uint32)
           | (rng.integers(0, 2, size=200_000, dtype=np.uint64).astype(np.uint32) << 31))
    ties = (mid & 0xFFFFE000) | 0x1000
    u = np.concatenate([u, mid, ties, np.array([0x477FE000, 0x477FF000, 0x33000000, 0x33000001,
                                                0x387FC000, 0x387FE000, 0x38800000], np.uint32)])
    f = _bits_to_f32(u)
    ok = ~np.isnan(f)
    with np.errstate(over="ignore", invalid="ignore"):
        got = orc.round_to_storage(orc.F16, f.astype(np.float64))
        want = f.astype(np.float16).view(np.uint16)
    assert (got[ok] == want[ok]).all()
