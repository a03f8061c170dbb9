"""The harness's HBM arena hands out aligned, disjoint tensors inside the requested regions."""
import pytest
import torch

from paper_2405_17870_amd import nezha_sim as nz
from paper_2405_17870_amd import placement

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
