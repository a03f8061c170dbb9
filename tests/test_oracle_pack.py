"""Pins for the oracle's pack / unpack (CPU only).

A rail's slice is staged from the user buffer into a contiguous per-rail buffer
and the result returned to it (Nezha Sec. 3.2).  Pinned by NumPy slicing and
concatenation, the round trip, and canaries around everything not addressed.
"""
import random

import numpy as np
import pytest


@pytest.mark.parametrize("e", [2, 4])
def test_pack_is_concatenation_and_unpack_its_inverse(orc, e):
    rnd = random.Random(e)
    for _ in range(40):
        N = rnd.choice([1, 2, 3, 8, 31])
        R = rnd.randint(1, 4)
        n = rnd.randint(0, 3000)
        seg = orc.segment_map(orc.rail_partition(n, [rnd.randint(0, 9) + (k == 0) for k in range(R)],
                                                 e, rnd.choice([e, 16, 256])), N)
        rail = rnd.randrange(R)
        ids = [rnd.randrange(N) for _ in range(rnd.randint(0, N))]
        if rnd.random() < 0.3:
            ids = list(range(N))                                   # whole rail
        rng = np.random.default_rng(n)
        src = rng.integers(0, 256, size=n * e, dtype=np.uint8)
        packed, nbytes = orc.pack(src, seg, rail, ids, e)
        want = np.concatenate([src[int(seg[rail, j]) * e:int(seg[rail, j + 1]) * e] for j in ids]
                              + [np.zeros(0, np.uint8)])
        assert nbytes == want.size and (packed == want).all()
        if ids == list(range(N)):                                  # whole rail == a plain slice
            assert (packed == src[int(seg[rail, 0]) * e:int(seg[rail, N]) * e]).all()
        # unpack into a canary-filled destination: listed segments restored, nothing else touched
        uniq = list(dict.fromkeys(ids))
        packed_u, _ = orc.pack(src, seg, rail, uniq, e)
        dst = np.full(n * e, 0xA5, dtype=np.uint8)
        orc.unpack(packed_u, seg, rail, uniq, e, dst)
        touched = np.zeros(n * e, dtype=bool)
        for j in uniq:
            touched[int(seg[rail, j]) * e:int(seg[rail, j + 1]) * e] = True
        assert (dst[touched] == src[touched]).all()
        assert (dst[~touched] == 0xA5).all()


def test_pack_respects_capacity_layout(orc):
    # a larger send buffer: bytes past packed_bytes stay as they were
    seg = orc.segment_map(orc.rail_partition(100, [1], 4, 4), 4)
    src = np.arange(100, dtype=np.int32)
    send = np.full(1000, 0xEE, dtype=np.uint8)
    _, nbytes = orc.pack(src, seg, 0, [3, 1], 4, send)
    assert nbytes == 200
    assert (send[:200].view(np.int32) == np.concatenate([src[75:100], src[25:50]])).all()
    assert (send[200:] == 0xEE).all()
