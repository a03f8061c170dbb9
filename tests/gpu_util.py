"""Helpers shared by the GPU parity tests: guarded device buffers, calls through the
C-ABI binding, and the comparison rules.

Comparison rules (what "equal to the oracle" means per type):
  int32, index maps, copies, ring-mode results ... bit-exact;
  fp32 fused ... |gpu - s| <= 1e-6 * sum|x_i| per element, s the oracle's fp64 sum;
  bf16 / fp16 fused ... at most 1 ulp (of the storage type) from the oracle's
      storage(fp32(s)); where the sum cancels so far that one ulp of the result is smaller
      than the fp32 accumulation error itself, the fp32 bound above (plus half an ulp for
      the final rounding) applies instead -- such elements are counted and reported.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from paper_2405_17870_amd import inputs
from paper_2405_17870_amd import nezha_sim as nz

DEV = "cuda:0"
GUARD_BYTES = 512
ORC_CODE = {"f32": 0, "bf16": 1, "f16": 2, "i32": 3}
FP32_REL = 1e-6


class Guarded:
    """A device buffer with canary bands in front and behind, base aligned to 256 bytes."""

    def __init__(self, n_elems: int, dtype: str, fill: Optional[torch.Tensor] = None,
                 canary: int = 0x5A):
        e = inputs.ELEM_BYTES[dtype]
        self.n, self.dtype, self.e, self.canary = n_elems, dtype, e, canary
        body = n_elems * e
        self.raw = torch.full((GUARD_BYTES + body + GUARD_BYTES,), canary, dtype=torch.uint8,
                              device=DEV)
        assert self.raw.data_ptr() % 256 == 0
        self.t = self.raw[GUARD_BYTES:GUARD_BYTES + body].view(inputs.TORCH_DTYPE[dtype])
        assert self.t.data_ptr() % 256 == 0
        if fill is not None:
            self.t.copy_(fill)

    def guards_intact(self) -> bool:
        body = self.n * self.e
        return bool((self.raw[:GUARD_BYTES] == self.canary).all().item()
                    and (self.raw[GUARD_BYTES + body:] == self.canary).all().item())

    def host(self) -> np.ndarray:
        return inputs.to_host_storage(self.t)


def device_inputs(host_tensors: Sequence[torch.Tensor], dtype: str) -> List[Guarded]:
    return [Guarded(t.numel(), dtype, fill=t.to(DEV)) for t in host_tensors]


def fresh_outputs(n_nodes: int, n_elems: int, dtype: str) -> List[Guarded]:
    return [Guarded(n_elems, dtype, canary=0xC3) for _ in range(n_nodes)]


def allreduce(ins: Sequence[Guarded], outs: Sequence[Guarded], ratios, mode: str) -> None:
    n = ins[0].n
    nz.nz_allreduce_sim([g.t for g in ins], n, ratios, ins[0].dtype, mode, [g.t for g in outs])
    torch.cuda.synchronize()


def monotone(bits: np.ndarray) -> np.ndarray:
    """Map 16-bit float patterns to integers ordered like the values they encode."""
    b = bits.astype(np.int32)
    mag = b & 0x7FFF
    return np.where(b & 0x8000, -mag, mag)


def half_to_f64(bits: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return bits.view(np.float16).astype(np.float64)


def is_nan16(bits: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return ((bits & 0x7F80) == 0x7F80) & ((bits & 0x007F) != 0)
    return ((bits & 0x7C00) == 0x7C00) & ((bits & 0x03FF) != 0)


def check_fused_against_oracle(orc, dtype: str, got: np.ndarray, host_ins: Sequence[np.ndarray],
                               label: str = "") -> int:
    """Apply the comparison rule for `dtype`; returns how many elements needed the
    cancellation clause (always 0 for int32 and fp32)."""
    if dtype == "i32":
        want = orc.sum_i32(host_ins)
        assert np.array_equal(got, want), f"{label}: int32 sum differs"
        return 0
    s, a = orc.sum_float(ORC_CODE[dtype], host_ins)
    if dtype == "f32":
        g = got.astype(np.float64)
        nan = np.isnan(s)
        assert np.array_equal(np.isnan(g), nan), f"{label}: NaN placement differs"
        inf = np.isinf(s)
        assert np.array_equal(g[inf], s[inf]), f"{label}: infinities differ"
        ok = ~(nan | inf)
        err = np.abs(g[ok] - s[ok])
        bound = FP32_REL * a[ok]
        worst = np.max(err - bound) if err.size else 0.0
        assert (err <= bound).all(), f"{label}: fp32 error exceeds 1e-6*sum|x| by {worst}"
        return 0
    want = orc.round_to_storage(ORC_CODE[dtype], s)
    # Elements whose bits agree need no further look; the rest (typically well under 1 %) go
    # through the ulp rule.
    diff = np.flatnonzero(got != want)
    if diff.size == 0:
        return 0
    g_d, w_d, s_d, a_d = got[diff], want[diff], s[diff], a[diff]
    nan_w, nan_g = is_nan16(w_d, dtype), is_nan16(g_d, dtype)
    assert np.array_equal(nan_w, nan_g), f"{label}: NaN placement differs"
    ok = ~nan_w
    dist = np.abs(monotone(g_d[ok]) - monotone(w_d[ok]))
    far = dist > 1
    if far.any():
        g = half_to_f64(g_d[ok][far], dtype)
        eps = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -11      # half an ulp, relative
        bound = FP32_REL * a_d[ok][far] + eps * np.abs(g)
        assert (np.abs(g - s_d[ok][far]) <= bound).all(), \
            f"{label}: {dtype} result more than 1 ulp away and outside the fp32 bound"
    return int(far.sum())


def assert_same_bits(a: np.ndarray, b: np.ndarray, dtype: str, label: str = "") -> None:
    """Bit equality, except that any NaN matches any NaN (payloads are not compared)."""
    if dtype in ("bf16", "f16"):
        na, nb = is_nan16(a, dtype), is_nan16(b, dtype)
        assert np.array_equal(na, nb), f"{label}: NaN placement differs"
        assert np.array_equal(a[~na], b[~nb]), f"{label}: bits differ"
    elif dtype == "f32":
        na, nb = np.isnan(a), np.isnan(b)
        assert np.array_equal(na, nb), f"{label}: NaN placement differs"
        assert np.array_equal(a[~na].view(np.uint32), b[~nb].view(np.uint32)), f"{label}: bits differ"
    else:
        assert np.array_equal(a, b), f"{label}: values differ"
