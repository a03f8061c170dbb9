"""Seeded synthetic gradient buffers and the workload table.

This module only *makes inputs*: it holds no partition, segment, reduction or
packing arithmetic.  Both the GPU path's callers and the CPU checker's callers
take their bytes from here, so the two sides always see identical inputs.

The workloads stand in for flat gradient buckets of the sizes a data-parallel
job all-reduces (Nezha, arXiv 2405.17870, Sec. 2.1.1 and Sec. 5.1): only the
node count, element count, element type and value distribution matter to an
allreduce, so normally distributed values of gradient-like magnitude are used.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np
import torch

SEED_BASE = 0x4E5A0000

TORCH_DTYPE = {
    "f32": torch.float32,
    "bf16": torch.bfloat16,
    "f16": torch.float16,
    "i32": torch.int32,
}
ELEM_BYTES = {"f32": 4, "bf16": 2, "f16": 2, "i32": 4}


@dataclass(frozen=True)
class Workload:
    """One synthetic allreduce workload."""
    name: str
    n_nodes: int
    n_elems: int
    dtype: str
    ratios: Tuple[int, ...]
    std: float
    outlier_frac: float = 0.0
    outlier_scale: float = 100.0
    seed: int = SEED_BASE

    @property
    def payload_bytes(self) -> int:
        return self.n_elems * ELEM_BYTES[self.dtype]


WORKLOADS = {
    "c1": Workload("c1", 8, 1_048_576, "f32", (100, 40), 1e-2, seed=SEED_BASE + 1),
    "c1_i32": Workload("c1_i32", 8, 1_048_576, "i32", (100, 40), 0.0, seed=SEED_BASE + 1),
    "c2": Workload("c2", 8, 25_557_032, "f32", (100, 40), 1e-3, seed=SEED_BASE + 2),
    "c3": Workload("c3", 8, 138_357_544, "bf16", (100, 100, 40), 1e-3, outlier_frac=0.01,
                   seed=SEED_BASE + 3),
    "c3_f16": Workload("c3_f16", 8, 138_357_544, "f16", (100, 100, 40), 1e-3, outlier_frac=0.01,
                       seed=SEED_BASE + 6),
    "c4": Workload("c4", 32, 335_000_000, "bf16", (100, 25), 1e-3, seed=SEED_BASE + 4),
    "c5": Workload("c5", 128, 16_777_216, "f32", (100, 100, 40, 10), 1e-2, seed=SEED_BASE + 5),
}


def _generator(seed: int, node: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) << 12) + int(node))
    return g


def node_buffer(dtype: str, n_elems: int, seed: int, node: int, device="cpu", std: float = 1e-2,
                outlier_frac: float = 0.0, outlier_scale: float = 100.0,
                int_range: int = 1000) -> torch.Tensor:
    """One node's gradient buffer.

    Floating types: normal, mean 0, standard deviation ``std``; a fraction
    ``outlier_frac`` of entries (independent Bernoulli draws) is multiplied by
    ``outlier_scale``; the values are rounded to the storage type once.
    ``i32``: integers uniform in [-int_range, int_range].
    """
    g = _generator(seed, node, device)
    if dtype == "i32":
        return torch.randint(-int_range, int_range + 1, (n_elems,), generator=g, device=device,
                             dtype=torch.int32)
    x = torch.randn(n_elems, generator=g, device=device, dtype=torch.float32)
    x.mul_(std)
    if outlier_frac > 0.0:
        mask = torch.rand(n_elems, generator=g, device=device) < outlier_frac
        x = torch.where(mask, x * outlier_scale, x)
        del mask
    return x.to(TORCH_DTYPE[dtype])


def workload_buffers(w: Workload, device="cpu", n_elems: Optional[int] = None,
                     n_nodes: Optional[int] = None) -> List[torch.Tensor]:
    """All nodes' buffers of a workload (optionally at a reduced size)."""
    n = w.n_elems if n_elems is None else n_elems
    N = w.n_nodes if n_nodes is None else n_nodes
    return [node_buffer(w.dtype, n, w.seed, i, device=device, std=w.std,
                        outlier_frac=w.outlier_frac, outlier_scale=w.outlier_scale)
            for i in range(N)]


def fingerprint_buffers(dtype: str, n_nodes: int, n_elems: int, device="cpu",
                        active: Optional[range] = None) -> List[torch.Tensor]:
    """Node i holds the constant 2**(i - first active node); inactive nodes hold 0.

    With at most 24 (fp32), 8 (bf16), 11 (fp16) or 31 (int32) active nodes the
    sum of any subset is exact, so every output bit names one (node, element).
    """
    act = range(n_nodes) if active is None else active
    out = []
    for i in range(n_nodes):
        v = float(2 ** (i - act.start)) if i in act else 0.0
        if dtype == "i32":
            out.append(torch.full((n_elems,), int(v), dtype=torch.int32, device=device))
        else:
            out.append(torch.full((n_elems,), v, dtype=TORCH_DTYPE[dtype], device=device))
    return out


def index_buffers(n_nodes: int, n_elems: int, device="cpu") -> List[torch.Tensor]:
    """int32 buffers with in[i][x] = (x mod 2**16) * (i + 1)."""
    x = torch.arange(n_elems, dtype=torch.int64, device=device) % 65536
    return [(x * (i + 1)).to(torch.int32) for i in range(n_nodes)]


def to_host_storage(t: torch.Tensor) -> np.ndarray:
    """Host copy of a buffer as a NumPy array; 16-bit floats travel as uint16."""
    t = t.detach().cpu().contiguous()
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def from_host_storage(a: np.ndarray, dtype: str, device="cpu") -> torch.Tensor:
    """Inverse of :func:`to_host_storage`."""
    if dtype in ("bf16", "f16"):
        t = torch.from_numpy(np.ascontiguousarray(a).view(np.int16).copy()).view(TORCH_DTYPE[dtype])
    else:
        t = torch.from_numpy(np.ascontiguousarray(a).copy())
    return t.to(device)
