"""NumPy-facing wrapper around the plain-C oracle in ``nz_oracle.c``.

TEST INFRASTRUCTURE ONLY: see the header of ``nz_oracle.c``.  The wrapper
does argument marshalling and nothing else; all arithmetic is in the C file.

Citations (Nezha, arXiv 2405.17870): rail slices -- Sec. 3.4, 3.5, 4.2 and
the proportions under Eq. 5; ring schedule -- Sec. 2.1.1, Eq. 1; the sum --
Sec. 4.2 (aggregation phase); staging buffers -- Sec. 3.2.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nz_oracle.c")
_LIB = os.path.join(_HERE, "libnz_oracle.so")

F32, BF16, F16, I32 = 0, 1, 2, 3
ELEM_BYTES = {F32: 4, BF16: 2, F16: 2, I32: 4}
_NP_STORAGE = {F32: np.float32, BF16: np.uint16, F16: np.uint16, I32: np.int32}

__all__ = [
    "F32", "BF16", "F16", "I32", "ELEM_BYTES", "build", "threads", "set_threads",
    "rail_partition", "segment_map", "sum_float", "sum_i32", "round_to_storage",
    "ring_allreduce", "ring_allgather", "ring_allreduce_chunked", "failover_target", "pack", "unpack",
    "t_cold", "t_hot", "balance_iterate", "balance_optimum", "threshold", "net_efficiency", "efficiency_ratio",
    "bf16_to_f32", "f32_to_bf16", "f16_to_f32", "f32_to_f16", "storage_dtype",
]


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, OpenMP for the element loop)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u64, u32, i32 = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int
        vp = ctypes.c_void_p
        lib.orc_rail_partition.argtypes = [u64, u64, vp, u32, vp]
        lib.orc_segment_map.argtypes = [vp, u32, u32, vp]
        lib.orc_sum_float.argtypes = [i32, vp, u32, u64, vp, vp]
        lib.orc_sum_i32.argtypes = [vp, u32, u64, vp]
        lib.orc_round_to_storage.argtypes = [i32, vp, u64, vp]
        lib.orc_ring_allreduce.argtypes = [i32, vp, u32, u64, vp, u32, i32, vp]
        lib.orc_ring_allgather.argtypes = [i32, vp, u32, u64, vp, u32, vp]
        lib.orc_ring_allreduce_chunked.argtypes = [i32, vp, u32, u64, vp, u32, u64, vp, vp]
        lib.orc_failover_target.argtypes = [vp, u32, vp, vp]
        dbl = ctypes.c_double
        lib.orc_t_cold.argtypes = [u32, vp, vp, dbl, vp]
        lib.orc_t_cold.restype = dbl
        lib.orc_t_hot.argtypes = [u32, vp, vp, dbl, vp, vp]
        lib.orc_t_hot.restype = dbl
        lib.orc_balance_iterate.argtypes = [u32, vp, vp, dbl, u32, vp]
        lib.orc_balance_iterate.restype = dbl
        lib.orc_balance_optimum.argtypes = [u32, vp, vp, dbl, vp]
        lib.orc_balance_optimum.restype = dbl
        lib.orc_threshold.argtypes = [u32, vp, vp]
        lib.orc_threshold.restype = dbl
        lib.orc_net_efficiency.argtypes = [dbl, dbl, dbl]
        lib.orc_net_efficiency.restype = dbl
        lib.orc_efficiency_ratio.argtypes = [dbl] * 6
        lib.orc_efficiency_ratio.restype = dbl
        lib.orc_pack.argtypes = [vp, vp, u32, u32, vp, u32, u32, vp, vp]
        lib.orc_unpack.argtypes = [vp, vp, u32, u32, vp, u32, u32, vp]
        lib.orc_bf16_to_f32.argtypes = [ctypes.c_uint16]
        lib.orc_bf16_to_f32.restype = ctypes.c_float
        lib.orc_f32_to_bf16.argtypes = [ctypes.c_float]
        lib.orc_f32_to_bf16.restype = ctypes.c_uint16
        lib.orc_f16_to_f32.argtypes = [ctypes.c_uint16]
        lib.orc_f16_to_f32.restype = ctypes.c_float
        lib.orc_f32_to_f16.argtypes = [ctypes.c_float]
        lib.orc_f32_to_f16.restype = ctypes.c_uint16
        lib.orc_threads.restype = ctypes.c_int
        lib.orc_set_threads.argtypes = [ctypes.c_int]
        lib.orc_set_threads.restype = None
        _lib = lib
    return _lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"oracle: {what}: invalid argument")


def threads() -> int:
    """Number of host threads the definitional sums use."""
    return int(_L().orc_threads())


def set_threads(n: int) -> None:
    """Host threads for the definitional sums from now on (used to time one thread and all)."""
    _L().orc_set_threads(int(n))


def storage_dtype(dtype: int):
    """NumPy dtype used to carry one element (16-bit floats travel as uint16)."""
    return _NP_STORAGE[dtype]


def _ptr_array(arrs: Sequence[np.ndarray]):
    pa = (ctypes.c_void_p * len(arrs))()
    for i, a in enumerate(arrs):
        pa[i] = a.ctypes.data
    return pa


def _as_storage(a: np.ndarray, dtype: int) -> np.ndarray:
    a = np.ascontiguousarray(a)
    want = np.dtype(_NP_STORAGE[dtype])
    if a.dtype != want:
        if a.dtype.itemsize != want.itemsize:
            raise TypeError(f"expected {want.itemsize}-byte elements, got {a.dtype}")
        a = a.view(want)
    return a


def rail_partition(n: int, ratios: Sequence[int], elem_bytes: int,
                   align_bytes: int = 256) -> np.ndarray:
    """Rail boundaries b[0..R] in elements (Sec. 3.5; proportions under Eq. 5)."""
    if align_bytes % elem_bytes:
        raise ValueError("alignment must be a whole number of elements")
    w = np.asarray(ratios, dtype=np.uint32)
    b = np.zeros(len(w) + 1, dtype=np.uint64)
    _check(_L().orc_rail_partition(n, align_bytes // elem_bytes, w.ctypes.data, len(w),
                                   b.ctypes.data), "rail_partition")
    return b


def segment_map(rail_off: Sequence[int], n_nodes: int) -> np.ndarray:
    """Per-rail ring segments, shape [R, N+1] (Eq. 1: N pieces per message)."""
    b = np.ascontiguousarray(rail_off, dtype=np.uint64)
    R = len(b) - 1
    seg = np.zeros((R, n_nodes + 1), dtype=np.uint64)
    _check(_L().orc_segment_map(b.ctypes.data, R, n_nodes, seg.ctypes.data), "segment_map")
    return seg


def sum_float(dtype: int, node_bufs: Sequence[np.ndarray]) -> Tuple[np.ndarray, np.ndarray]:
    """fp64 sum over nodes and fp64 sum of magnitudes, per element (Sec. 4.2)."""
    bufs = [_as_storage(a, dtype) for a in node_bufs]
    n = bufs[0].size
    assert all(a.size == n for a in bufs)
    s = np.empty(n, dtype=np.float64)
    a = np.empty(n, dtype=np.float64)
    _check(_L().orc_sum_float(dtype, _ptr_array(bufs), len(bufs), n, s.ctypes.data,
                              a.ctypes.data), "sum_float")
    return s, a


def sum_i32(node_bufs: Sequence[np.ndarray]) -> np.ndarray:
    """Wrapping int32 sum over nodes, per element."""
    bufs = [_as_storage(a, I32) for a in node_bufs]
    n = bufs[0].size
    assert all(a.size == n for a in bufs)
    out = np.empty(n, dtype=np.int32)
    _check(_L().orc_sum_i32(_ptr_array(bufs), len(bufs), n, out.ctypes.data), "sum_i32")
    return out


def round_to_storage(dtype: int, s: np.ndarray) -> np.ndarray:
    """fp64 sums -> fp32 -> storage type, each rounding to nearest even."""
    s = np.ascontiguousarray(s, dtype=np.float64)
    out = np.empty(s.size, dtype=_NP_STORAGE[dtype])
    _check(_L().orc_round_to_storage(dtype, s.ctypes.data, s.size, out.ctypes.data),
           "round_to_storage")
    return out


def ring_allreduce(dtype: int, node_bufs: Sequence[np.ndarray], seg: np.ndarray,
                   reduce_scatter_only: bool = False
                   ) -> Tuple[List[np.ndarray], np.ndarray]:
    """Step-by-step ring allreduce on private copies (Eq. 1).

    Returns (per-node result buffers, bytes each node sent).
    """
    bufs = [_as_storage(a, dtype).copy() for a in node_bufs]
    n = bufs[0].size
    assert all(a.size == n for a in bufs)
    seg = np.ascontiguousarray(seg, dtype=np.uint64)
    R, Np1 = seg.shape
    assert Np1 == len(bufs) + 1
    sent = np.zeros(len(bufs), dtype=np.uint64)
    _check(_L().orc_ring_allreduce(dtype, _ptr_array(bufs), len(bufs), n, seg.ctypes.data, R,
                                   1 if reduce_scatter_only else 0, sent.ctypes.data),
           "ring_allreduce")
    return bufs, sent


def ring_allgather(dtype: int, node_bufs: Sequence[np.ndarray], seg: np.ndarray
                   ) -> Tuple[List[np.ndarray], np.ndarray]:
    """The allgather half of the ring on private copies (Eq. 1): node r enters owning segment
    (r + 1) mod N of every rail.  Returns (per-node result buffers, bytes each node sent)."""
    bufs = [_as_storage(a, dtype).copy() for a in node_bufs]
    n = bufs[0].size
    seg = np.ascontiguousarray(seg, dtype=np.uint64)
    R, Np1 = seg.shape
    assert Np1 == len(bufs) + 1
    sent = np.zeros(len(bufs), dtype=np.uint64)
    _check(_L().orc_ring_allgather(dtype, _ptr_array(bufs), len(bufs), n, seg.ctypes.data, R,
                                   sent.ctypes.data), "ring_allgather")
    return bufs, sent


def ring_allreduce_chunked(dtype: int, node_bufs: Sequence[np.ndarray], seg: np.ndarray,
                           chunk_elems: int) -> Tuple[List[np.ndarray], np.ndarray, np.ndarray]:
    """Ring allreduce with transfers cut into pieces of at most chunk_elems elements
    (the Ring_Chunked variant of the evaluation section).  Returns (buffers, bytes sent per
    node, messages sent per node)."""
    bufs = [_as_storage(a, dtype).copy() for a in node_bufs]
    n = bufs[0].size
    seg = np.ascontiguousarray(seg, dtype=np.uint64)
    R, Np1 = seg.shape
    assert Np1 == len(bufs) + 1
    sent = np.zeros(len(bufs), dtype=np.uint64)
    msgs = np.zeros(len(bufs), dtype=np.uint64)
    _check(_L().orc_ring_allreduce_chunked(dtype, _ptr_array(bufs), len(bufs), n, seg.ctypes.data,
                                           R, chunk_elems, sent.ctypes.data, msgs.ctypes.data),
           "ring_allreduce_chunked")
    return bufs, sent, msgs


def failover_target(rail_off: Sequence[int], alive: Sequence[bool]) -> int:
    """The surviving rail that takes over a failed rail's slice (Sec. 4.4)."""
    b = np.ascontiguousarray(rail_off, dtype=np.uint64)
    a = np.asarray([1 if x else 0 for x in alive], dtype=np.uint8)
    assert len(a) == len(b) - 1
    t = ctypes.c_uint32(0)
    _check(_L().orc_failover_target(b.ctypes.data, len(a), a.ctypes.data, ctypes.byref(t)),
           "failover_target")
    return int(t.value)


def _model(t_setup, bw):
    ts = np.ascontiguousarray(t_setup, dtype=np.float64)
    b = np.ascontiguousarray(bw, dtype=np.float64)
    assert ts.shape == b.shape and ts.ndim == 1
    return ts, b


def t_cold(t_setup, bw, S: float) -> Tuple[float, int]:
    """Eq. 4: latency with all data on the best single rail; returns (T_cold, that rail)."""
    ts, b = _model(t_setup, bw)
    best = ctypes.c_uint32(0)
    t = _L().orc_t_cold(len(ts), ts.ctypes.data, b.ctypes.data, float(S), ctypes.byref(best))
    return float(t), int(best.value)


def t_hot(t_setup, bw, S: float, alpha) -> float:
    """Eq. 5: latency when rail i carries the share alpha[i] (rails given nothing sit out)."""
    ts, b = _model(t_setup, bw)
    a = np.ascontiguousarray(alpha, dtype=np.float64)
    return float(_L().orc_t_hot(len(ts), ts.ctypes.data, b.ctypes.data, float(S), a.ctypes.data, None))


def balance_iterate(t_setup, bw, S: float, iterations: int = 20000) -> Tuple[np.ndarray, float]:
    """Eq. 8 starting shares, then Eq. 7's descent; returns (shares, T_hot reached)."""
    ts, b = _model(t_setup, bw)
    a = np.zeros(len(ts), dtype=np.float64)
    t = _L().orc_balance_iterate(len(ts), ts.ctypes.data, b.ctypes.data, float(S), iterations,
                                 a.ctypes.data)
    if t < 0:
        raise ValueError("oracle: balance_iterate: invalid argument")
    return a, float(t)


def balance_optimum(t_setup, bw, S: float) -> Tuple[np.ndarray, float]:
    """The minimum of Eq. 5 over all shares (bisection on the finishing time); returns
    (shares, that minimum)."""
    ts, b = _model(t_setup, bw)
    a = np.zeros(len(ts), dtype=np.float64)
    t = _L().orc_balance_optimum(len(ts), ts.ctypes.data, b.ctypes.data, float(S), a.ctypes.data)
    if t < 0:
        raise ValueError("oracle: balance_optimum: invalid argument")
    return a, float(t)


def threshold(t_setup, bw) -> float:
    """Eq. 6: the largest message size at which cold start and the best hot start take the
    same time (infinity if sharing never pays)."""
    ts, b = _model(t_setup, bw)
    t = _L().orc_threshold(len(ts), ts.ctypes.data, b.ctypes.data)
    if t < 0:
        raise ValueError("oracle: threshold: invalid argument")
    return float(t)


def net_efficiency(t_setup: float, bw: float, S: float) -> float:
    """Eq. 2: T_theoretical / T_actual of one network on S bytes (S > 0)."""
    assert S > 0 and bw > 0
    f = _L().orc_net_efficiency
    return float(f(float(t_setup), float(bw), float(S)))


def efficiency_ratio(t_setup_i: float, bw_i: float, S_i: float,
                     t_setup_j: float, bw_j: float, S_j: float) -> float:
    """Eq. 3: throughput of network i on S_i bytes over that of network j on S_j bytes."""
    assert S_i > 0 and S_j > 0
    f = _L().orc_efficiency_ratio
    return float(f(float(t_setup_i), float(bw_i), float(S_i), float(t_setup_j), float(bw_j), float(S_j)))


def pack(node_buf: np.ndarray, seg: np.ndarray, rail: int, seg_ids: Sequence[int],
         elem_bytes: int, send_buf: Optional[np.ndarray] = None) -> Tuple[np.ndarray, int]:
    """Concatenate the listed segments of one rail (Sec. 3.2). Returns (bytes, count)."""
    src = np.ascontiguousarray(node_buf).view(np.uint8)
    seg = np.ascontiguousarray(seg, dtype=np.uint64)
    ids = np.asarray(seg_ids, dtype=np.uint32)
    n_nodes = seg.shape[1] - 1
    if send_buf is None:
        total = int(sum(int(seg[rail, j + 1] - seg[rail, j]) for j in ids)) * elem_bytes
        send_buf = np.zeros(total, dtype=np.uint8)
    packed = ctypes.c_uint64(0)
    _check(_L().orc_pack(src.ctypes.data, seg.ctypes.data, n_nodes, rail, ids.ctypes.data,
                         len(ids), elem_bytes, send_buf.ctypes.data, ctypes.byref(packed)),
           "pack")
    return send_buf, int(packed.value)


def unpack(send_buf: np.ndarray, seg: np.ndarray, rail: int, seg_ids: Sequence[int],
           elem_bytes: int, node_buf: np.ndarray) -> None:
    """Scatter a packed buffer back into the listed segments of node_buf (in place)."""
    assert node_buf.flags["C_CONTIGUOUS"] and node_buf.flags["WRITEABLE"]
    src = np.ascontiguousarray(send_buf).view(np.uint8)
    seg = np.ascontiguousarray(seg, dtype=np.uint64)
    ids = np.asarray(seg_ids, dtype=np.uint32)
    n_nodes = seg.shape[1] - 1
    _check(_L().orc_unpack(src.ctypes.data, seg.ctypes.data, n_nodes, rail, ids.ctypes.data,
                           len(ids), elem_bytes, node_buf.ctypes.data), "unpack")


def bf16_to_f32(h: int) -> float:
    return float(_L().orc_bf16_to_f32(int(h) & 0xFFFF))


def f32_to_bf16(f: float) -> int:
    return int(_L().orc_f32_to_bf16(ctypes.c_float(f)))


def f16_to_f32(h: int) -> float:
    return float(_L().orc_f16_to_f32(int(h) & 0xFFFF))


def f32_to_f16(f: float) -> int:
    return int(_L().orc_f32_to_f16(ctypes.c_float(f)))
