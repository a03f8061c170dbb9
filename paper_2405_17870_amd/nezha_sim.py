"""Thin binding over the C-ABI library ``libnezha_sim.so`` (see include/nezha_sim.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels (or, for the two index maps, in its host C++).  PyTorch is used for
device memory and streams.  There is no fallback: if the library has not been
built or cannot be loaded, the first call raises.

Function names and argument order follow the C header; each docstring cites
the passage of Nezha (arXiv 2405.17870) that defines the operation.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnezha_sim.so")

NZ_MAX_NODES = 128
NZ_MAX_RAILS = 8

NZ_F32, NZ_BF16, NZ_F16, NZ_I32 = 0, 1, 2, 3
NZ_RING_STEPWISE, NZ_FUSED = 0, 1

DTYPE_CODE = {"f32": NZ_F32, "bf16": NZ_BF16, "f16": NZ_F16, "i32": NZ_I32}
MODE_CODE = {"ring-stepwise": NZ_RING_STEPWISE, "ring": NZ_RING_STEPWISE, "fused": NZ_FUSED}
ELEM_BYTES = {"f32": 4, "bf16": 2, "f16": 2, "i32": 4}

EXPORTS = [
    "nz_status_str", "nz_last_hip_error", "nz_dtype_bytes", "nz_rail_partition",
    "nz_rail_partition_ex", "nz_segment_map", "nz_allreduce_sim", "nz_reduce_scatter_sim",
    "nz_allgather_sim", "nz_allreduce_sim_chunked", "nz_failover_target",
    "nz_allreduce_sim_failover", "nz_pack", "nz_unpack", "nz_balance", "nz_balance_threshold",
    "nz_balance_iterate", "nz_hbm_place", "nz_allreduce_launches",
    "nz_net_efficiency", "nz_efficiency_ratio",
]


class NezhaSimError(RuntimeError):
    """A library call returned a status other than NZ_OK."""

    def __init__(self, status: int, text: str):
        super().__init__(f"nezha_sim: status {status}: {text}")
        self.status = status


_lib = None


def load() -> ctypes.CDLL:
    """Load ``libnezha_sim.so``; raises if it is missing (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2405_17870_amd.build "
            "or __graft_entry__.build()); there is no fallback path")
    import torch  # loads the HIP runtime this library must share with torch
    _TORCH_DTYPE.update({"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16,
                         "i32": torch.int32})
    lib = ctypes.CDLL(LIB_PATH)
    u64, u32, vp, i32 = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_int
    lib.nz_status_str.argtypes = [i32]
    lib.nz_status_str.restype = ctypes.c_char_p
    lib.nz_last_hip_error.argtypes = []
    lib.nz_last_hip_error.restype = ctypes.c_char_p
    lib.nz_dtype_bytes.argtypes = [i32]
    lib.nz_dtype_bytes.restype = u32
    lib.nz_rail_partition.argtypes = [u64, u32, vp, u32, vp]
    lib.nz_rail_partition_ex.argtypes = [u64, u32, u32, vp, u32, vp]
    lib.nz_segment_map.argtypes = [vp, u32, u32, vp]
    lib.nz_allreduce_sim.argtypes = [vp, u32, u64, vp, u32, i32, i32, vp, vp]
    lib.nz_reduce_scatter_sim.argtypes = [vp, u32, u64, vp, u32, i32, i32, vp, vp]
    lib.nz_allgather_sim.argtypes = [vp, u32, u64, vp, u32, i32, i32, vp]
    lib.nz_allreduce_sim_chunked.argtypes = [vp, u32, u64, vp, u32, i32, u64, vp, vp]
    lib.nz_failover_target.argtypes = [vp, u32, vp, vp]
    lib.nz_allreduce_sim_failover.argtypes = [vp, u32, u64, vp, u32, i32, i32, vp, u32, vp, vp]
    lib.nz_pack.argtypes = [vp, u32, vp, u32, u32, vp, u32, u32, vp, u64, vp, vp]
    lib.nz_unpack.argtypes = [vp, u32, vp, u32, u32, vp, u32, u32, vp, vp]
    for name in ("nz_rail_partition", "nz_rail_partition_ex", "nz_segment_map",
                 "nz_allreduce_sim", "nz_reduce_scatter_sim", "nz_allgather_sim", "nz_pack",
                 "nz_unpack", "nz_allreduce_sim_chunked", "nz_failover_target",
                 "nz_allreduce_sim_failover"):
        getattr(lib, name).restype = i32
    lib.nz_balance.argtypes = [vp, u32, ctypes.c_double, vp, vp, vp, vp, vp, vp]
    lib.nz_balance.restype = i32
    lib.nz_balance_threshold.argtypes = [vp, u32, vp]
    lib.nz_balance_threshold.restype = i32
    lib.nz_balance_iterate.argtypes = [vp, u32, ctypes.c_double, u32, vp, vp, vp, vp]
    lib.nz_balance_iterate.restype = i32
    lib.nz_allreduce_launches.argtypes = [u32, u64, vp, u32, i32, i32, u32, u64, vp]
    lib.nz_allreduce_launches.restype = i32
    lib.nz_hbm_place.argtypes = [u64, vp, u32, u64, i32, u32, vp]
    lib.nz_hbm_place.restype = i32
    lib.nz_net_efficiency.argtypes = [vp, ctypes.c_double, vp]
    lib.nz_net_efficiency.restype = i32
    lib.nz_efficiency_ratio.argtypes = [vp, u32, ctypes.c_double, vp, vp]
    lib.nz_efficiency_ratio.restype = i32
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != 0:
        lib = load()
        text = lib.nz_status_str(status).decode()
        hip = lib.nz_last_hip_error().decode()
        raise NezhaSimError(status, text + (f" ({hip})" if status == 5 and hip else ""))


_u32_cache = {}


def _u32_array(values: Sequence[int]):
    """A ctypes array of unsigned 32-bit values; arrays of short tuples (rail weights, segment
    lists) are kept, since callers pass the same ones again and again."""
    key = tuple(values) if len(values) <= 16 else None
    if key is not None:
        hit = _u32_cache.get(key)
        if hit is not None:
            return hit
    vals = [int(v) for v in values]
    for v in vals:
        if v < 0 or v > 0xFFFFFFFF:
            raise ValueError("value does not fit an unsigned 32-bit integer")
    arr = (ctypes.c_uint32 * max(len(vals), 1))(*vals)
    if key is not None and len(_u32_cache) < 1024:
        _u32_cache[key] = arr
    return arr


_TORCH_DTYPE = {}          # dtype string -> torch dtype, filled by load()


class BufferTable:
    """A host array of device addresses that has been checked once and can be handed to any
    number of calls (the per-call cost of checking 2 N tensors is what a small allreduce
    notices).  Keeps the tensors alive.  ``n_elems`` is what every buffer is known to hold."""

    def __init__(self, tensors, dtype: Optional[str] = None, elem_bytes: Optional[int] = None,
                 what: str = "buffer"):
        self.tensors = list(tensors)
        self.dtype, self.elem_bytes = dtype, elem_bytes
        self.n_elems = min((t.numel() for t in self.tensors if hasattr(t, "numel")), default=0)
        self.array = _ptr_array(self.tensors, 0, dtype, elem_bytes, what)

    def __len__(self):
        return len(self.tensors)


def _ptr_array(tensors, min_elems: int = 0, dtype: Optional[str] = None,
               elem_bytes: Optional[int] = None, what: str = "buffer") -> ctypes.Array:
    """Host array of device addresses.  A torch tensor is checked before its address is taken --
    on the device, contiguous, of the stated element type (or element size) and holding at
    least ``min_elems`` elements -- because the kernels trust these facts; a raw integer
    address is passed through as it is.  A BufferTable was checked when it was made."""
    if isinstance(tensors, BufferTable):
        if dtype is not None and tensors.dtype is not None and tensors.dtype != dtype:
            raise ValueError(f"{what} table was made for {tensors.dtype}, the call says {dtype}")
        if tensors.n_elems < min_elems and any(hasattr(t, "numel") for t in tensors.tensors):
            raise ValueError(f"{what} table holds {tensors.n_elems} elements per buffer, the call needs {min_elems}")
        return tensors.array
    arr = (ctypes.c_void_p * max(len(tensors), 1))()
    want = _TORCH_DTYPE.get(dtype) if dtype is not None else None
    check_size = elem_bytes in (2, 4)          # other sizes: the library refuses
    for i, t in enumerate(tensors):
        if not hasattr(t, "data_ptr"):
            arr[i] = int(t)
            continue
        if not t.is_cuda:
            raise ValueError(f"{what} {i} is not a device tensor")
        if not t.is_contiguous():
            raise ValueError(f"{what} {i} is not contiguous")
        if want is not None and t.dtype is not want:
            raise ValueError(f"{what} {i} has dtype {t.dtype}, the call says {dtype}")
        if check_size and t.element_size() != elem_bytes:
            raise ValueError(f"{what} {i} has {t.element_size()}-byte elements, the call says {elem_bytes}")
        if t.numel() < min_elems:
            raise ValueError(f"{what} {i} holds {t.numel()} elements, the call needs {min_elems}")
        arr[i] = t.data_ptr()
    return arr


def _stream_handle(stream) -> ctypes.c_void_p:
    """A torch stream, a raw hipStream_t as an integer, or None for torch's current stream."""
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def nz_rail_partition(n_elems: int, elem_bytes: int, ratios: Sequence[int],
                      align_bytes: Optional[int] = None) -> np.ndarray:
    """Rail boundaries in elements, ``n_rails + 1`` entries (Sec. 3.4, 3.5; shares sum to
    one, Sec. 4.3 under Eq. 5).  ``align_bytes=None`` is the library's fixed 256 bytes."""
    lib = load()
    w = _u32_array(ratios)
    out = np.zeros(len(ratios) + 1, dtype=np.uint64)
    if align_bytes is None:
        _check(lib.nz_rail_partition(n_elems, elem_bytes, w, len(ratios), out.ctypes.data))
    else:
        _check(lib.nz_rail_partition_ex(n_elems, elem_bytes, align_bytes, w, len(ratios),
                                        out.ctypes.data))
    return out


def nz_segment_map(rail_off: Sequence[int], n_nodes: int) -> np.ndarray:
    """Ring segments of every rail, shape ``[n_rails, n_nodes + 1]`` (Sec. 2.1.1, Eq. 1)."""
    lib = load()
    b = np.ascontiguousarray(rail_off, dtype=np.uint64)
    n_rails = len(b) - 1
    seg = np.zeros((max(n_rails, 0), n_nodes + 1), dtype=np.uint64)
    _check(lib.nz_segment_map(b.ctypes.data, n_rails, n_nodes, seg.ctypes.data))
    return seg


def nz_allreduce_sim(node_bufs: Sequence, n_elems: int, ratios: Sequence[int], dtype: str,
                     mode: str, out_bufs: Sequence, stream=None) -> None:
    """Sum of the nodes' buffers into every output buffer (Sec. 4.2 aggregation phase; ring
    schedule of Sec. 2.1.1 / Eq. 1; rails per Sec. 4.1).  Asynchronous on ``stream``
    (default: torch's current stream).  Buffers are torch tensors or raw device addresses."""
    lib = load()
    if len(out_bufs) != len(node_bufs):
        raise ValueError("out_bufs must have one entry per node")
    _check(lib.nz_allreduce_sim(_ptr_array(node_bufs, n_elems, dtype, what="node buffer"), len(node_bufs), n_elems,
                                _u32_array(ratios), len(ratios), DTYPE_CODE[dtype],
                                MODE_CODE[mode], _ptr_array(out_bufs, n_elems, dtype, what="output buffer"),
                                _stream_handle(stream)))


def nz_allreduce_launches(n_nodes: int, n_elems: int, ratios: Sequence[int], dtype: str, mode: str,
                          n_distinct_outputs: int, outputs_span_bytes: int = 0) -> int:
    """Kernel launches one nz_allreduce_sim call issues for these arguments.  Host only.
    outputs_span_bytes: from the start of the lowest output buffer to the end of the highest
    (0: not known, taken to lie close together)."""
    lib = load()
    out = ctypes.c_uint64(0)
    _check(lib.nz_allreduce_launches(n_nodes, n_elems, _u32_array(ratios), len(ratios), DTYPE_CODE[dtype],
                                     MODE_CODE[mode], n_distinct_outputs, outputs_span_bytes, ctypes.byref(out)))
    return int(out.value)


def nz_reduce_scatter_sim(node_bufs: Sequence, n_elems: int, ratios: Sequence[int], dtype: str,
                          mode: str, out_bufs: Sequence, stream=None) -> None:
    """The reduce-scatter half (Sec. 2.1.1, Eq. 1): out_bufs[(j - 1) mod N] receives the sum of
    segment j of every rail; the rest of the outputs is unspecified."""
    lib = load()
    if len(out_bufs) != len(node_bufs):
        raise ValueError("out_bufs must have one entry per node")
    _check(lib.nz_reduce_scatter_sim(_ptr_array(node_bufs, n_elems, dtype, what="node buffer"), len(node_bufs), n_elems,
                                     _u32_array(ratios), len(ratios), DTYPE_CODE[dtype],
                                     MODE_CODE[mode], _ptr_array(out_bufs, n_elems, dtype, what="output buffer"),
                                     _stream_handle(stream)))


def nz_allgather_sim(bufs: Sequence, n_elems: int, ratios: Sequence[int], dtype: str, mode: str,
                     stream=None) -> None:
    """The allgather half, in place (Sec. 2.1.1, Eq. 1): node r enters owning segment
    (r + 1) mod N of every rail; every buffer leaves holding every segment."""
    lib = load()
    _check(lib.nz_allgather_sim(_ptr_array(bufs, n_elems, dtype), len(bufs), n_elems, _u32_array(ratios),
                                len(ratios), DTYPE_CODE[dtype], MODE_CODE[mode],
                                _stream_handle(stream)))


def nz_allreduce_sim_chunked(node_bufs: Sequence, n_elems: int, ratios: Sequence[int], dtype: str,
                             chunk_elems: int, out_bufs: Sequence, stream=None) -> None:
    """Ring_Chunked allreduce (evaluation section: packets split and pipelined): the ring with
    every transfer cut into pieces of at most ``chunk_elems`` elements, one launch per piece."""
    lib = load()
    if len(out_bufs) != len(node_bufs):
        raise ValueError("out_bufs must have one entry per node")
    _check(lib.nz_allreduce_sim_chunked(_ptr_array(node_bufs, n_elems, dtype, what="node buffer"), len(node_bufs), n_elems,
                                        _u32_array(ratios), len(ratios), DTYPE_CODE[dtype],
                                        chunk_elems, _ptr_array(out_bufs, n_elems, dtype, what="output buffer"),
                                        _stream_handle(stream)))


def nz_failover_target(rail_off: Sequence[int], alive: Sequence[bool]) -> int:
    """The surviving rail that takes over a failed rail's slice (Sec. 4.4). Host only."""
    lib = load()
    b = np.ascontiguousarray(rail_off, dtype=np.uint64)
    a = np.asarray([1 if x else 0 for x in alive], dtype=np.uint8)
    if len(a) != len(b) - 1:
        raise ValueError("one flag per rail")
    t = ctypes.c_uint32(0)
    _check(lib.nz_failover_target(b.ctypes.data, len(a), a.ctypes.data, ctypes.byref(t)))
    return int(t.value)


def nz_allreduce_sim_failover(node_bufs: Sequence, n_elems: int, ratios: Sequence[int], dtype: str,
                              mode: str, out_bufs: Sequence, failed_rail: int, stream=None) -> int:
    """Allreduce with one rail failing (Sec. 4.4): its slice is processed as a second pass by
    the surviving rail with the most data.  Returns that rail's index."""
    lib = load()
    if len(out_bufs) != len(node_bufs):
        raise ValueError("out_bufs must have one entry per node")
    t = ctypes.c_uint32(0)
    _check(lib.nz_allreduce_sim_failover(_ptr_array(node_bufs, n_elems, dtype, what="node buffer"), len(node_bufs), n_elems,
                                         _u32_array(ratios), len(ratios), DTYPE_CODE[dtype],
                                         MODE_CODE[mode], _ptr_array(out_bufs, n_elems, dtype, what="output buffer"), failed_rail,
                                         ctypes.byref(t), _stream_handle(stream)))
    return int(t.value)


def nz_pack(node_bufs: Sequence, seg_off: np.ndarray, rail: int, seg_ids: Sequence[int],
            elem_bytes: int, send_bufs: Sequence, send_capacity_bytes: int, stream=None) -> int:
    """Stage the listed segments of one rail into contiguous send buffers, all nodes at once
    (Sec. 3.2: UnboundBuffer to the rail's Buffer).  Returns the packed bytes per node."""
    lib = load()
    seg = np.ascontiguousarray(seg_off, dtype=np.uint64)
    n_rails, n_nodes = seg.shape[0], seg.shape[1] - 1
    if len(node_bufs) != n_nodes or len(send_bufs) != n_nodes:
        raise ValueError("one node buffer and one send buffer per node")
    packed = ctypes.c_uint64(0)
    sized = elem_bytes in (2, 4)             # any other element size is the library's to refuse
    span = int(seg[rail, n_nodes]) if sized and 0 <= rail < n_rails else 0
    cap_elems = -(-int(send_capacity_bytes) // elem_bytes) if sized else 0
    _check(lib.nz_pack(_ptr_array(node_bufs, span, elem_bytes=elem_bytes, what="node buffer"), n_nodes,
                       seg.ctypes.data, n_rails, rail, _u32_array(seg_ids), len(seg_ids), elem_bytes,
                       _ptr_array(send_bufs, cap_elems, elem_bytes=elem_bytes, what="send buffer"),
                       send_capacity_bytes, ctypes.byref(packed), _stream_handle(stream)))
    return int(packed.value)


def nz_unpack(send_bufs: Sequence, seg_off: np.ndarray, rail: int, seg_ids: Sequence[int],
              elem_bytes: int, node_bufs: Sequence, stream=None) -> None:
    """Scatter contiguous send buffers back into the listed segments (Sec. 3.2: results
    return from the rail's Buffer to the UnboundBuffer)."""
    lib = load()
    seg = np.ascontiguousarray(seg_off, dtype=np.uint64)
    n_rails, n_nodes = seg.shape[0], seg.shape[1] - 1
    if len(node_bufs) != n_nodes or len(send_bufs) != n_nodes:
        raise ValueError("one node buffer and one send buffer per node")
    sized = elem_bytes in (2, 4) and 0 <= rail < n_rails
    span = int(seg[rail, n_nodes]) if sized else 0
    total = sum(int(seg[rail, j + 1] - seg[rail, j]) for j in seg_ids if 0 <= int(j) < n_nodes) if sized else 0
    _check(lib.nz_unpack(_ptr_array(send_bufs, total, elem_bytes=elem_bytes, what="send buffer"), n_nodes,
                         seg.ctypes.data, n_rails, rail, _u32_array(seg_ids), len(seg_ids), elem_bytes,
                         _ptr_array(node_bufs, span, elem_bytes=elem_bytes, what="node buffer"),
                         _stream_handle(stream)))


NZ_RATIO_SCALE = 1 << 20


def _models(setup_s: Sequence[float], bytes_per_s: Sequence[float]):
    if len(setup_s) != len(bytes_per_s):
        raise ValueError("one startup latency and one bandwidth per rail")
    arr = (ctypes.c_double * (2 * max(len(setup_s), 1)))()
    for i, (t, b) in enumerate(zip(setup_s, bytes_per_s)):
        arr[2 * i], arr[2 * i + 1] = float(t), float(b)
    return arr


def nz_balance(setup_s: Sequence[float], bytes_per_s: Sequence[float], msg_bytes: float) -> dict:
    """Shares of a message among rails of known startup latency and bandwidth (Sec. 4.3,
    Eq. 4-8).  Host only.  Returns alpha, ratios (sum 2**20), t_cold, t_hot, best_rail, hot."""
    lib = load()
    R = len(setup_s)
    alpha = np.zeros(max(R, 1), dtype=np.float64)
    ratios = np.zeros(max(R, 1), dtype=np.uint32)
    tc, th = ctypes.c_double(0), ctypes.c_double(0)
    best, hot = ctypes.c_uint32(0), ctypes.c_int(0)
    _check(lib.nz_balance(_models(setup_s, bytes_per_s), R, float(msg_bytes), alpha.ctypes.data,
                          ratios.ctypes.data, ctypes.byref(tc), ctypes.byref(th), ctypes.byref(best),
                          ctypes.byref(hot)))
    return {"alpha": alpha[:R], "ratios": ratios[:R], "t_cold": tc.value, "t_hot": th.value,
            "best_rail": int(best.value), "hot": bool(hot.value)}


def nz_balance_threshold(setup_s: Sequence[float], bytes_per_s: Sequence[float]) -> float:
    """Message size up to which all data goes over the best single rail (Sec. 4.3, Eq. 6)."""
    lib = load()
    out = ctypes.c_double(0)
    _check(lib.nz_balance_threshold(_models(setup_s, bytes_per_s), len(setup_s), ctypes.byref(out)))
    return out.value


def nz_balance_iterate(setup_s: Sequence[float], bytes_per_s: Sequence[float], msg_bytes: float,
                       max_iterations: int = 100) -> dict:
    """The shares by the paper's iteration (Sec. 4.3): Eq. 8 start, then steps of Eq. 7 until the
    data-length table has converged.  Host only.  Returns alpha, ratios, t_hot, iterations."""
    lib = load()
    R = len(setup_s)
    alpha = np.zeros(max(R, 1), dtype=np.float64)
    ratios = np.zeros(max(R, 1), dtype=np.uint32)
    th, it = ctypes.c_double(0), ctypes.c_uint32(0)
    _check(lib.nz_balance_iterate(_models(setup_s, bytes_per_s), R, float(msg_bytes),
                                  int(max_iterations), alpha.ctypes.data, ratios.ctypes.data,
                                  ctypes.byref(th), ctypes.byref(it)))
    return {"alpha": alpha[:R], "ratios": ratios[:R], "t_hot": th.value, "iterations": int(it.value)}


NZ_TOLERANCE_TAU = 5.0


def nz_net_efficiency(setup_s: float, bytes_per_s: float, msg_bytes: float) -> float:
    """Network efficiency of one rail on a message (Sec. 2.1.2, Eq. 2).  Host only."""
    lib = load()
    out = ctypes.c_double(0)
    _check(lib.nz_net_efficiency(_models([setup_s], [bytes_per_s]), float(msg_bytes), ctypes.byref(out)))
    return out.value


def nz_efficiency_ratio(setup_s: Sequence[float], bytes_per_s: Sequence[float], msg_bytes: float,
                        alpha: Optional[Sequence[float]] = None) -> float:
    """Real-time efficiency ratio of the rails under the given shares (Sec. 2.2.1, Eq. 3):
    highest throughput over lowest; splitting pays only while it stays below tau = 5."""
    lib = load()
    a = None
    if alpha is not None:
        if len(alpha) != len(setup_s):
            raise ValueError("one share per rail")
        a = (ctypes.c_double * max(len(alpha), 1))(*[float(x) for x in alpha])
    out = ctypes.c_double(0)
    _check(lib.nz_efficiency_ratio(_models(setup_s, bytes_per_s), len(setup_s), float(msg_bytes), a,
                                   ctypes.byref(out)))
    return out.value


NZ_HBM_REGIONS = 3
NZ_HBM_REGION_BYTES = 96 << 30


def nz_hbm_place(arena_bytes: int, used: np.ndarray, count: int, bytes_each: int, spread: bool,
                 first_region: int = 0) -> np.ndarray:
    """Offsets of ``count`` buffers inside one arena that covers HBM: spread over the three 96 GiB
    regions (buffers that get written) or together in one region (buffers that are only read).
    ``used`` (uint64, three counters, zeros at first) is updated in place.  Host only."""
    lib = load()
    if used.dtype != np.uint64 or used.shape != (NZ_HBM_REGIONS,) or not used.flags["C_CONTIGUOUS"]:
        raise ValueError("used must be a contiguous array of three uint64 counters")
    off = np.zeros(max(count, 1), dtype=np.uint64)
    _check(lib.nz_hbm_place(int(arena_bytes), used.ctypes.data, int(count), int(bytes_each),
                            1 if spread else 0, int(first_region), off.ctypes.data))
    return off[:count]
