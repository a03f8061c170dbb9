#!/usr/bin/env python3
"""Benchmark of the allreduce reduction engine on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic gradients
already resident in HBM:

  1. nz_allreduce_sim, fused mode         (rail partition + segment cut + N-way reduce/broadcast)
  2. nz_allreduce_sim, ring-stepwise mode (the same sums as 2(N-1) ring steps)
  3. nz_pack of every rail, all nodes     (node buffers -> contiguous send buffers)
  4. nz_unpack of every rail, all nodes   (send buffers -> node buffers)

The reported value is effective HBM throughput of the step: the bytes the method itself must
move (fused (N+K)*S, ring-stepwise 5(N-1)*S, pack 2*N*S, unpack 2*N*S; S = payload bytes per
node, K = distinct output buffers = N) divided by the step time.  Per-part times come from HIP
events on the stream the kernels run on; `roofline` describes the fused kernel.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak


def parse_args():
    p = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=20)
    p.add_argument("--warmup", type=int, default=5)
    p.add_argument("--workload", default="c4", help="c1, c1_i32, c2, c3, c4 (default), c5")
    p.add_argument("--parts", default="fused,ring,pack,unpack",
                   help="comma list of parts to run in a step (default: all four); also available: "
                        "rs, ag = fused reduce-scatter-only / allgather-only; chunked = Ring_Chunked; "
                        "failover = fused allreduce with the last rail failing; "
                        "packed = fused allreduce, in place, of every rail's contiguous send buffers "
                        "(the route pack -> allreduce -> unpack; put it between pack and unpack); "
                        "packed_out = the same allreduce from the send buffers into separate result "
                        "buffers (out of place; unpack_out then unpacks from those)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--placement", default="spread", choices=["spread", "packed", "torch"],
                   help="where the buffers live in HBM: spread = inputs in the first 96 GiB region, "
                        "written buffers striped over all three regions (default); packed = all in the "
                        "first region; torch = plain torch allocations")
    p.add_argument("--no-plain", action="store_true",
                   help="skip the second measurement of every part on plain torch allocations "
                        "(reported as plain_allocations when the timed placement is another one)")
    p.add_argument("--packed-offset-gib", type=float, default=0.0,
                   help="with --placement packed: arena offset at which the buffers start")
    p.add_argument("--chunk-elems", type=int, default=1 << 20,
                   help="piece length of the optional part 'chunked' (Ring_Chunked)")
    p.add_argument("--shared-output", action="store_true",
                   help="fused part: every node's output is the same buffer (K = 1 distinct output)")
    p.add_argument("--pack-order", default="rail", choices=["rail", "ring"],
                   help="segment list of pack/unpack: the whole rail in order (one aligned run per "
                        "node) or the order a node sends its segments in (misaligned runs: the re-alignment path)")
    p.add_argument("--graph", action="store_true",
                   help="capture one step in a HIP graph and time its replays (no per-part times); "
                        "with --sweep: capture the calls of each size and time the replay")
    p.add_argument("--shapes", action="store_true",
                   help="time every entry point over node counts, sizes and rail layouts beyond the five "
                        "workloads (plain allocations; one JSON line; ungraded)")
    p.add_argument("--sweep", action="store_true",
                   help="instead of the step: time fused and ring-stepwise allreduce over message sizes "
                        "2 KB .. 64 MB (fp32, 2 rails 1:1) at 4 and 8 nodes and print one JSON line")
    p.add_argument("--cpu-sample-elems", type=int, default=32 * 1024 * 1024)
    return p.parse_args()


def device_code_digest() -> str:
    """SHA-256 over the device code the counters were taken on (csrc/nz_device.h)."""
    src = os.path.join(ROOT, "paper_2405_17870_amd", "csrc", "nz_device.h")
    return hashlib.sha256(open(src, "rb").read()).hexdigest()


def recorded_traffic(kind: str):
    """HBM bytes per launch from the committed counter runs, or None if the kernels have
    changed since they were taken."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        rec = json.load(open(path))
        if rec.get("kernel_source_sha256") != device_code_digest():
            return None
        return rec.get(kind)
    except (OSError, ValueError):
        return None


def device_facts(torch):
    """What the runtime reports about the card (informational; the roofline uses the published peak)."""
    p = torch.cuda.get_device_properties(0)
    facts = {"name": p.name, "compute_units": p.multi_processor_count,
             "hbm_bytes": p.total_memory}
    for key in ("gcnArchName", "memory_clock_rate", "memory_bus_width", "L2_cache_size"):
        if hasattr(p, key):
            facts[key] = getattr(p, key)
    return facts


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(w, n_sample: int, parts):
    """The oracle, as it stands, on a bounded slice of the same workload (same node count, same
    ratios, the first n_sample elements of every node).  Every leg is reported on its own, in
    algorithmic bytes per second of what that leg does:
      sum, one thread / all threads ... the definitional N-way sum + rounding to the storage
          type: N reads and one result written per element, (N + 1) * S;
      ring, one thread ... the literal ring, 5 (N - 1) * S;
      pack and unpack, one thread ... 2 * S each per node and rail.
    `value` is the all-threads definitional sum."""
    import numpy as np
    import oracle as orc
    from paper_2405_17870_amd import inputs

    code = {"f32": orc.F32, "bf16": orc.BF16, "f16": orc.F16, "i32": orc.I32}[w.dtype]
    e = inputs.ELEM_BYTES[w.dtype]
    N = w.n_nodes
    n = min(n_sample, w.n_elems)
    host = [inputs.to_host_storage(t) for t in inputs.workload_buffers(w, device="cpu", n_elems=n)]
    S = n * e
    seg = orc.segment_map(orc.rail_partition(n, w.ratios, e), N)
    all_threads = orc.threads()

    def definitional_sum(bufs):
        if w.dtype == "i32":
            orc.sum_i32(bufs)
        else:
            s, _ = orc.sum_float(code, bufs)
            orc.round_to_storage(code, s)

    legs = {}
    t_all = time.perf_counter()
    t0 = time.perf_counter()
    definitional_sum(host)
    dt = time.perf_counter() - t0
    legs["sum_all_threads"] = {"GBps": round((N + 1) * S / dt / 1e9, 3), "seconds": round(dt, 3),
                               "threads": all_threads, "elems_per_node": n}
    n1 = max(n // 8, 1)                                  # one thread is slow: an eighth of the slice
    orc.set_threads(1)
    try:
        t0 = time.perf_counter()
        definitional_sum([h[:n1] for h in host])
        dt = time.perf_counter() - t0
    finally:
        orc.set_threads(all_threads)
    legs["sum_one_thread"] = {"GBps": round((N + 1) * n1 * e / dt / 1e9, 3), "seconds": round(dt, 3),
                              "threads": 1, "elems_per_node": n1}
    if "ring" in parts:
        t0 = time.perf_counter()
        orc.ring_allreduce(code, host, seg)
        dt = time.perf_counter() - t0
        legs["ring_one_thread"] = {"GBps": round(5 * (N - 1) * S / dt / 1e9, 3), "seconds": round(dt, 3),
                                   "threads": 1, "elems_per_node": n}
    if "pack" in parts or "unpack" in parts:
        ids = list(range(N))
        moved = 0
        t0 = time.perf_counter()
        for rail in range(len(w.ratios)):
            for m in range(N):
                buf, _ = orc.pack(host[m], seg, rail, ids, e)
                orc.unpack(buf, seg, rail, ids, e, host[m])
                moved += 4 * buf.size
        dt = time.perf_counter() - t0
        legs["pack_unpack_one_thread"] = {"GBps": round(moved / dt / 1e9, 3), "seconds": round(dt, 3),
                                          "threads": 1, "elems_per_node": n}
    total = time.perf_counter() - t_all
    return {
        "value": legs["sum_all_threads"]["GBps"], "unit": "GB/s", "cores": all_threads,
        "kind": "oracle", "seconds": round(total, 3), "cpu": cpu_model(),
        "hardware_threads": os.cpu_count(), "legs": legs,
        "sample": (f"the first {n} elements of each of the {N} nodes of {w.name}; value = the oracle's "
                   f"definitional {N}-way sum and rounding on {all_threads} OpenMP threads, "
                   f"({N} + 1) * S bytes over its time; the other legs (one thread) are listed under legs"),
    }


def size_sweep(torch, nz, dev, use_graph: bool = False) -> int:
    """Latency and payload throughput (message bytes / time, the paper's definition) of one
    allreduce per message size, the range of the paper's allreduce benchmark.  The fit
    t = t0 + S / B per mode gives the fixed cost per call and the asymptotic payload rate,
    the two quantities of the paper's network efficiency model (Sec. 2.1.2, Eq. 2).
    With use_graph the calls of one size are captured in a HIP graph and its replay is timed:
    the fixed cost is then the GPU's per launch, without the host's per call."""
    rows = []
    for N in (4, 8):
        for log2 in range(11, 27):
            S = 1 << log2
            n = S // 4
            ins_t = [torch.randn(n, device=dev) * 1e-2 for _ in range(N)]
            outs_t = [torch.empty_like(t) for t in ins_t]
            # checked once, used by every call of this size (what a caller in a loop does)
            ins, outs = nz.BufferTable(ins_t, "f32"), nz.BufferTable(outs_t, "f32")
            row = {"n_nodes": N, "msg_bytes": S}
            st = None if use_graph else torch.cuda.current_stream().cuda_stream     # the raw stream handle
            for mode in ("fused", "ring-stepwise"):
                reps = 200 if S <= (1 << 22) else 30
                for _ in range(5):
                    nz.nz_allreduce_sim(ins, n, (1, 1), "f32", mode, outs)
                torch.cuda.synchronize()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                if use_graph:
                    graph = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(graph):
                        for _ in range(reps):
                            nz.nz_allreduce_sim(ins, n, (1, 1), "f32", mode, outs)
                    graph.replay()
                    torch.cuda.synchronize()
                    a.record()
                    graph.replay()
                    b.record()
                else:
                    a.record()
                    for _ in range(reps):
                        nz.nz_allreduce_sim(ins, n, (1, 1), "f32", mode, outs, st)
                    b.record()
                torch.cuda.synchronize()
                us = a.elapsed_time(b) * 1e3 / reps
                row[mode] = {"us": round(us, 2), "payload_GBps": round(S / us / 1e3, 3)}
            rows.append(row)
    fits = {}
    for N in (4, 8):
        for mode in ("fused", "ring-stepwise"):
            pts = [(r["msg_bytes"], r[mode]["us"]) for r in rows if r["n_nodes"] == N]
            # least squares of t = t0 + S / B
            m = len(pts)
            sx = sum(x for x, _ in pts); sy = sum(y for _, y in pts)
            sxx = sum(x * x for x, _ in pts); sxy = sum(x * y for x, y in pts)
            slope = (m * sxy - sx * sy) / (m * sxx - sx * sx)
            t0 = (sy - slope * sx) / m
            fits[f"{mode}_N{N}"] = {"t0_us": round(t0, 2), "payload_GBps": round(1.0 / slope / 1e3, 2),
                                    "half_efficiency_bytes": int(t0 / slope)}
    # The Load Balancer (Sec. 4.3) on rails whose startup latency and bandwidth are the fitted
    # ones: what it would do with two rails that behave like the two modes measured here.
    balancer = {}
    for N in (4, 8):
        f, r = fits[f"fused_N{N}"], fits[f"ring-stepwise_N{N}"]
        setup = [f["t0_us"] * 1e-6, r["t0_us"] * 1e-6]
        rate = [f["payload_GBps"] * 1e9, r["payload_GBps"] * 1e9]
        if min(setup) <= 0 or min(rate) <= 0:
            continue
        splits = []
        for S in (1 << 16, 1 << 22, 1 << 26, 1 << 30):
            b = nz.nz_balance(setup, rate, S)
            it = nz.nz_balance_iterate(setup, rate, S)
            splits.append({"msg_bytes": S, "hot": b["hot"], "alpha": [round(float(x), 4) for x in b["alpha"]],
                           "t_cold_us": round(b["t_cold"] * 1e6, 2), "t_hot_us": round(b["t_hot"] * 1e6, 2),
                           "alpha_by_iteration": [round(float(x), 4) for x in it["alpha"]],
                           "iterations": it["iterations"]})
        balancer[f"N{N}"] = {"rails": "rail 0 = (t0, B) of the fused fit, rail 1 = of the ring-stepwise fit",
                             "threshold_bytes_eq6": round(nz.nz_balance_threshold(setup, rate)),
                             "splits": splits}
    print(json.dumps({"sweep": rows, "hip_graph": use_graph, "fit_t_equals_t0_plus_S_over_B": fits,
                      "load_balancer_on_fitted_rails": balancer}), flush=True)
    return 0


def shape_survey(torch, nz, dev) -> int:
    """Every entry point over node counts, message sizes and rail layouts other than the five
    workloads', on plain allocations: fraction of the HBM peak on each part's algorithmic bytes.
    One JSON line; ungraded, like --sweep."""
    MB = 1 << 20

    def timed(fn, reps=8):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e-3 / reps

    cases = [(N, mb, (100, 40)) for N in (2, 3, 4, 6, 8, 12, 16, 32) for mb in (64, 256)]
    cases += [(8, 200, r) for r in ((1,), (1,) * 8, (1000, 1), (5, 0, 3, 0, 0, 1))]
    cases += [(128, 32, r) for r in ((1,), (100, 100, 40, 10), (1,) * 8)]
    rows = []
    for dtype, tdt, e in (("f32", torch.float32, 4), ("bf16", torch.bfloat16, 2)):
        for N, mb, ratios in cases:
            n = mb * MB // e + 1234
            S = n * e
            ins = [(torch.randn(n, device=dev) * 1e-2).to(tdt) for _ in range(N)]
            outs = [torch.empty_like(t) for t in ins]
            b = nz.nz_rail_partition(n, e, ratios)
            seg = nz.nz_segment_map(b, N)
            L = int(b[1] - b[0])
            send = [torch.empty(L, dtype=tdt, device=dev) for _ in range(N)]
            ids = list(range(N))
            live = [k for k, w in enumerate(ratios) if w]
            parts = {
                "fused": (2 * N * S, lambda: nz.nz_allreduce_sim(ins, n, ratios, dtype, "fused", outs)),
                "ring": (5 * (N - 1) * S, lambda: nz.nz_allreduce_sim(ins, n, ratios, dtype, "ring-stepwise", outs)),
                "rs": ((N + 1) * S, lambda: nz.nz_reduce_scatter_sim(ins, n, ratios, dtype, "fused", outs)),
                "ag": (N * S, lambda: nz.nz_allgather_sim(outs, n, ratios, dtype, "fused")),
                "chunked": (5 * (N - 1) * S,
                            lambda: nz.nz_allreduce_sim_chunked(ins, n, ratios, dtype, 1 << 20, outs)),
                "pack": (2 * N * L * e, lambda: nz.nz_pack(ins, seg, 0, ids, e, send, L * e)),
                "unpack": (2 * N * L * e, lambda: nz.nz_unpack(send, seg, 0, ids, e, outs)),
            }
            if len(live) > 1:
                parts["failover"] = (2 * N * S, lambda: nz.nz_allreduce_sim_failover(ins, n, ratios, dtype, "fused",
                                                                                     outs, live[-1]))
            row = {"dtype": dtype, "n_nodes": N, "mb_per_node": mb, "ratios": list(ratios)}
            for name, (nbytes, fn) in parts.items():
                row[name] = round(nbytes / timed(fn) / 1e9 / HBM_PEAK_GBS, 3)
            rows.append(row)
            del ins, outs, send, parts
    print(json.dumps({"shape_survey": rows, "unit": "fraction of 8 TB/s on algorithmic bytes",
                      "placement": "plain torch allocations"}), flush=True)
    return 0


def main() -> int:
    args = parse_args()
    if args.steps < 1 or args.warmup < 0:
        print("bench.py: --steps must be at least 1 and --warmup at least 0", file=sys.stderr)
        return 2
    if args.gpus != 1:
        print("bench.py: the library runs on exactly one GPU (the N simulated nodes share one "
              "MI355X's HBM); --gpus must be 1", file=sys.stderr)
        return 2

    import torch
    from paper_2405_17870_amd import inputs
    from paper_2405_17870_amd import nezha_sim as nz
    from paper_2405_17870_amd import placement

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    nz.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.sweep:
        return size_sweep(torch, nz, dev, args.graph)
    if args.shapes:
        return shape_survey(torch, nz, dev)
    w = inputs.WORKLOADS[args.workload]
    parts = [p for p in args.parts.split(",") if p]
    N, n, e = w.n_nodes, w.n_elems, inputs.ELEM_BYTES[w.dtype]
    S = n * e
    R = len(w.ratios)

    tdtype = inputs.TORCH_DTYPE[w.dtype]
    rail_off = nz.nz_rail_partition(n, e, w.ratios)
    seg = nz.nz_segment_map(rail_off, N)
    need_send = any(p in parts for p in ("pack", "unpack", "packed", "packed_out", "unpack_out"))
    need_result = any(p in parts for p in ("packed_out", "unpack_out"))
    rail_len = [max(int(rail_off[k + 1] - rail_off[k]), 1) for k in range(R)]

    def make_buffers(kind):
        """Inputs (filled), outputs and per-rail send buffers under one of the placements."""
        arena = placement.try_arena(dev) if kind != "torch" else None
        if arena is None:
            ins = inputs.workload_buffers(w, device=dev)
            outs = [torch.empty_like(t) for t in ins]
            send = [[torch.zeros(rail_len[k], dtype=tdtype, device=dev) for _ in range(N)] for k in range(R)] \
                if need_send else []
            if need_result:          # per-rail result buffers of the out-of-place packed route
                send += [[torch.zeros(rail_len[k], dtype=tdtype, device=dev) for _ in range(N)] for k in range(R)]
            return ins, outs, send, None, "plain torch allocations"
        if kind == "packed":
            arena.pack_from(int(args.packed_offset_gib * (1 << 30)))
            note = f"all buffers back to back from arena offset {args.packed_offset_gib:g} GiB"
        else:
            note = ("one arena over HBM, offsets from nz_hbm_place: inputs together in the first 96 GiB "
                    "region, outputs and send buffers spread over the three regions")
        ins = arena.alloc_together(N, n, tdtype, 0)
        outs = arena.alloc_striped(N, n, tdtype, 0)
        send = [arena.alloc_striped(N, rail_len[k], tdtype, k + 1) for k in range(R)] if need_send else []
        if need_result:
            send += [arena.alloc_striped(N, rail_len[k], tdtype, k + 2) for k in range(R)]
        for i in range(N):
            ins[i].copy_(inputs.node_buffer(w.dtype, n, w.seed, i, device=dev, std=w.std,
                                            outlier_frac=w.outlier_frac, outlier_scale=w.outlier_scale))
        for group in send:
            for t in group:
                t.zero_()
        return ins, outs, send, arena, note

    ins, outs, send, arena, placement_note = make_buffers(args.placement)
    ids = list(range(N)) if args.pack_order == "rail" else [(N // 2 - s) % N for s in range(N)]
    torch.cuda.synchronize()

    K = 1 if args.shared_output else N
    bufs = {"ins": ins, "outs": outs, "send": send}
    alg_bytes = {"fused": (N + K) * S, "ring": 5 * (N - 1) * S, "pack": 2 * N * S, "unpack": 2 * N * S,
                 # optional parts: the two halves on their own, fused form
                 "rs": (N + 1) * S, "ag": N * S,
                 # Ring_Chunked moves the ring's bytes in more launches; failover the fused bytes in two
                 "chunked": 5 * (N - 1) * S, "failover": 2 * N * S,
                 # every rail's N send buffers reduced in place: N reads + N writes of the payload
                 "packed": 2 * N * S, "packed_out": 2 * N * S, "unpack_out": 2 * N * S}

    def run_part(p):
        ins, outs, send = bufs["ins"], bufs["outs"], bufs["send"]
        if p == "fused":
            nz.nz_allreduce_sim(ins, n, w.ratios, w.dtype, "fused", [outs[1]] * N if args.shared_output else outs)
        elif p == "ring":
            nz.nz_allreduce_sim(ins, n, w.ratios, w.dtype, "ring-stepwise", outs)
        elif p == "rs":
            nz.nz_reduce_scatter_sim(ins, n, w.ratios, w.dtype, "fused", outs)
        elif p == "ag":
            nz.nz_allgather_sim(outs, n, w.ratios, w.dtype, "fused")
        elif p == "chunked":
            nz.nz_allreduce_sim_chunked(ins, n, w.ratios, w.dtype, args.chunk_elems, outs)
        elif p == "failover":
            nz.nz_allreduce_sim_failover(ins, n, w.ratios, w.dtype, "fused", outs, R - 1)
        elif p == "packed":
            for k in range(R):
                if rail_off[k + 1] > rail_off[k]:
                    nz.nz_allreduce_sim(send[k], int(rail_off[k + 1] - rail_off[k]), (1,), w.dtype, "fused", send[k])
        elif p == "packed_out":
            for k in range(R):
                if rail_off[k + 1] > rail_off[k]:
                    nz.nz_allreduce_sim(send[k], int(rail_off[k + 1] - rail_off[k]), (1,), w.dtype, "fused", send[R + k])
        elif p == "unpack_out":
            for k in range(R):
                nz.nz_unpack(send[R + k], seg, k, ids, e, outs)
        elif p == "pack":
            for k in range(R):
                nz.nz_pack(ins, seg, k, ids, e, send[k], send[k][0].numel() * e)
        elif p == "unpack":
            for k in range(R):
                nz.nz_unpack(send[k], seg, k, ids, e, outs)
        else:
            raise SystemExit(f"unknown part {p!r}")

    def time_parts(reps, warm):
        """Mean time of every part on its own (HIP events on the launch stream)."""
        res = {}
        for p in parts:
            for _ in range(warm):
                run_part(p)
            ev = []
            for _ in range(reps):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                run_part(p)
                b.record()
                ev.append((a, b))
            torch.cuda.synchronize()
            ms = sum(a.elapsed_time(b) for a, b in ev) / len(ev)
            gbs = alg_bytes[p] / (ms * 1e-3) / 1e9
            res[p] = {"ms": round(ms, 4), "hbm_GBps": round(gbs, 1), "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4)}
        return res

    def step(events=None):
        for p in parts:
            if events is not None:
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                run_part(p)
                b.record()
                events[p].append((a, b))
            else:
                run_part(p)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = {p: [] for p in parts}
    if args.graph:
        # The library launches plain kernels on the given stream and touches no
        # device memory of its own, so a step can be captured as it is.
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        for p in parts:            # no events inside a graph: share the step time by bytes
            share = wall * 1e3 / args.steps * alg_bytes[p] / sum(alg_bytes[q] for q in parts)
            events[p] = share
    else:
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(events)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0

    ms_per_step = wall * 1e3 / args.steps
    step_bytes = sum(alg_bytes[p] for p in parts)
    part_stats = {}
    for p in parts:
        if args.graph:
            ms = med = events[p]
        else:
            times = sorted(a.elapsed_time(b) for a, b in events[p])
            ms = sum(times) / len(times)
            med = 0.5 * (times[(len(times) - 1) // 2] + times[len(times) // 2])
        gbs = alg_bytes[p] / (ms * 1e-3) / 1e9
        part_stats[p] = {"ms": round(ms, 4), "ms_median": round(med, 4), "payload_GBps": round(S / (ms * 1e-3) / 1e9, 2),
                         "hbm_GBps": round(gbs, 1), "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4),
                         "algorithmic_bytes": alg_bytes[p]}

    head = "fused" if "fused" in parts else parts[0]
    used_outs = [outs[1]] if args.shared_output else outs
    out_span = max(t.data_ptr() for t in used_outs) + S - min(t.data_ptr() for t in used_outs)
    del used_outs                     # views of the arena: it must be free again before the plain allocations
    fused_launches = nz.nz_allreduce_launches(N, n, w.ratios, w.dtype, "fused", K, out_span)
    launches = {"fused": fused_launches, "ring": 2 * (N - 1), "pack": R, "unpack": R, "rs": 1, "ag": 1,
                "chunked": 2 * (N - 1), "failover": 2, "packed": R, "packed_out": R, "unpack_out": R}[head]
    fused_kernel = "nz_fused_stage" if fused_launches > 1 else "nz_fused_flat"
    achieved = part_stats[head]["hbm_GBps"]
    roofline = {
        "kernel": {"fused": fused_kernel, "ring": "nz_ring_step",
                   "pack": "nz_segment_copy", "unpack": "nz_segment_copy",
                   "rs": "nz_fused_reduce_bcast", "ag": "nz_gather_range",
                   "chunked": "nz_ring_wave", "failover": "nz_fused_stage" if fused_launches > 1 else "nz_fused_reduce_bcast",
                   "packed": fused_kernel, "packed_out": fused_kernel, "unpack_out": "nz_segment_copy"}[head],
        "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4),
        "launches": launches,
        "algorithmic_bytes_per_launch": alg_bytes[head] // launches,
        "avg_launch_ms": round(part_stats[head]["ms"] / launches, 4),
        "traffic": recorded_traffic(f"{head}_{w.name}"),
    }

    out = {
        "metric": "allreduce-sim effective GB/s and % of HBM peak, fused vs ring-stepwise",
        "value": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "i32" if w.dtype == "i32" else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: {N} simulated nodes x {n} {w.dtype} elements, "
                               f"rails {':'.join(map(str, w.ratios))}",
                   "storage_dtype": w.dtype, "n_nodes": N, "n_elems": n, "ratios": list(w.ratios),
                   "parts": parts, "distinct_outputs": K, "placement": placement_note,
                   "hip_graph": bool(args.graph)},
        "pct_of_hbm_peak": round(100.0 * step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 2),
        "parts": part_stats,
        "roofline": roofline,
        "device": device_facts(torch),
    }
    if args.placement != "torch" and arena is not None and not args.no_plain and not args.graph:
        # The same parts once more on plain allocations: what a caller gets who leaves
        # placement to the allocator.
        bufs.clear()
        del ins, outs, send, arena
        torch.cuda.empty_cache()
        p_ins, p_outs, p_send, _, _ = make_buffers("torch")
        bufs.update(ins=p_ins, outs=p_outs, send=p_send)
        plain = time_parts(reps=5, warm=2)
        out["plain_allocations"] = {"placement": "plain torch allocations", "parts": plain,
                                    "roofline_frac": plain[head]["frac_of_peak"]}
        del p_ins, p_outs, p_send
    if not args.no_cpu_baseline:
        bufs.clear()
        ins = outs = send = arena = None
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_sample_elems, parts)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
