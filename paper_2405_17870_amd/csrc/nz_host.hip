// Host side of the allreduce reduction engine: argument validation, rail and
// segment geometry for the kernels, launches, and the C-ABI entry points that
// run on the GPU (see include/nezha_sim.h; the kernels are in nz_device.h).
//
// Nezha (arXiv 2405.17870): Sec. 4.2 (allreduce over rails), Sec. 2.1.1 / Eq. 1
// (ring schedule, its two halves, Ring_Chunked in the evaluation), Sec. 4.4
// (failover), Sec. 3.2 (pack / unpack).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <utility>

#include "nz_device.h"

namespace {

thread_local char g_hip_error[256] = "";

nz_status hip_failed(hipError_t e, const char *what)
{
    std::snprintf(g_hip_error, sizeof g_hip_error, "%s: %s", what, hipGetErrorString(e));
    return NZ_ERR_HIP;
}

// Launch a kernel whose only parameter is its argument struct and return the
// launch's own status (hipGetLastError could hand back an older error that
// some other code of the process left behind).
template <class Args>
hipError_t launch(void (*kernel)(const Args), u32 blocks, const Args &args, hipStream_t st)
{
    void *params[] = {const_cast<Args *>(&args)};
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), dim3(blocks), dim3(kThreads), params, 0, st);
}

// Debugging aid: with NZ_DEBUG set to anything but "" or "0" in the environment
// (looked up at every call), an entry point waits for its stream before it
// returns, so a failure during execution is reported by the call that caused it.
bool debug_sync_enabled()
{
    const char *v = std::getenv("NZ_DEBUG");
    return v != nullptr && v[0] != '\0' && std::strcmp(v, "0") != 0;
}

nz_status finish(nz_status s, hipStream_t st)
{
    if (s != NZ_OK || !debug_sync_enabled()) return s;
    const hipError_t e = hipStreamSynchronize(st);
    return e == hipSuccess ? NZ_OK : hip_failed(e, "execution (NZ_DEBUG wait)");
}

bool aligned256(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }

constexpr u64 kNothingToDo = UINT64_MAX;  // every selected rail is empty

// Fill the geometry for tiles of tile_vecs 16-byte vectors.  rail_mask selects
// the rails that take part (bit k = rail k); piece_elems < UINT64_MAX makes the
// launch work on pieces of that many elements of every segment.  Returns the
// number of workgroups, kNothingToDo if there is no element to work on, or 0 if
// the work does not fit a grid.
u64 build_geometry(RailGeom &g, const u64 *rail_off, u32 n_rails, u32 n_nodes, u32 elem_shift,
                   u32 tile_vecs, u32 rail_mask = 0xffffffffu, u64 piece_elems = UINT64_MAX)
{
    std::memset(&g, 0, sizeof g);
    g.n_rails = n_rails;
    g.n_nodes = n_nodes;
    g.win_off = 0;
    g.win_len = piece_elems;
    u64 total = 0;
    for (u32 k = 0; k < n_rails; ++k) {
        // A rail left out of this launch keeps its place but has no elements.
        const u64 len = (rail_mask >> k & 1u) ? rail_off[k + 1] - rail_off[k] : 0;
        g.off[k] = rail_off[k];
        g.q[k] = len / n_nodes;
        g.rem[k] = (u32)(len % n_nodes);
        u64 most = 0;
        if (piece_elems != UINT64_MAX && len > 0) {
            // Pieces start anywhere: bound the tiles a piece can touch.
            const u64 longest = std::min<u64>(g.q[k] + (g.rem[k] ? 1 : 0), piece_elems);
            const u64 vecs = ((longest << elem_shift) + 15) / 16 + 1;
            most = longest ? (vecs + tile_vecs - 1) / tile_vecs + 1 : 0;
        } else {
            // Exact maximum, over the rail's segments, of the tiles a segment touches.
            for (u32 j = 0; j < n_nodes && len > 0; ++j) {
                const u64 beg = g.off[k] + j * g.q[k] + std::min<u64>(j, g.rem[k]);
                const u64 sl = g.q[k] + (j < g.rem[k] ? 1 : 0);
                if (sl == 0) continue;
                const u64 v0 = (beg << elem_shift) >> 4;
                const u64 v1 = (((beg + sl) << elem_shift) + 15) >> 4;
                most = std::max<u64>(most, (v1 - 1) / tile_vecs - v0 / tile_vecs + 1);
            }
        }
        if (most > 0xffffffffull) return 0;
        g.tps[k] = (u32)most;
        g.tile0[k] = (u32)total;
        total += most * n_nodes;
        if (total > 0x7fffffffull) return 0;
    }
    g.off[n_rails] = rail_off[n_rails];
    g.tile0[n_rails] = (u32)total;
    return total == 0 ? kNothingToDo : total;
}

// Bytes a single-launch fused call moves up to which it uses cache-allocating
// accesses (half of the 256 MB last-level cache): a job of that size finds its
// inputs in cache and leaves its results there for whoever reads them next.
constexpr u64 kFusedCachedBytes = 128ull << 20;

template <class T, bool CACHED>
hipError_t launch_fused_class(const FusedArgs &a, u32 blocks, hipStream_t st)
{
    return a.g.n_nodes <= 8    ? launch(nz_fused_reduce_bcast<T, kUpTo8, CACHED>, blocks, a, st)
           : a.g.n_nodes <= 32 ? launch(nz_fused_reduce_bcast<T, kUpTo32, CACHED>, blocks, a, st)
                               : launch(nz_fused_reduce_bcast<T, kAnyN, CACHED>, blocks, a, st);
}

// moved_bytes: what the launch reads and writes.
template <class T>
nz_status launch_fused(const FusedArgs &a, u32 blocks, hipStream_t st, u64 moved_bytes)
{
    const hipError_t e = moved_bytes <= kFusedCachedBytes ? launch_fused_class<T, true>(a, blocks, st)
                                                          : launch_fused_class<T, false>(a, blocks, st);
    return e == hipSuccess ? NZ_OK : hip_failed(e, "fused reduce launch");
}

// Vectors per thread of the whole-message fused kernel for a job that runs out
// of the last-level cache: a thread should have about eight loads of its own in
// flight, which the blocked sum provides from five nodes on.  (A job that
// streams from HBM gains nothing from more: measured 1 to 3 % slower.)
#ifndef NZ_FUSED_VPT_UPTO2
#define NZ_FUSED_VPT_UPTO2 4
#endif
#ifndef NZ_FUSED_VPT_UPTO4
#define NZ_FUSED_VPT_UPTO4 2
#endif
#ifndef NZ_FUSED_VPT_MIN_BLOCKS
#define NZ_FUSED_VPT_MIN_BLOCKS 2048  // eight workgroups per compute unit
#endif
// A small job keeps small tiles so that it still spreads over the whole chip.
u32 fused_vpt(u32 n_nodes, u64 bytes, bool cached)
{
    if (!cached) return 1;
    u32 vpt = n_nodes <= 2 ? NZ_FUSED_VPT_UPTO2 : n_nodes <= 4 ? NZ_FUSED_VPT_UPTO4 : 1;
    while (vpt > 1 && bytes / ((u64)vpt * kThreads * 16) < NZ_FUSED_VPT_MIN_BLOCKS) vpt >>= 1;
    return vpt;
}

template <class T, bool CACHED>
hipError_t launch_flat_class(const FlatArgs &a, u32 blocks, hipStream_t st)
{
    return a.n_nodes <= 8    ? launch(nz_fused_flat<T, kUpTo8, CACHED, 1>, blocks, a, st)
           : a.n_nodes <= 32 ? launch(nz_fused_flat<T, kUpTo32, CACHED, 1>, blocks, a, st)
                             : launch(nz_fused_flat<T, kAnyN, CACHED, 1>, blocks, a, st);
}

// The allreduce over the whole message in one launch.
template <class T>
nz_status launch_flat(const FlatArgs &a, hipStream_t st)
{
    const bool cached = a.bytes * (a.n_nodes + a.n_out) <= kFusedCachedBytes;
    const u32 vpt = fused_vpt(a.n_nodes, a.bytes, cached);
    const u64 tile_bytes = (u64)vpt * kThreads * 16;
    const u64 blocks = (a.bytes + tile_bytes - 1) / tile_bytes;
    if (blocks > 0x7fffffffull) return NZ_ERR_UNSUPPORTED;
    const hipError_t e = vpt == 4   ? launch(nz_fused_flat<T, kUpTo8, true, 4>, (u32)blocks, a, st)
                         : vpt == 2 ? launch(nz_fused_flat<T, kUpTo8, true, 2>, (u32)blocks, a, st)
                         : cached   ? launch_flat_class<T, true>(a, (u32)blocks, st)
                                    : launch_flat_class<T, false>(a, (u32)blocks, st);
    return e == hipSuccess ? NZ_OK : hip_failed(e, "fused reduce launch");
}

// The fused allreduce is issued as the staged pipeline (see nz_fused_stage)
// from this payload per node, ...
#ifndef NZ_STAGE_MIN_BYTES
#define NZ_STAGE_MIN_BYTES (1ull << 20)
#endif
constexpr u64 kStageMinBytes = NZ_STAGE_MIN_BYTES;
// ... this many bytes written to all outputs together (measured on plain
// allocations: 32 outputs win from 4 MB per node, 8 outputs from 16 MB) ...
#ifndef NZ_STAGE_MIN_OUTPUT_BYTES
#define NZ_STAGE_MIN_OUTPUT_BYTES (128ull << 20)
#endif
constexpr u64 kStageMinOutputBytes = NZ_STAGE_MIN_OUTPUT_BYTES;
// ... and this many distinct outputs: staging costs one more read of the
// result, 1 / (N + K) of the traffic, which few write streams do not repay
// (measured: 2 to 4 outputs lose 3 to 20 %, 6 break even, 8 gain 7 %).
#ifndef NZ_STAGE_MIN_OUTPUTS
#define NZ_STAGE_MIN_OUTPUTS 7
#endif
constexpr u32 kStageMinOutputs = NZ_STAGE_MIN_OUTPUTS;
// Output buffers that span more than the length of a memory region (see
// nz_hbm_place) cannot all lie in one region.  Write streams spread over
// regions are much less of a burden: the single launch then runs at 80-83 % of
// peak whatever the number of outputs, which the pipeline only passes with
// many of them (73 % with 7, 75 % with 8, 78 % with 12, 79 % with 16, 83 % with
// 24 to 32, 85-86 % with 32 to 128 large ones).
#ifndef NZ_STAGE_MIN_SPREAD_OUTPUTS
#define NZ_STAGE_MIN_SPREAD_OUTPUTS 17
#endif
constexpr u32 kStageMinSpreadOutputs = NZ_STAGE_MIN_SPREAD_OUTPUTS;
// out_span: bytes from the start of the lowest distinct output buffer to the
// end of the highest.
bool staged_allreduce(u32 n_out, u64 active_bytes, u64 out_span)
{
    const u32 min_outputs = out_span > NZ_HBM_REGION_BYTES ? kStageMinSpreadOutputs : kStageMinOutputs;
    return n_out >= min_outputs && active_bytes >= kStageMinBytes && active_bytes * n_out >= kStageMinOutputBytes;
}

u64 round_up(u64 x, u64 m) { return (x + m - 1) / m * m; }

// A span of `span` bytes is cut into equal pieces of at most kStagePieceBytes,
// each a whole number of 4 KB tiles.
u64 stage_piece_bytes(u64 span)
{
    const u64 n_pieces = (span + kStagePieceBytes - 1) / kStagePieceBytes;
    return round_up((span + n_pieces - 1) / n_pieces, (u64)kThreads * 16);
}

template <class T>
nz_status launch_stage(StageArgs &a, hipStream_t st)
{
    constexpr u64 kTileBytes = (u64)kThreads * 16;
    const u64 n_a = round_up((a.a_hi - a.a_lo + kTileBytes - 1) / kTileBytes, 8);
    const u64 b_tiles =
        round_up((a.b_hi - a.b_lo + kStageCopyIters * kTileBytes - 1) / (kStageCopyIters * kTileBytes), 8);
    const u64 blocks = n_a + b_tiles * (a.n_out - 1);
    if (blocks == 0) return NZ_OK;
    if (blocks > 0x7fffffffull) return NZ_ERR_UNSUPPORTED;
    a.n_a_blocks = (u32)n_a;
    a.b_tiles = (u32)b_tiles;
    const hipError_t e = a.n_nodes <= 8    ? launch(nz_fused_stage<T, kUpTo8>, (u32)blocks, a, st)
                         : a.n_nodes <= 32 ? launch(nz_fused_stage<T, kUpTo32>, (u32)blocks, a, st)
                                           : launch(nz_fused_stage<T, kAnyN>, (u32)blocks, a, st);
    return e == hipSuccess ? NZ_OK : hip_failed(e, "staged fused launch");
}

// The staged pipeline over the participating rails: neighbouring rails form
// one span of bytes; a span is cut into equal pieces of at most
// kStagePieceBytes; launch c reduces piece c and spreads piece c - 1.
template <class T>
nz_status launch_staged(StageArgs &a, const u64 *rail_off, u32 n_rails, u32 rail_mask, u32 elem_shift,
                        hipStream_t st)
{
    // More pieces than any memory holds: refuse before anything is launched.
    if ((rail_off[n_rails] << elem_shift) / kStagePieceBytes > (1u << 16)) return NZ_ERR_UNSUPPORTED;
    u64 spread_lo = 0, spread_hi = 0;  // the piece the next launch spreads
    u32 k = 0;
    while (k < n_rails) {
        if (!(rail_mask >> k & 1u) || rail_off[k + 1] == rail_off[k]) {
            ++k;
            continue;
        }
        u32 end = k + 1;
        while (end < n_rails && (rail_mask >> end & 1u)) ++end;
        const u64 lo = rail_off[k] << elem_shift, hi = rail_off[end] << elem_shift;
        k = end;
        if (hi == lo) continue;
        const u64 piece = stage_piece_bytes(hi - lo);
        for (u64 p = lo; p < hi; p += piece) {
            a.a_lo = p;
            a.a_hi = std::min(hi, p + piece);
            a.b_lo = spread_lo;
            a.b_hi = spread_hi;
            const nz_status ls = launch_stage<T>(a, st);
            if (ls != NZ_OK) return ls;
            spread_lo = a.a_lo;
            spread_hi = a.a_hi;
        }
    }
    a.a_lo = a.a_hi = 0;
    a.b_lo = spread_lo;
    a.b_hi = spread_hi;
    return launch_stage<T>(a, st);
}

#ifndef NZ_RING_ITERS
#define NZ_RING_ITERS 1
#endif
constexpr int kRingIters = NZ_RING_ITERS;
#ifndef NZ_GATHER_ITERS
#define NZ_GATHER_ITERS 4
#endif
constexpr int kGatherIters = NZ_GATHER_ITERS;

enum Collective { kAllreduce, kReduceScatter, kAllgather };

// Bytes of one ring step up to which the step's output is kept in cache for
// the next step to read (half of the 256 MB last-level cache).
#ifndef NZ_RING_REUSE_BYTES
#define NZ_RING_REUSE_BYTES (128ull << 20)
#endif
constexpr u64 kRingReuseBytes = NZ_RING_REUSE_BYTES;

// The launches of a ring: N - 1 reduce-scatter steps, then N - 1 allgather
// steps (one half only for the phase collectives), each over whole segments.
template <class T, bool REUSE>
nz_status launch_ring_steps(RingArgs &a, u32 blocks, hipStream_t st, Collective what)
{
    const u32 N = a.g.n_nodes;
    for (u32 s = 0; s + 1 < N && what != kAllgather; ++s) {
        a.step = s;
        const hipError_t e = launch(nz_ring_step<T, kRingIters, false, REUSE>, blocks, a, st);
        if (e != hipSuccess) return hip_failed(e, "ring reduce-scatter launch");
    }
    for (u32 s = 0; s + 1 < N && what != kReduceScatter; ++s) {
        a.step = s;
        const hipError_t e = launch(nz_ring_step<T, kRingIters, true, REUSE>, blocks, a, st);
        if (e != hipSuccess) return hip_failed(e, "ring allgather launch");
    }
    return NZ_OK;
}

// Ring_Chunked: n_pieces pieces of a.g.win_len elements of every segment, each
// going through the 2 (N - 1) steps; launch w carries step w - c of every
// piece c that has such a step (see nz_ring_wave): n_pieces + 2 (N - 1) - 1
// launches, each piece one step behind the piece before it.
template <class T, bool REUSE>
nz_status launch_ring_pipeline(const RingArgs &a, hipStream_t st, u64 n_pieces)
{
    RingWaveArgs w;
    std::memset(&w, 0, sizeof w);
    w.ring = a;
    const u32 R = a.g.n_rails, N = a.g.n_nodes;
    const u64 n_steps = 2ull * (N - 1);
    u64 rail_pieces[NZ_MAX_RAILS];  // a rail with shorter segments has fewer pieces
    constexpr u64 kTileVecs = (u64)kRingIters * kThreads;
    for (u32 k = 0; k < R; ++k) {
        const u64 longest = a.g.q[k] + (a.g.rem[k] ? 1 : 0);
        rail_pieces[k] = (longest + a.g.win_len - 1) / a.g.win_len;
        w.last_piece[k] = 0;
        w.tps_last[k] = 1;
        if (rail_pieces[k] == 0) continue;
        // The last piece is as long as what the others leave; the tiles it can touch are
        // bounded as build_geometry bounds those of a full piece.
        const u64 last_len = longest - (rail_pieces[k] - 1) * a.g.win_len;
        const u64 vecs = ((last_len << a.elem_shift) + 15) / 16 + 1;
        w.last_piece[k] = (u32)(rail_pieces[k] - 1);
        w.tps_last[k] = (u32)std::min<u64>((vecs + kTileVecs - 1) / kTileVecs + 1, a.g.tps[k]);
    }
    // Sizes first: nothing is launched if a launch would not fit a grid.
    for (int pass = 0; pass < 2; ++pass) {
        for (u64 wave = 0; wave + 1 < n_pieces + n_steps; ++wave) {
            u64 blocks = 0;
            for (u32 k = 0; k < R; ++k) {
                const u64 lo = wave >= n_steps ? wave - n_steps + 1 : 0;  // first piece still on its way
                const u64 started = std::min<u64>(wave + 1, rail_pieces[k]);  // pieces 0 .. started - 1 have begun
                w.piece_lo[k] = (u32)lo;
                w.block0[k] = (u32)blocks;
                w.full_blocks[k] = 0;
                if (started > lo) {
                    const bool has_last = started == rail_pieces[k];
                    const u64 full = (started - lo - (has_last ? 1 : 0)) * N * a.g.tps[k];
                    blocks += full + (has_last ? (u64)N * w.tps_last[k] : 0);
                    if (blocks > 0x7fffffffull) return NZ_ERR_UNSUPPORTED;
                    w.full_blocks[k] = (u32)full;
                }
            }
            w.block0[R] = (u32)blocks;
            if (pass == 0 || blocks == 0) continue;
            w.wave = (u32)wave;
            const hipError_t e = launch(nz_ring_wave<T, kRingIters, REUSE>, (u32)blocks, w, st);
            if (e != hipSuccess) return hip_failed(e, "chunked ring launch");
        }
    }
    return NZ_OK;
}

// Bytes one launch stores: every node's piece (or whole segment) of every rail.
u64 ring_launch_bytes(const RingArgs &a)
{
    u64 elems = 0;
    for (u32 k = 0; k < a.g.n_rails; ++k) {
        const u64 longest = a.g.q[k] + (a.g.rem[k] ? 1 : 0);
        elems += (u64)a.g.n_nodes * std::min<u64>(longest, a.g.win_len);
    }
    return elems << a.elem_shift;
}

template <class T>
nz_status launch_ring(RingArgs &a, u32 blocks, hipStream_t st, Collective what, u64 n_pieces)
{
    if (n_pieces > 1) {
        // What one launch stores: up to min(pieces, steps) piece-steps.
        const u64 in_flight = std::min<u64>(n_pieces, 2ull * (a.g.n_nodes - 1));
        return ring_launch_bytes(a) * in_flight <= kRingReuseBytes
                   ? launch_ring_pipeline<T, true>(a, st, n_pieces)
                   : launch_ring_pipeline<T, false>(a, st, n_pieces);
    }
    return ring_launch_bytes(a) <= kRingReuseBytes ? launch_ring_steps<T, true>(a, blocks, st, what)
                                                   : launch_ring_steps<T, false>(a, blocks, st, what);
}

template <class T>
nz_status launch_gather(const GatherArgs &a, u32 blocks, hipStream_t st)
{
    const hipError_t e = launch(nz_gather_bcast<T, kGatherIters>, blocks, a, st);
    return e == hipSuccess ? NZ_OK : hip_failed(e, "direct allgather launch");
}

template <class T>
nz_status launch_gather_range(const GatherRangeArgs &a, u32 blocks, hipStream_t st)
{
    const hipError_t e = launch(nz_gather_range<T, kGatherIters>, blocks, a, st);
    return e == hipSuccess ? NZ_OK : hip_failed(e, "direct allgather launch");
}

// Geometry of the direct allgather one destination at a time: per rail pieces
// x N destinations x tiles.  Rails whose segments are shorter than a tile are
// not for this kernel: they get no workgroup here and their bits are returned
// in *short_rails.  Returns the number of workgroups (as build_geometry).
u64 build_gather_ranges(GatherRangeArgs &a, const u64 *rail_off, u32 n_rails, u32 n_nodes, u32 elem_shift,
                        u32 tile_vecs, u32 rail_mask, u32 *short_rails)
{
    std::memset(&a.g, 0, sizeof a.g);
    RailGeom &g = a.g;
    g.n_rails = n_rails;
    g.n_nodes = n_nodes;
    const u64 tile_bytes = (u64)tile_vecs * 16;
    u64 total = 0;
    *short_rails = 0;
    for (u32 k = 0; k < n_rails; ++k) {
        // A rail left out of this launch keeps its place but gets no workgroup.
        const u64 len = (rail_mask >> k & 1u) ? rail_off[k + 1] - rail_off[k] : 0;
        g.off[k] = rail_off[k];
        g.q[k] = (rail_off[k + 1] - rail_off[k]) / n_nodes;
        g.rem[k] = (u32)((rail_off[k + 1] - rail_off[k]) % n_nodes);
        g.tile0[k] = (u32)total;
        a.pieces[k] = 0;
        g.tps[k] = 1;
        if (len == 0) continue;
        if ((g.q[k] << elem_shift) < tile_bytes) {
            *short_rails |= 1u << k;
            continue;
        }
        const u64 bytes = len << elem_shift;
        const u64 tps = round_up((stage_piece_bytes(bytes) + tile_bytes - 1) / tile_bytes, 8);
        const u64 pieces = (bytes + tps * tile_bytes - 1) / (tps * tile_bytes);
        if (pieces > 0xffffffffull) return 0;
        a.pieces[k] = (u32)pieces;
        g.tps[k] = (u32)tps;
        total += pieces * n_nodes * tps;
        if (total > 0x7fffffffull) return 0;
    }
    g.off[n_rails] = rail_off[n_rails];
    g.tile0[n_rails] = (u32)total;
    return total == 0 ? kNothingToDo : total;
}

// Pack / unpack launches.  Tiles of 8 KB per workgroup are best while a launch
// moves little, 4 KB tiles from about 2 GB on (measured on buffers that lie
// close together, 2 to 128 nodes: 8 KB tiles reach 80 % of peak below 1 GB and
// fall to 73 % at 4 GB and beyond, 4 KB tiles stay at 77 to 79 % throughout).
constexpr u64 kCopySmallTileBytes = 2ull << 30;
// Node index fastest only up to this many nodes (write streams at a time).
constexpr u32 kCopyInterleaveMaxNodes = 32;

nz_status segment_copy(const void *const *src, void *const *dst, u32 n_nodes, const u64 *seg_off,
                       u32 n_rails, u32 rail, const u32 *seg_ids, u32 n_segs, u32 elem_bytes,
                       bool packing, u64 capacity, u64 *packed_bytes, hipStream_t st)
{
    if (src == nullptr || dst == nullptr || seg_off == nullptr) return NZ_ERR_INVALID_ARG;
    if (n_nodes == 0 || n_rails == 0 || rail >= n_rails) return NZ_ERR_INVALID_ARG;
    if (n_segs > 0 && seg_ids == nullptr) return NZ_ERR_INVALID_ARG;
    if (elem_bytes != 2 && elem_bytes != 4) return NZ_ERR_INVALID_ARG;
    if (n_nodes > NZ_MAX_NODES || n_rails > NZ_MAX_RAILS || n_segs > NZ_MAX_NODES)
        return NZ_ERR_UNSUPPORTED;
    const u64 *row = seg_off + (size_t)rail * (n_nodes + 1);
    for (u32 j = 0; j < n_nodes; ++j)
        if (row[j + 1] < row[j] || row[j + 1] > (UINT64_MAX >> 3)) return NZ_ERR_INVALID_ARG;
    bool seen[NZ_MAX_NODES] = {};
    u64 total = 0;
    for (u32 i = 0; i < n_segs; ++i) {
        if (seg_ids[i] >= n_nodes) return NZ_ERR_INVALID_ARG;
        if (!packing) {
            if (seen[seg_ids[i]]) return NZ_ERR_INVALID_ARG;
            seen[seg_ids[i]] = true;
        }
        total += (row[seg_ids[i] + 1] - row[seg_ids[i]]) * elem_bytes;
    }
    if (packing && total > capacity) return NZ_ERR_CAPACITY;
    const u64 node_span_lo = row[0] * elem_bytes, node_span_hi = row[n_nodes] * elem_bytes;
    for (u32 m = 0; m < n_nodes; ++m) {
        if (src[m] == nullptr || dst[m] == nullptr) return NZ_ERR_INVALID_ARG;
        if (!aligned256(src[m]) || !aligned256(dst[m])) return NZ_ERR_ALIGNMENT;
    }
    // A written range may not overlap any other range.  The packed side of
    // buffer m is [base, base + total), the node side is the rail's span.
    if (total > 0) {
        const nz_status os = packing ? nz::check_copy_buffers(src, dst, n_nodes, node_span_lo, node_span_hi, 0, total)
                                     : nz::check_copy_buffers(src, dst, n_nodes, 0, total, node_span_lo, node_span_hi);
        if (os != NZ_OK) return os;
    }
    if (packed_bytes) *packed_bytes = total;
    if (total == 0) return NZ_OK;

    // Runs: consecutive list entries that are also consecutive in the node
    // buffer merge into one (a whole rail in order is a single run).
    struct Run { u64 node_off, pack_off, len; };
    Run runs[NZ_MAX_NODES];
    size_t n_runs = 0;
    u64 pos = 0;
    for (u32 i = 0; i < n_segs; ++i) {
        const u64 off = row[seg_ids[i]] * elem_bytes;
        const u64 len = (row[seg_ids[i] + 1] - row[seg_ids[i]]) * elem_bytes;
        if (len == 0) continue;
        if (n_runs > 0 && runs[n_runs - 1].node_off + runs[n_runs - 1].len == off)
            runs[n_runs - 1].len += len;
        else
            runs[n_runs++] = {off, pos, len};
        pos += len;
    }

    // Where the buffers lie decides the order of the workgroups (see nz_segment_copy).
    uintptr_t src_lo = UINTPTR_MAX, src_hi = 0, dst_lo = UINTPTR_MAX, dst_hi = 0;
    for (u32 m = 0; m < n_nodes; ++m) {
        const uintptr_t sp = reinterpret_cast<uintptr_t>(src[m]), dp = reinterpret_cast<uintptr_t>(dst[m]);
        src_lo = std::min(src_lo, sp);
        src_hi = std::max(src_hi, sp);
        dst_lo = std::min(dst_lo, dp);
        dst_hi = std::max(dst_hi, dp);
    }
    const bool interleave_nodes = n_nodes <= kCopyInterleaveMaxNodes && dst_hi - dst_lo > NZ_HBM_REGION_BYTES &&
                                  src_hi - src_lo <= NZ_HBM_REGION_BYTES;

    size_t next = 0;
    while (next < n_runs) {
        CopyArgs a;
        std::memset(&a, 0, sizeof a);
        a.elem_bytes = elem_bytes;
        a.node_major = interleave_nodes ? 0u : 1u;
        // The runs of this launch, and from their bytes the tile size.
        const size_t first = next, last = std::min(n_runs, next + (size_t)kCopyMaxRuns);
        u64 launch_bytes = 0;
        for (size_t i = first; i < last; ++i) launch_bytes += runs[i].len;
        const bool big_tiles = interleave_nodes || 2 * launch_bytes * n_nodes < kCopySmallTileBytes;
        const u64 TILE = (big_tiles ? 2u : 1u) * (u64)kThreads;
        u64 blocks = 0;
        u32 r = 0;
        for (; next < last; ++r, ++next) {
            const Run &run = runs[next];
            a.src_off[r] = packing ? run.node_off : run.pack_off;
            a.dst_off[r] = packing ? run.pack_off : run.node_off;
            a.len[r] = run.len;
            a.tile0[r] = (u32)blocks;
            const u64 v0 = a.dst_off[r] >> 4, v1 = (a.dst_off[r] + run.len + 15) >> 4;
            blocks += (v1 - 1) / TILE - v0 / TILE + 1;
            if (blocks * n_nodes > 0x7fffffffull) return NZ_ERR_UNSUPPORTED;
        }
        a.tile0[r] = (u32)blocks;
        a.n_runs = r;
        a.n_nodes = n_nodes;
        for (u32 m = 0; m < n_nodes; ++m) {
            a.src[m] = src[m];
            a.dst[m] = dst[m];
        }
        bool aligned = true;
        for (u32 i = 0; i < r; ++i) aligned = aligned && ((a.src_off[i] - a.dst_off[i]) & 15) == 0;
        const u32 grid = (u32)(blocks * n_nodes);
        const hipError_t e = aligned ? (big_tiles ? launch(nz_segment_copy<true, 2>, grid, a, st)
                                                  : launch(nz_segment_copy<true, 1>, grid, a, st))
                                     : (big_tiles ? launch(nz_segment_copy<false, 2>, grid, a, st)
                                                  : launch(nz_segment_copy<false, 1>, grid, a, st));
        if (e != hipSuccess) return hip_failed(e, "segment copy launch");
    }
    return NZ_OK;
}

// Common host side of the three collectives.  For kAllgather node_bufs and
// out_bufs are the same array: the operation is in place.
// rail_mask selects the rails a call works on (bit k = rail k); piece_elems is
// the Ring_Chunked piece length (UINT64_MAX: whole segments).
nz_status run_collective(Collective what, const void *const *node_bufs, uint32_t n_nodes, uint64_t n_elems,
                         const uint32_t *ratios, uint32_t n_rails, nz_dtype dtype, nz_mode mode,
                         void *const *out_bufs, hipStream_t st, u32 rail_mask = 0xffffffffu,
                         u64 piece_elems = UINT64_MAX)
{
    if (node_bufs == nullptr || out_bufs == nullptr || ratios == nullptr) return NZ_ERR_INVALID_ARG;
    if (n_nodes == 0 || n_rails == 0) return NZ_ERR_INVALID_ARG;
    const u32 eb = nz_dtype_bytes(dtype);
    if (eb == 0) return NZ_ERR_INVALID_ARG;
    if (mode != NZ_RING_STEPWISE && mode != NZ_FUSED) return NZ_ERR_INVALID_ARG;
    if (n_nodes > NZ_MAX_NODES || n_rails > NZ_MAX_RAILS) return NZ_ERR_UNSUPPORTED;

    u64 rail_off[NZ_MAX_RAILS + 1];
    const nz_status ps = nz::rail_partition(n_elems, eb, NZ_RAIL_ALIGN_BYTES, ratios, n_rails, rail_off);
    if (ps != NZ_OK) return ps;

    for (u32 i = 0; i < n_nodes; ++i) {
        if (node_bufs[i] == nullptr || out_bufs[i] == nullptr) return NZ_ERR_INVALID_ARG;
        if (!aligned256(node_bufs[i]) || !aligned256(out_bufs[i])) return NZ_ERR_ALIGNMENT;
    }
    const u64 bytes = n_elems * eb;
    {
        const nz_status os = nz::check_collective_buffers(node_bufs, out_bufs, n_nodes, bytes,
                                                          mode == NZ_RING_STEPWISE || what != kAllreduce);
        if (os != NZ_OK) return os;
    }
    if (n_elems == 0) return NZ_OK;

    const u32 shift = (eb == 4) ? 2 : 1;

    if (mode == NZ_FUSED && what == kAllgather) {
        if (n_nodes == 1) return NZ_OK;
        // One destination buffer at a time for the rails whose segments are at least a tile
        // long, all destinations at once for the others.  Both geometries are built before
        // anything is launched, so a refusal launches nothing.
        GatherRangeArgs ra;
        GatherArgs ga;
        u32 short_rails = 0;
        const u32 tile_vecs = (u32)kGatherIters * kThreads;
        const u64 range_blocks =
            build_gather_ranges(ra, rail_off, n_rails, n_nodes, shift, tile_vecs, rail_mask, &short_rails);
        if (range_blocks == 0) return NZ_ERR_UNSUPPORTED;
        u64 short_blocks = kNothingToDo;
        if (short_rails != 0) {
            short_blocks = build_geometry(ga.g, rail_off, n_rails, n_nodes, shift, tile_vecs, short_rails);
            if (short_blocks == 0) return NZ_ERR_UNSUPPORTED;
        }
        if (range_blocks != kNothingToDo) {
            for (u32 i = 0; i < n_nodes; ++i) ra.buf[i] = out_bufs[i];
            const nz_status s = eb == 4 ? launch_gather_range<TI32>(ra, (u32)range_blocks, st)
                                        : launch_gather_range<TBF16>(ra, (u32)range_blocks, st);
            if (s != NZ_OK) return s;
        }
        if (short_blocks != kNothingToDo) {
            for (u32 i = 0; i < n_nodes; ++i) ga.buf[i] = out_bufs[i];
            return eb == 4 ? launch_gather<TI32>(ga, (u32)short_blocks, st)
                           : launch_gather<TBF16>(ga, (u32)short_blocks, st);
        }
        return NZ_OK;
    }

    if (mode == NZ_FUSED) {
        FusedArgs a;
        a.owner_only = (what == kReduceScatter) ? 1u : 0u;
        a.n_out = 0;
        for (u32 i = 0; i < n_nodes; ++i) {
            a.in[i] = node_bufs[i];
            bool dup = false;
            for (u32 o = 0; o < a.n_out && !a.owner_only; ++o) dup = dup || (a.out[o] == out_bufs[i]);
            if (!dup) a.out[a.n_out++] = out_bufs[i];
        }
        u64 active_bytes = 0;
        for (u32 k = 0; k < n_rails; ++k)
            if (rail_mask >> k & 1u) active_bytes += (rail_off[k + 1] - rail_off[k]) << shift;
        uintptr_t out_lo = UINTPTR_MAX, out_hi = 0;
        for (u32 o = 0; o < a.n_out; ++o) {
            const uintptr_t p = reinterpret_cast<uintptr_t>(a.out[o]);
            out_lo = std::min(out_lo, p);
            out_hi = std::max(out_hi, p + bytes);
        }
        if (what == kAllreduce && staged_allreduce(a.n_out, active_bytes, out_hi - out_lo)) {
            // Large message, several outputs: the staged pipeline.
            StageArgs sa;
            std::memset(&sa, 0, sizeof sa);
            sa.n_nodes = n_nodes;
            sa.n_out = a.n_out;
            for (u32 i = 0; i < n_nodes; ++i) sa.in[i] = a.in[i];
            for (u32 i = 0; i < a.n_out; ++i) sa.out[i] = a.out[i];
            // The sums are staged through the output that lies farthest from the
            // inputs: a write stream into the memory region the reduce part is
            // reading from slows those reads down, and under a layout that
            // spreads the outputs (nz_hbm_place) the farthest one is in another
            // region.  Which output comes first changes no result.
            {
                uintptr_t in_lo = UINTPTR_MAX, in_hi = 0;
                for (u32 i = 0; i < n_nodes; ++i) {
                    const uintptr_t p = reinterpret_cast<uintptr_t>(a.in[i]);
                    in_lo = std::min(in_lo, p);
                    in_hi = std::max(in_hi, p + bytes);
                }
                u32 best = 0;
                uintptr_t best_gap = 0;
                for (u32 o = 0; o < a.n_out; ++o) {
                    const uintptr_t p = reinterpret_cast<uintptr_t>(a.out[o]);
                    const uintptr_t gap = p >= in_hi ? p - in_hi : (p + bytes <= in_lo ? in_lo - (p + bytes) : 0);
                    if (gap > best_gap) {
                        best_gap = gap;
                        best = o;
                    }
                }
                std::swap(sa.out[0], sa.out[best]);
            }
            switch (dtype) {
            case NZ_F32: return launch_staged<TF32>(sa, rail_off, n_rails, rail_mask, shift, st);
            case NZ_I32: return launch_staged<TI32>(sa, rail_off, n_rails, rail_mask, shift, st);
            case NZ_BF16: return launch_staged<TBF16>(sa, rail_off, n_rails, rail_mask, shift, st);
            case NZ_F16: return launch_staged<TF16>(sa, rail_off, n_rails, rail_mask, shift, st);
            }
            return NZ_ERR_INVALID_ARG;
        }
        if (what == kAllreduce && active_bytes == bytes) {
            // Every rail takes part: the sums do not depend on where rails and segments begin.
            FlatArgs fa;
            fa.bytes = bytes;
            fa.n_nodes = n_nodes;
            fa.n_out = a.n_out;
            for (u32 i = 0; i < n_nodes; ++i) fa.in[i] = a.in[i];
            for (u32 i = 0; i < a.n_out; ++i) fa.out[i] = a.out[i];
            switch (dtype) {
            case NZ_F32: return launch_flat<TF32>(fa, st);
            case NZ_I32: return launch_flat<TI32>(fa, st);
            case NZ_BF16: return launch_flat<TBF16>(fa, st);
            case NZ_F16: return launch_flat<TF16>(fa, st);
            }
            return NZ_ERR_INVALID_ARG;
        }
        u64 blocks = build_geometry(a.g, rail_off, n_rails, n_nodes, shift, kThreads, rail_mask);
        if (blocks == 0) return NZ_ERR_UNSUPPORTED;
        if (blocks == kNothingToDo) return NZ_OK;
        blocks += (u64)n_rails * n_nodes;  // the workgroups for segment edges
        const u64 moved = active_bytes * (n_nodes + (a.owner_only ? 1 : a.n_out));
        switch (dtype) {
        case NZ_F32: return launch_fused<TF32>(a, (u32)blocks, st, moved);
        case NZ_I32: return launch_fused<TI32>(a, (u32)blocks, st, moved);
        case NZ_BF16: return launch_fused<TBF16>(a, (u32)blocks, st, moved);
        case NZ_F16: return launch_fused<TF16>(a, (u32)blocks, st, moved);
        }
        return NZ_ERR_INVALID_ARG;
    }

    RingArgs a;
    const u64 blocks = build_geometry(a.g, rail_off, n_rails, n_nodes, shift, (u32)kRingIters * kThreads,
                                      rail_mask, piece_elems);
    if (blocks == 0) return NZ_ERR_UNSUPPORTED;
    if (blocks == kNothingToDo) return NZ_OK;
    u64 n_pieces = 1;
    if (piece_elems != UINT64_MAX) {
        u64 longest = 0;
        for (u32 k = 0; k < n_rails; ++k) longest = std::max<u64>(longest, a.g.q[k] + (a.g.rem[k] ? 1 : 0));
        n_pieces = std::max<u64>((longest + piece_elems - 1) / piece_elems, 1);
        if (n_pieces > 1u << 20) return NZ_ERR_UNSUPPORTED;  // more launches than anybody means
        if (n_pieces == 1) a.g.win_len = UINT64_MAX;
    }
    a.elem_shift = shift;
    a.step = 0;
    for (u32 i = 0; i < n_nodes; ++i) {
        a.in[i] = node_bufs[i];
        a.out[i] = out_bufs[i];
    }
    if (n_nodes == 1) {
        // A ring of one node has no steps: the result is the node's own data.
        if (what != kAllgather && out_bufs[0] != node_bufs[0]) {
            const hipError_t e = hipMemcpyAsync(out_bufs[0], node_bufs[0], bytes, hipMemcpyDeviceToDevice, st);
            if (e != hipSuccess) return hip_failed(e, "single-node copy");
        }
        return NZ_OK;
    }
    switch (dtype) {
    case NZ_F32: return launch_ring<TF32>(a, (u32)blocks, st, what, n_pieces);
    case NZ_I32: return launch_ring<TI32>(a, (u32)blocks, st, what, n_pieces);
    case NZ_BF16: return launch_ring<TBF16>(a, (u32)blocks, st, what, n_pieces);
    case NZ_F16: return launch_ring<TF16>(a, (u32)blocks, st, what, n_pieces);
    }
    return NZ_ERR_INVALID_ARG;
}

}  // namespace

extern "C" {

const char *nz_last_hip_error(void) { return g_hip_error; }

nz_status nz_allreduce_sim(const void *const *node_bufs, uint32_t n_nodes, uint64_t n_elems,
                           const uint32_t *ratios, uint32_t n_rails, nz_dtype dtype, nz_mode mode,
                           void *const *out_bufs, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    return finish(run_collective(kAllreduce, node_bufs, n_nodes, n_elems, ratios, n_rails, dtype, mode, out_bufs, st),
                  st);
}

nz_status nz_allreduce_launches(uint32_t n_nodes, uint64_t n_elems, const uint32_t *ratios, uint32_t n_rails,
                                nz_dtype dtype, nz_mode mode, uint32_t n_distinct_outputs,
                                uint64_t outputs_span_bytes, uint64_t *launches)
{
    if (ratios == nullptr || launches == nullptr || n_nodes == 0 || n_rails == 0) return NZ_ERR_INVALID_ARG;
    const u32 eb = nz_dtype_bytes(dtype);
    if (eb == 0 || (mode != NZ_RING_STEPWISE && mode != NZ_FUSED)) return NZ_ERR_INVALID_ARG;
    if (n_nodes > NZ_MAX_NODES || n_rails > NZ_MAX_RAILS) return NZ_ERR_UNSUPPORTED;
    u64 rail_off[NZ_MAX_RAILS + 1];
    const nz_status ps = nz::rail_partition(n_elems, eb, NZ_RAIL_ALIGN_BYTES, ratios, n_rails, rail_off);
    if (ps != NZ_OK) return ps;
    *launches = 0;
    if (n_elems == 0) return NZ_OK;
    if (mode == NZ_RING_STEPWISE) {
        *launches = n_nodes > 1 ? 2ull * (n_nodes - 1) : (n_distinct_outputs > 0 ? 1 : 0);
        return NZ_OK;
    }
    const u64 bytes = n_elems * eb;
    if (!staged_allreduce(n_distinct_outputs, bytes, outputs_span_bytes)) {
        *launches = 1;
        return NZ_OK;
    }
    // The staged pipeline: all rails take part, so the message is one span; one
    // launch per piece and one more that spreads the last piece.
    const u64 piece = stage_piece_bytes(bytes);
    *launches = (bytes + piece - 1) / piece + 1;
    return NZ_OK;
}

nz_status nz_reduce_scatter_sim(const void *const *node_bufs, uint32_t n_nodes, uint64_t n_elems,
                                const uint32_t *ratios, uint32_t n_rails, nz_dtype dtype, nz_mode mode,
                                void *const *out_bufs, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    return finish(run_collective(kReduceScatter, node_bufs, n_nodes, n_elems, ratios, n_rails, dtype, mode,
                                 out_bufs, st),
                  st);
}

nz_status nz_allgather_sim(void *const *bufs, uint32_t n_nodes, uint64_t n_elems, const uint32_t *ratios,
                           uint32_t n_rails, nz_dtype dtype, nz_mode mode, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    return finish(run_collective(kAllgather, reinterpret_cast<const void *const *>(bufs), n_nodes, n_elems,
                                 ratios, n_rails, dtype, mode, bufs, st),
                  st);
}

nz_status nz_allreduce_sim_chunked(const void *const *node_bufs, uint32_t n_nodes, uint64_t n_elems,
                                   const uint32_t *ratios, uint32_t n_rails, nz_dtype dtype,
                                   uint64_t chunk_elems, void *const *out_bufs, void *stream)
{
    if (chunk_elems == 0) return NZ_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    return finish(run_collective(kAllreduce, node_bufs, n_nodes, n_elems, ratios, n_rails, dtype,
                                 NZ_RING_STEPWISE, out_bufs, st, 0xffffffffu,
                                 chunk_elems == UINT64_MAX ? UINT64_MAX - 1 : chunk_elems),
                  st);
}

nz_status nz_allreduce_sim_failover(const void *const *node_bufs, uint32_t n_nodes, uint64_t n_elems,
                                    const uint32_t *ratios, uint32_t n_rails, nz_dtype dtype,
                                    nz_mode mode, void *const *out_bufs, uint32_t failed_rail,
                                    uint32_t *takeover_rail, void *stream)
{
    if (ratios == nullptr || n_rails == 0 || failed_rail >= n_rails) return NZ_ERR_INVALID_ARG;
    if (n_rails > NZ_MAX_RAILS) return NZ_ERR_UNSUPPORTED;
    const u32 eb = nz_dtype_bytes(dtype);
    if (eb == 0) return NZ_ERR_INVALID_ARG;
    u64 rail_off[NZ_MAX_RAILS + 1];
    const nz_status ps = nz::rail_partition(n_elems, eb, NZ_RAIL_ALIGN_BYTES, ratios, n_rails, rail_off);
    if (ps != NZ_OK) return ps;
    uint8_t alive[NZ_MAX_RAILS];
    for (u32 k = 0; k < n_rails; ++k) alive[k] = (k != failed_rail);
    u32 target = 0;
    const nz_status ts = nz_failover_target(rail_off, n_rails, alive, &target);
    if (ts != NZ_OK) return ts;  // no rail survives
    if (takeover_rail) *takeover_rail = target;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // First the surviving rails' own slices, then -- on the same stream, as the
    // take-over rail's next task -- the failed rail's slice, still cut as it was.
    const u32 all = (n_rails >= 32) ? 0xffffffffu : ((1u << n_rails) - 1u);
    const nz_status first = run_collective(kAllreduce, node_bufs, n_nodes, n_elems, ratios, n_rails, dtype,
                                           mode, out_bufs, st, all & ~(1u << failed_rail));
    if (first != NZ_OK) return first;
    return finish(run_collective(kAllreduce, node_bufs, n_nodes, n_elems, ratios, n_rails, dtype, mode, out_bufs,
                                 st, 1u << failed_rail),
                  st);
}

nz_status nz_pack(const void *const *node_bufs, uint32_t n_nodes, const uint64_t *seg_off,
                  uint32_t n_rails, uint32_t rail, const uint32_t *seg_ids, uint32_t n_segs,
                  uint32_t elem_bytes, void *const *send_bufs, uint64_t send_capacity_bytes,
                  uint64_t *packed_bytes, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    return finish(segment_copy(node_bufs, send_bufs, n_nodes, seg_off, n_rails, rail, seg_ids, n_segs,
                               elem_bytes, true, send_capacity_bytes, packed_bytes, st),
                  st);
}

nz_status nz_unpack(const void *const *send_bufs, uint32_t n_nodes, const uint64_t *seg_off,
                    uint32_t n_rails, uint32_t rail, const uint32_t *seg_ids, uint32_t n_segs,
                    uint32_t elem_bytes, void *const *node_bufs, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    return finish(segment_copy(send_bufs, node_bufs, n_nodes, seg_off, n_rails, rail, seg_ids, n_segs,
                               elem_bytes, false, 0, nullptr, st),
                  st);
}

}  // extern "C"
