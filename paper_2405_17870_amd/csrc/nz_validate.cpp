// Which buffer overlaps a call accepts (see "Aliasing" in nezha_sim.h), decided
// on the host before anything is launched.  Pure C++: no GPU call, no
// allocation (fixed arrays on the stack), so the sanitizer build covers it.
#include <algorithm>
#include <utility>

#include "nz_internal.h"

namespace {

typedef uint64_t u64;
typedef uint32_t u32;

struct PtrRef {
    uintptr_t p;
    bool written;
};

// Buffers of `bytes` bytes each: a written buffer may not partially overlap
// any other buffer.  v has n entries and is reordered.
bool partial_overlap(PtrRef *v, size_t n, u64 bytes)
{
    std::sort(v, v + n, [](const PtrRef &x, const PtrRef &y) { return x.p < y.p; });
    // merge equal pointers
    size_t w = 0;
    for (size_t i = 0; i < n; ++i) {
        if (w > 0 && v[w - 1].p == v[i].p)
            v[w - 1].written = v[w - 1].written || v[i].written;
        else
            v[w++] = v[i];
    }
    for (size_t i = 0; i + 1 < w; ++i)
        if (v[i + 1].p - v[i].p < bytes && (v[i].written || v[i + 1].written)) return true;
    return false;
}

// The common layouts need no sorting: the addresses of an array of buffers
// run in one direction with at least `bytes` between neighbours (what an
// allocator hands out one after the other).  Gives the span they cover.
bool monotone_disjoint(const void *const *bufs, u32 n, u64 bytes, uintptr_t &lo, uintptr_t &hi)
{
    const uintptr_t first = reinterpret_cast<uintptr_t>(bufs[0]);
    const uintptr_t last = reinterpret_cast<uintptr_t>(bufs[n - 1]);
    const bool up = last >= first;
    for (u32 i = 0; i + 1 < n; ++i) {
        const uintptr_t a = reinterpret_cast<uintptr_t>(bufs[i]), b = reinterpret_cast<uintptr_t>(bufs[i + 1]);
        if (up ? (b < a || b - a < bytes) : (a < b || a - b < bytes)) return false;
    }
    lo = up ? first : last;
    hi = (up ? last : first) + bytes;
    return true;
}

struct Range {
    uintptr_t lo, hi;
    bool written;
};

// True if a written range overlaps any other range (read ranges may overlap
// each other freely).  v has n entries and is reordered.
bool written_range_overlaps(Range *v, size_t n)
{
    std::sort(v, v + n, [](const Range &x, const Range &y) { return x.lo < y.lo; });
    uintptr_t end_any = 0, end_written = 0;
    for (size_t i = 0; i < n; ++i) {
        const Range &r = v[i];
        if (r.lo == r.hi) continue;
        if (r.written ? r.lo < end_any : r.lo < end_written) return true;
        end_any = std::max(end_any, r.hi);
        if (r.written) end_written = std::max(end_written, r.hi);
    }
    return false;
}

}  // namespace

namespace nz {

nz_status check_collective_buffers(const void *const *node_bufs, void *const *out_bufs, uint32_t n_nodes,
                                   uint64_t bytes, bool distinct_outputs_needed)
{
    if (n_nodes == 0 || n_nodes > NZ_MAX_NODES) return NZ_ERR_UNSUPPORTED;
    // Fast way out for the two layouts callers normally have: inputs and
    // outputs each handed out one after the other by an allocator and apart
    // from each other, or every output its own node's input (in place).
    {
        uintptr_t in_lo, in_hi, out_lo, out_hi;
        if (bytes > 0 && monotone_disjoint(node_bufs, n_nodes, bytes, in_lo, in_hi) &&
            monotone_disjoint(reinterpret_cast<const void *const *>(out_bufs), n_nodes, bytes, out_lo, out_hi)) {
            bool in_place = true;
            for (u32 i = 0; i < n_nodes; ++i) in_place = in_place && node_bufs[i] == out_bufs[i];
            if (in_place || in_hi <= out_lo || out_hi <= in_lo) return NZ_OK;
        }
    }
    {
        PtrRef refs[2 * NZ_MAX_NODES];
        for (u32 i = 0; i < n_nodes; ++i) {
            refs[2 * i] = {reinterpret_cast<uintptr_t>(node_bufs[i]), false};
            refs[2 * i + 1] = {reinterpret_cast<uintptr_t>(out_bufs[i]), true};
        }
        if (partial_overlap(refs, 2 * (size_t)n_nodes, bytes)) return NZ_ERR_UNSUPPORTED;
    }
    if (distinct_outputs_needed) {
        // Outputs pairwise distinct; an output may alias only its own node's input.
        std::pair<uintptr_t, u32> ins[NZ_MAX_NODES], outs[NZ_MAX_NODES];
        for (u32 i = 0; i < n_nodes; ++i) {
            ins[i] = {reinterpret_cast<uintptr_t>(node_bufs[i]), i};
            outs[i] = {reinterpret_cast<uintptr_t>(out_bufs[i]), i};
        }
        std::sort(ins, ins + n_nodes);
        std::sort(outs, outs + n_nodes);
        for (u32 i = 0; i + 1 < n_nodes; ++i)
            if (outs[i].first == outs[i + 1].first) return NZ_ERR_UNSUPPORTED;
        for (u32 i = 0; i < n_nodes; ++i) {
            auto it = std::lower_bound(ins, ins + n_nodes, std::make_pair(outs[i].first, 0u));
            for (; it != ins + n_nodes && it->first == outs[i].first; ++it)
                if (it->second != outs[i].second) return NZ_ERR_UNSUPPORTED;
        }
    }
    return NZ_OK;
}

nz_status check_copy_buffers(const void *const *src, void *const *dst, uint32_t n_nodes, uint64_t src_lo,
                             uint64_t src_hi, uint64_t dst_lo, uint64_t dst_hi)
{
    if (n_nodes == 0 || n_nodes > NZ_MAX_NODES) return NZ_ERR_UNSUPPORTED;
    Range ranges[2 * NZ_MAX_NODES];
    for (u32 m = 0; m < n_nodes; ++m) {
        const uintptr_t s0 = reinterpret_cast<uintptr_t>(src[m]), d0 = reinterpret_cast<uintptr_t>(dst[m]);
        ranges[2 * m] = {s0 + src_lo, s0 + src_hi, false};
        ranges[2 * m + 1] = {d0 + dst_lo, d0 + dst_hi, true};
    }
    return written_range_overlaps(ranges, 2 * (size_t)n_nodes) ? NZ_ERR_UNSUPPORTED : NZ_OK;
}

}  // namespace nz
