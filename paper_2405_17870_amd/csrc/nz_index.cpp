// Host-side index maps of the multi-rail allreduce: which elements each rail
// owns and how a rail's range is cut into ring segments.  Pure integer
// arithmetic, no GPU involved.
//
// Nezha (arXiv 2405.17870): Sec. 3.4 / 3.5 give every member network one
// contiguous (ptr, data_length) slice derived from its share of the data
// volume; the shares sum to one (Sec. 4.3, under Eq. 5); a ring over N workers
// handles a message in N pieces (Sec. 2.1.1, Eq. 1).
#include "nz_internal.h"

namespace nz {

nz_status rail_partition(uint64_t n_elems, uint32_t elem_bytes, uint32_t align_bytes,
                         const uint32_t *ratios, uint32_t n_rails, uint64_t *rail_off)
{
    if (ratios == nullptr || rail_off == nullptr || n_rails == 0) return NZ_ERR_INVALID_ARG;
    if (elem_bytes != 2 && elem_bytes != 4) return NZ_ERR_INVALID_ARG;
    if (align_bytes == 0 || align_bytes % elem_bytes != 0) return NZ_ERR_INVALID_ARG;
    if (n_elems > (UINT64_MAX >> 3)) return NZ_ERR_INVALID_ARG;  // byte offsets must fit 64 bits

    uint64_t weight_sum = 0;
    for (uint32_t k = 0; k < n_rails; ++k) weight_sum += ratios[k];
    if (weight_sum == 0) return NZ_ERR_INVALID_ARG;

    const uint64_t unit = align_bytes / elem_bytes;  // alignment in elements
    uint64_t before = 0;                              // weight of the rails in front of boundary k
    rail_off[0] = 0;
    for (uint32_t k = 1; k < n_rails; ++k) {
        before += ratios[k - 1];
        if (before == weight_sum) {
            // Only zero-weight rails follow: they get nothing, so the rail in
            // front of this boundary ends at the end of the message.
            rail_off[k] = n_elems;
            continue;
        }
        // Whole alignment units in front of the proportional point n * before / sum.
        const unsigned __int128 scaled = static_cast<unsigned __int128>(n_elems) * before;
        const unsigned __int128 units = scaled / (static_cast<unsigned __int128>(weight_sum) * unit);
        rail_off[k] = static_cast<uint64_t>(units) * unit;
    }
    rail_off[n_rails] = n_elems;
    return NZ_OK;
}

nz_status segment_map(const uint64_t *rail_off, uint32_t n_rails, uint32_t n_nodes,
                      uint64_t *seg_off)
{
    if (rail_off == nullptr || seg_off == nullptr || n_rails == 0 || n_nodes == 0)
        return NZ_ERR_INVALID_ARG;
    for (uint32_t k = 0; k < n_rails; ++k)
        if (rail_off[k + 1] < rail_off[k]) return NZ_ERR_INVALID_ARG;
    for (uint32_t k = 0; k < n_rails; ++k) {
        const uint64_t len = rail_off[k + 1] - rail_off[k];
        const uint64_t base = len / n_nodes;
        const uint64_t extra = len % n_nodes;  // the first `extra` segments are one longer
        uint64_t *row = seg_off + static_cast<size_t>(k) * (n_nodes + 1);
        for (uint32_t j = 0; j <= n_nodes; ++j)
            row[j] = rail_off[k] + j * base + (j < extra ? j : extra);
    }
    return NZ_OK;
}

}  // namespace nz

extern "C" {

nz_status nz_rail_partition(uint64_t n_elems, uint32_t elem_bytes, const uint32_t *ratios,
                            uint32_t n_rails, uint64_t *rail_off)
{
    return nz::rail_partition(n_elems, elem_bytes, NZ_RAIL_ALIGN_BYTES, ratios, n_rails, rail_off);
}

nz_status nz_rail_partition_ex(uint64_t n_elems, uint32_t elem_bytes, uint32_t align_bytes,
                               const uint32_t *ratios, uint32_t n_rails, uint64_t *rail_off)
{
    return nz::rail_partition(n_elems, elem_bytes, align_bytes, ratios, n_rails, rail_off);
}

nz_status nz_segment_map(const uint64_t *rail_off, uint32_t n_rails, uint32_t n_nodes,
                         uint64_t *seg_off)
{
    return nz::segment_map(rail_off, n_rails, n_nodes, seg_off);
}

// Sec. 4.4: the surviving rail that was allocated the most data takes over a
// failed rail's slice.
nz_status nz_failover_target(const uint64_t *rail_off, uint32_t n_rails, const uint8_t *alive,
                             uint32_t *target)
{
    if (rail_off == nullptr || alive == nullptr || target == nullptr || n_rails == 0)
        return NZ_ERR_INVALID_ARG;
    bool found = false;
    uint64_t most = 0;
    for (uint32_t k = 0; k < n_rails; ++k) {
        if (rail_off[k + 1] < rail_off[k]) return NZ_ERR_INVALID_ARG;
        if (!alive[k]) continue;
        const uint64_t len = rail_off[k + 1] - rail_off[k];
        if (!found || len > most) {
            found = true;
            most = len;
            *target = k;
        }
    }
    return found ? NZ_OK : NZ_ERR_INVALID_ARG;
}

uint32_t nz_dtype_bytes(nz_dtype dtype)
{
    switch (dtype) {
    case NZ_F32:
    case NZ_I32: return 4;
    case NZ_BF16:
    case NZ_F16: return 2;
    }
    return 0;
}

const char *nz_status_str(nz_status s)
{
    switch (s) {
    case NZ_OK: return "ok";
    case NZ_ERR_INVALID_ARG: return "invalid argument";
    case NZ_ERR_ALIGNMENT: return "device buffer not aligned to 256 bytes";
    case NZ_ERR_UNSUPPORTED: return "unsupported: over a limit or buffers overlap";
    case NZ_ERR_CAPACITY: return "destination buffer too small";
    case NZ_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

}  // extern "C"
