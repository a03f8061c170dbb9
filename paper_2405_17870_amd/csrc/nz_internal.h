// Internal declarations shared by the host-side index maps and the HIP file.
#ifndef NZ_INTERNAL_H
#define NZ_INTERNAL_H

#include <cstddef>
#include <cstdint>

#include "nezha_sim.h"

namespace nz {

nz_status rail_partition(uint64_t n_elems, uint32_t elem_bytes, uint32_t align_bytes,
                         const uint32_t *ratios, uint32_t n_rails, uint64_t *rail_off);

nz_status segment_map(const uint64_t *rail_off, uint32_t n_rails, uint32_t n_nodes,
                      uint64_t *seg_off);

// Buffer-overlap rules, decided before any launch (nz_validate.cpp).
// Collectives: buffers of `bytes` bytes each; a written buffer may not partly
// overlap any other; with distinct_outputs_needed the outputs are pairwise
// distinct and an output may equal its own node's input only.
nz_status check_collective_buffers(const void *const *node_bufs, void *const *out_bufs, uint32_t n_nodes,
                                   uint64_t bytes, bool distinct_outputs_needed);

// Pack / unpack: source m is read in [src[m] + src_lo, src[m] + src_hi), destination m written
// in [dst[m] + dst_lo, dst[m] + dst_hi); a written range may not overlap any other range.
nz_status check_copy_buffers(const void *const *src, void *const *dst, uint32_t n_nodes, uint64_t src_lo,
                             uint64_t src_hi, uint64_t dst_lo, uint64_t dst_hi);

}  // namespace nz

#endif
