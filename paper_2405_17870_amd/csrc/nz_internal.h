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

}  // namespace nz

#endif
