// Host-side launch helpers shared by the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "exmy_common.hpp"

namespace exmy {

// Compute units of the current device (cached per device ordinal).
int compute_units();

// Grid size for a grid-stride loop over `tiles` tiles: every tile gets a block
// until the device holds blocks_per_cu resident blocks per compute unit.
inline uint32_t grid_for_tiles(uint64_t tiles, int blocks_per_cu) {
  const uint64_t cap = (uint64_t)compute_units() * (uint64_t)blocks_per_cu;
  uint64_t g = tiles < cap ? tiles : cap;
  return (uint32_t)(g ? g : 1);
}

hipError_t encode_dispatch(exmy_dtype_t dt, int W, bool wide, bool with_hist, const void* src, void* dst,
                           uint64_t n, const FormatConsts& fc, uint64_t* hist, hipStream_t stream);
hipError_t decode_dispatch(exmy_dtype_t dt, int W, bool x8, const void* src, void* dst, uint64_t n,
                           const FormatConsts& fc, hipStream_t stream);
hipError_t emulate_dispatch(exmy_dtype_t dt, bool wide, void* data, uint64_t n, const FormatConsts& fc,
                            hipStream_t stream);
hipError_t histogram_dispatch(exmy_dtype_t dt, const void* src, uint64_t n, uint64_t* hist, hipStream_t stream);

}  // namespace exmy
