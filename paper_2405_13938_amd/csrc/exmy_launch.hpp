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

// Grid size for one block per chunk of `chunk` tiles.  A launch that would need
// more blocks than a grid dimension can hold is capped; the kernels then stride.
// (The dispatch packet counts work-items in 32 bits: blocks * block_size < 2^32.)
inline uint32_t grid_for_chunks(uint64_t tiles, int chunk, int block_size) {
  const uint64_t blocks = (tiles + (uint64_t)chunk - 1) / (uint64_t)chunk;
  const uint64_t cap = 0xFFFFFFFFull / (uint64_t)block_size;
  const uint64_t g = blocks < cap ? blocks : cap;
  return (uint32_t)(g ? g : 1);
}

// Grid of the kernels that take one tile per workgroup without a loop: tile = blockIdx.z * gridDim.x +
// blockIdx.x, tensor = blockIdx.y.  x stops at 2^20 workgroups, so that tensors of more than 2^30 elements
// (which the large-tensor tests reach) already use z.
constexpr uint64_t kFlatGridX = 1ull << 20;
inline dim3 grid_for_flat_tiles(uint64_t tiles, uint32_t tensors) {
  if (tiles == 0) tiles = 1;
  const uint64_t x = tiles < kFlatGridX ? tiles : kFlatGridX;
  return dim3((uint32_t)x, tensors, (uint32_t)((tiles + x - 1) / x));
}

// `n_max` is the largest element count among the batch's tensors (sizes the grid).
hipError_t encode_dispatch(exmy_dtype_t dt, int W, bool wide, bool with_hist, const BatchArgs& args, uint64_t n_max,
                           hipStream_t stream);
hipError_t decode_dispatch(exmy_dtype_t dt, int W, bool x8, const BatchArgs& args, uint64_t n_max,
                           hipStream_t stream);
// Record layout (the plane words of a group as W consecutive bytes), W <= 16 except 8 and 16, whose
// records are the planar form.  flag: encode - the fp64 rounding path; decode - X = 8.
hipError_t records_dispatch(exmy_dtype_t dt, int W, bool decode, bool flag, const void* src, void* dst, uint64_t n,
                            const FormatConsts& fc, const TensorConsts& tc, hipStream_t stream);
// Reserved NaN / Inf code points (W <= 16); tc.sat_bits holds the largest finite value.
hipError_t specials_dispatch(exmy_dtype_t dt, int W, bool decode, bool wide, const void* src, void* dst, uint64_t n,
                             const FormatConsts& fc, const TensorConsts& tc, const SpecialConsts& sc,
                             hipStream_t stream);
// W = 32 (e8m23 on fp32): the packed form is the array of codes; encode and decode clamp Inf / NaN patterns.
hipError_t codes32_dispatch(bool decode, const BatchArgs& args, uint64_t n_max, hipStream_t stream);
hipError_t emulate_dispatch(exmy_dtype_t dt, bool wide, void* data, uint64_t n, const FormatConsts& fc,
                            const TensorConsts& tc, hipStream_t stream);
// Per-block metadata (args.bi is filled in by the dispatcher from args.block_groups).
// `scaled` / `scale`: the float-scaling variants, which read or write args.scale
// instead of args.meta.
hipError_t encode_blocks_dispatch(exmy_dtype_t dt, int W, const BlockArgs& args, bool scaled, hipStream_t stream);
hipError_t decode_blocks_dispatch(exmy_dtype_t dt, int W, const BlockArgs& args, bool scaled, hipStream_t stream);
hipError_t emulate_blocks_dispatch(exmy_dtype_t dt, const BlockArgs& args, bool wide_format, bool scaled,
                                   hipStream_t stream);
// Metadata + codes in one pass; only for block sizes that encode_blocks_auto_fits accepts (args.meta is written).
bool encode_blocks_auto_fits(exmy_dtype_t dt, uint32_t block_groups);
hipError_t encode_blocks_auto_dispatch(exmy_dtype_t dt, int W, const BlockArgs& args, hipStream_t stream);
hipError_t block_max_exp_dispatch(exmy_dtype_t dt, const BlockArgs& args, bool scale, hipStream_t stream);
// Blocks that are columns or 2-D tiles (args.ti is filled in by the dispatcher through
// make_tile_index, in units of `unit_elems` elements).  tile_max_exp_dispatch clears
// args.meta and then folds the maxima into it (two launches).
TileIndex make_tile_index(const TileArgs& args, uint32_t unit_elems);
hipError_t encode_tiles_dispatch(exmy_dtype_t dt, int W, const TileArgs& args, hipStream_t stream);
hipError_t decode_tiles_dispatch(exmy_dtype_t dt, int W, const TileArgs& args, hipStream_t stream);
hipError_t emulate_tiles_dispatch(exmy_dtype_t dt, const TileArgs& args, bool wide_format, hipStream_t stream);
hipError_t tile_max_exp_dispatch(exmy_dtype_t dt, const TileArgs& args, hipStream_t stream);
// Packing along rows (args.tiles is filled in by the dispatcher).
hipError_t encode_rows_dispatch(exmy_dtype_t dt, int W, const RowsArgs& args, bool per_row, bool wide,
                                hipStream_t stream);
hipError_t decode_rows_dispatch(exmy_dtype_t dt, int W, const RowsArgs& args, bool per_row, bool x8,
                                hipStream_t stream);
// Two's complement reading of e0mY (W = 1 + Y).
hipError_t encode_int_dispatch(exmy_dtype_t dt, int W, const void* src, void* dst, uint64_t n, const IntConsts& ic,
                               hipStream_t stream);
hipError_t decode_int_dispatch(exmy_dtype_t dt, int W, const void* src, void* dst, uint64_t n, const IntConsts& ic,
                               hipStream_t stream);
hipError_t emulate_int_dispatch(exmy_dtype_t dt, void* data, uint64_t n, const IntConsts& ic, hipStream_t stream);
hipError_t histogram_dispatch(exmy_dtype_t dt, const void* src, uint64_t n, uint64_t* hist, hipStream_t stream);

}  // namespace exmy
