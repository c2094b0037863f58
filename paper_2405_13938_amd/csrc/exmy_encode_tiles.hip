// Host-side dispatch of the encode kernels for blocks that are columns or 2-D tiles
// (see exmy_tiles_kernel.hpp).
#include "exmy_launch.hpp"
#include "exmy_tiles_kernel.hpp"

namespace exmy {

TileIndex make_tile_index(const TileArgs& args, uint32_t unit_elems) {
  const bool columns = args.tile_cols == 1;
  TileIndex ti;
  ti.row = make_block_index(args.cols / unit_elems);
  ti.trow = make_block_index(args.tile_rows);
  ti.tcol = make_block_index(columns ? 1 : args.tile_cols / unit_elems);
  ti.meta_stride = (uint32_t)(columns ? args.cols : args.tiles_along_row);
  ti.unit_elems = unit_elems;
  return ti;
}

namespace {

// Same shapes as the per-block encoder: one workgroup tile per workgroup.
template <typename T>
struct Shape;
template <>
struct Shape<uint16_t> {
  static constexpr int kBlock = 64;
  static constexpr int kUnroll = 2;
};
template <>
struct Shape<f16_t> : Shape<uint16_t> {};
template <>
struct Shape<float> {
  static constexpr int kBlock = 128;
  static constexpr int kUnroll = 1;
};

template <typename T, int W>
hipError_t launch(TileArgs args, hipStream_t stream) {
  using S = Shape<T>;
  const uint64_t tile_groups = (uint64_t)S::kBlock * S::kUnroll;
  const uint64_t tiles = (args.rows * args.cols / 8 + tile_groups - 1) / tile_groups;
  args.ti = make_tile_index(args, 8);
  const dim3 grid = grid_for_flat_tiles(tiles, 1), block(S::kBlock);
  if (args.tile_cols == 1)
    hipLaunchKernelGGL((tiles::encode_tiles_kernel<T, W, S::kBlock, S::kUnroll, true, true>), grid, block, 0, stream, args);
  else
    hipLaunchKernelGGL((tiles::encode_tiles_kernel<T, W, S::kBlock, S::kUnroll, true, false>), grid, block, 0, stream, args);
  return hipGetLastError();
}

template <typename T>
hipError_t dispatch_w(int W, const TileArgs& args, hipStream_t stream) {
  switch (W) {
#define EXMY_CASE(w) \
  case w:            \
    return launch<T, w>(args, stream);
    EXMY_CASE(1) EXMY_CASE(2) EXMY_CASE(3) EXMY_CASE(4) EXMY_CASE(5) EXMY_CASE(6) EXMY_CASE(7) EXMY_CASE(8)
    EXMY_CASE(9) EXMY_CASE(10) EXMY_CASE(11) EXMY_CASE(12) EXMY_CASE(13) EXMY_CASE(14) EXMY_CASE(15) EXMY_CASE(16)
#undef EXMY_CASE
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t encode_tiles_dispatch(exmy_dtype_t dt, int W, const TileArgs& args, hipStream_t stream) {
  if (dt == EXMY_F16) return dispatch_w<f16_t>(W, args, stream);
  return dt == EXMY_F32 ? dispatch_w<float>(W, args, stream) : dispatch_w<uint16_t>(W, args, stream);
}

}  // namespace exmy
