// Host-side dispatch of the row-packing decode kernels (see exmy_rows_kernel.hpp).
#include "exmy_launch.hpp"
#include "exmy_rows_kernel.hpp"

namespace exmy {

namespace {

constexpr int kBlock = 64;

// Places (16-byte row pieces) per row block below which, unless they fill whole tiles, the tiles are folded
// over row blocks: the idle part of a row block's last tile would otherwise cost more than the per-lane
// metadata of the folded form.
constexpr uint64_t kFoldBelow = 512;

template <typename T, int W, bool kFold>
hipError_t launch_form(RowsArgs args, bool per_row, bool x8, hipStream_t stream) {
  const uint64_t places = args.cols / (16 / sizeof(T));  // per row block
  const uint64_t row_blocks = (args.rows + 7) / 8;
  uint64_t tiles;
  if (kFold) {
    args.tiles = make_block_index(places);
    tiles = (row_blocks * places + kBlock - 1) / kBlock;
  } else {
    const uint64_t tiles_per_row_block = (places + kBlock - 1) / kBlock;
    args.tiles = make_block_index(tiles_per_row_block);
    tiles = row_blocks * tiles_per_row_block;
  }
  args.xcd_chunk = 0;
  if ((args.cols * sizeof(T)) % 128) {  // rows start inside cache lines: see die_ranged_tile
    args.xcd_chunk = (tiles + 7) / 8;
    tiles = args.xcd_chunk * 8;
  }
  const dim3 grid = grid_for_flat_tiles(tiles, 1);
  if (per_row)
    hipLaunchKernelGGL((rows::decode_rows_kernel<T, W, kBlock, true, false, kFold>), grid, dim3(kBlock), 0, stream, args);
  else if (x8)
    hipLaunchKernelGGL((rows::decode_rows_kernel<T, W, kBlock, false, true, kFold>), grid, dim3(kBlock), 0, stream, args);
  else
    hipLaunchKernelGGL((rows::decode_rows_kernel<T, W, kBlock, false, false, kFold>), grid, dim3(kBlock), 0, stream, args);
  return hipGetLastError();
}

template <typename T, int W>
hipError_t launch(const RowsArgs& args, bool per_row, bool x8, hipStream_t stream) {
  const uint64_t places = args.cols / (16 / sizeof(T));
  if (places % kBlock && places < kFoldBelow) return launch_form<T, W, true>(args, per_row, x8, stream);
  return launch_form<T, W, false>(args, per_row, x8, stream);
}

template <typename T>
hipError_t dispatch_w(int W, const RowsArgs& args, bool per_row, bool x8, hipStream_t stream) {
  switch (W) {
#define EXMY_CASE(w) \
  case w:            \
    return launch<T, w>(args, per_row, x8, stream);
    EXMY_CASE(1) EXMY_CASE(2) EXMY_CASE(3) EXMY_CASE(4) EXMY_CASE(5) EXMY_CASE(6) EXMY_CASE(7) EXMY_CASE(8)
    EXMY_CASE(9) EXMY_CASE(10) EXMY_CASE(11) EXMY_CASE(12) EXMY_CASE(13) EXMY_CASE(14) EXMY_CASE(15) EXMY_CASE(16)
#undef EXMY_CASE
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t decode_rows_dispatch(exmy_dtype_t dt, int W, const RowsArgs& args, bool per_row, bool x8,
                                hipStream_t stream) {
  if (dt == EXMY_F16) return dispatch_w<f16_t>(W, args, per_row, x8, stream);
  return dt == EXMY_F32 ? dispatch_w<float>(W, args, per_row, x8, stream)
                        : dispatch_w<uint16_t>(W, args, per_row, x8, stream);
}

}  // namespace exmy
