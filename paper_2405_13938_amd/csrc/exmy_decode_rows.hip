// Host-side dispatch of the row-packing decode kernels (see exmy_rows_kernel.hpp).
#include "exmy_launch.hpp"
#include "exmy_rows_kernel.hpp"

namespace exmy {

namespace {

constexpr int kBlock = 64;

template <typename T, int W>
hipError_t launch(RowsArgs args, bool per_row, bool x8, hipStream_t stream) {
  constexpr uint64_t kTileCols = (uint64_t)kBlock * (16 / sizeof(T));
  const uint64_t tiles_per_row_block = (args.cols + kTileCols - 1) / kTileCols;
  args.tiles = make_block_index(tiles_per_row_block);
  const dim3 grid(grid_for_chunks(((args.rows + 7) / 8) * tiles_per_row_block, 1, kBlock));
  if (per_row)
    hipLaunchKernelGGL((rows::decode_rows_kernel<T, W, kBlock, true, false>), grid, dim3(kBlock), 0, stream, args);
  else if (x8)
    hipLaunchKernelGGL((rows::decode_rows_kernel<T, W, kBlock, false, true>), grid, dim3(kBlock), 0, stream, args);
  else
    hipLaunchKernelGGL((rows::decode_rows_kernel<T, W, kBlock, false, false>), grid, dim3(kBlock), 0, stream, args);
  return hipGetLastError();
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
