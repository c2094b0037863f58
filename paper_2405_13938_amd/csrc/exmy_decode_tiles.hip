// Host-side dispatch of the decode, emulation and maximum-exponent kernels for blocks
// that are columns or 2-D tiles (see exmy_tiles_kernel.hpp).
#include "exmy_launch.hpp"
#include "exmy_tiles_kernel.hpp"

namespace exmy {

namespace {

// Same shapes as the per-block decoder.
template <typename T>
struct Shape;
template <>
struct Shape<uint16_t> {
  static constexpr int kBlock = 128;
  static constexpr int kUnroll = 2;
};
template <>
struct Shape<f16_t> : Shape<uint16_t> {};
template <>
struct Shape<float> {
  static constexpr int kBlock = 256;
  static constexpr int kUnroll = 2;
};

template <typename T, int W>
hipError_t launch(TileArgs args, hipStream_t stream) {
  using S = Shape<T>;
  constexpr uint32_t E = 16 / sizeof(T);
  const uint64_t tile_units = (uint64_t)S::kBlock * S::kUnroll;
  const uint64_t tiles = (args.rows * args.cols / E + tile_units - 1) / tile_units;
  args.ti = make_tile_index(args, E);
  const dim3 grid = grid_for_flat_tiles(tiles, 1), block(S::kBlock);
  if (args.tile_cols == 1)
    hipLaunchKernelGGL((tiles::decode_tiles_kernel<T, W, S::kBlock, S::kUnroll, true, true>), grid, block, 0, stream, args);
  else
    hipLaunchKernelGGL((tiles::decode_tiles_kernel<T, W, S::kBlock, S::kUnroll, true, false>), grid, block, 0, stream, args);
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

constexpr int kEmuBlock = 128;
constexpr int kEmuUnroll = 1;

template <typename T>
hipError_t launch_emulate(TileArgs args, bool wide_format, hipStream_t stream) {
  constexpr uint32_t E = 16 / sizeof(T);
  const uint64_t tile_vecs = (uint64_t)kEmuBlock * kEmuUnroll;
  const uint64_t tiles = (args.rows * args.cols / E + tile_vecs - 1) / tile_vecs;
  args.ti = make_tile_index(args, E);
  const dim3 grid = grid_for_flat_tiles(tiles, 1), block(kEmuBlock);
  if (args.tile_cols == 1)
    hipLaunchKernelGGL((tiles::emulate_tiles_kernel<T, kEmuBlock, kEmuUnroll, true, true>), grid, block, 0, stream, args, wide_format);
  else
    hipLaunchKernelGGL((tiles::emulate_tiles_kernel<T, kEmuBlock, kEmuUnroll, true, false>), grid, block, 0, stream, args, wide_format);
  return hipGetLastError();
}

constexpr int kMaxBlock = 256;

template <typename T>
hipError_t launch_max_exp(TileArgs args, hipStream_t stream) {
  constexpr uint32_t E = 16 / sizeof(T);
  const bool columns = args.tile_cols == 1;
  args.ti = make_tile_index(args, E);
  tiles::MaxGeometry geo;
  geo.vpr = (uint32_t)(args.cols / E);
  // Column blocks give every element of a strip a metadata byte of its own to fold into: strips of 32 lanes
  // (512 bytes of a matrix row) with 8 rows per step fold 18 x fewer words than strips of 256 lanes, 4.15 -> 5.65 TB/s
  // on a (32768, 11008) bf16 matrix; 16 lanes measured the same, 8 lanes 5-15 % less.
  geo.lanes_x_log2 = columns ? 5 : 8;
  if (geo.vpr <= (columns ? 32u : 128u)) {
    geo.lanes_x_log2 = 0;
    while ((1u << geo.lanes_x_log2) < geo.vpr) ++geo.lanes_x_log2;
  }
  const uint32_t lanes_x = 1u << geo.lanes_x_log2;
  const uint32_t lanes_y = kMaxBlock >> geo.lanes_x_log2;
  geo.strips = (geo.vpr + lanes_x - 1) / lanes_x;
  geo.tile_rows_n = (args.rows + args.tile_rows - 1) / args.tile_rows;
  // Tall tiles are cut into row chunks, each folded into the metadata by its own workgroup: longer chunks
  // mean fewer folds, as long as enough regions are left: several times what the device holds at once (2048), so
  // that the last, partly filled round of workgroups is a small part of the launch.
  constexpr uint64_t kEnoughRegions = 8192;
  for (geo.row_steps = 64;; geo.row_steps /= 2) {
    geo.chunk_rows = lanes_y * geo.row_steps;
    geo.chunks = (uint32_t)((args.tile_rows + geo.chunk_rows - 1) / geo.chunk_rows);
    geo.regions = (uint64_t)geo.strips * geo.chunks * geo.tile_rows_n;
    if (geo.row_steps == 16 || (geo.regions >= kEnoughRegions && args.tile_rows >= geo.chunk_rows)) break;
  }
  geo.tcv = make_block_index(columns ? 1 : args.tile_cols / E);

  const uint64_t meta_bytes = geo.tile_rows_n * args.ti.meta_stride;
  // the 1-3 bytes of a last partial word are written by a kernel of their own (columns: cols, and with it
  // the array size, is a multiple of 8)
  const uint32_t tail_bytes = (uint32_t)(meta_bytes % 4);
  geo.tail_word = tail_bytes ? meta_bytes / 4 : ~0ull;
  if (meta_bytes >= 4) {
    const uint64_t clear_blocks = (meta_bytes / 4 + 255) / 256;
    hipLaunchKernelGGL(tiles::clear_words_kernel<256>, dim3((uint32_t)(clear_blocks < 4096 ? clear_blocks : 4096)), dim3(256), 0,
                       stream, args.meta, meta_bytes);
    if (hipError_t e = hipGetLastError()) return e;
    const dim3 grid(grid_for_chunks(geo.regions, 1, kMaxBlock)), block(kMaxBlock);
    if (columns)
      hipLaunchKernelGGL((tiles::tile_max_exp_kernel<T, kMaxBlock, true>), grid, block, 0, stream, args, geo);
    else
      hipLaunchKernelGGL((tiles::tile_max_exp_kernel<T, kMaxBlock, false>), grid, block, 0, stream, args, geo);
    if (hipError_t e = hipGetLastError()) return e;
  }
  if (tail_bytes) {
    const uint64_t tile_vecs = std::min<uint64_t>(args.tile_cols, args.cols) / E;
    uint32_t lx_log2 = 0;
    while (lx_log2 < 8 && (1ull << lx_log2) < tile_vecs) ++lx_log2;
    hipLaunchKernelGGL((tiles::tile_max_exp_tail_kernel<T, kMaxBlock>), dim3(tail_bytes), dim3(kMaxBlock), 0, stream, args,
                       meta_bytes - tail_bytes, lx_log2);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t decode_tiles_dispatch(exmy_dtype_t dt, int W, const TileArgs& args, hipStream_t stream) {
  if (dt == EXMY_F16) return dispatch_w<f16_t>(W, args, stream);
  return dt == EXMY_F32 ? dispatch_w<float>(W, args, stream) : dispatch_w<uint16_t>(W, args, stream);
}

hipError_t emulate_tiles_dispatch(exmy_dtype_t dt, const TileArgs& args, bool wide_format, hipStream_t stream) {
  if (dt == EXMY_F16) return launch_emulate<f16_t>(args, wide_format, stream);
  return dt == EXMY_F32 ? launch_emulate<float>(args, wide_format, stream) : launch_emulate<uint16_t>(args, wide_format, stream);
}

hipError_t tile_max_exp_dispatch(exmy_dtype_t dt, const TileArgs& args, hipStream_t stream) {
  if (dt == EXMY_F16) return launch_max_exp<f16_t>(args, stream);
  return dt == EXMY_F32 ? launch_max_exp<float>(args, stream) : launch_max_exp<uint16_t>(args, stream);
}

}  // namespace exmy
