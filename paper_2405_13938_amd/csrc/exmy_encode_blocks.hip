// Host-side dispatch of the per-block-metadata encode kernels (see exmy_encode_kernel.hpp).
#include "exmy_encode_kernel.hpp"
#include "exmy_launch.hpp"

namespace exmy {

namespace {

// Same shapes as the per-tensor encoder: one tile per workgroup.
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

template <typename T, int W, bool kScaled>
hipError_t launch(BlockArgs args, hipStream_t stream) {
  using S = Shape<T>;
  const uint64_t tile_groups = (uint64_t)S::kBlock * S::kUnroll;
  const uint64_t tiles = (args.n / 8 + tile_groups - 1) / tile_groups;
  args.bi = make_block_index(args.block_groups);
  hipLaunchKernelGGL((enc::encode_blocks_kernel<T, W, S::kBlock, S::kUnroll, true, kScaled>),
                     grid_for_flat_tiles(tiles, 1), dim3(S::kBlock), 0, stream, args);
  return hipGetLastError();
}

template <typename T, bool kScaled>
hipError_t dispatch_w(int W, const BlockArgs& args, hipStream_t stream) {
  switch (W) {
#define EXMY_CASE(w) \
  case w:            \
    return launch<T, w, kScaled>(args, stream);
    EXMY_CASE(1) EXMY_CASE(2) EXMY_CASE(3) EXMY_CASE(4) EXMY_CASE(5) EXMY_CASE(6) EXMY_CASE(7) EXMY_CASE(8)
    EXMY_CASE(9) EXMY_CASE(10) EXMY_CASE(11) EXMY_CASE(12) EXMY_CASE(13) EXMY_CASE(14) EXMY_CASE(15) EXMY_CASE(16)
#undef EXMY_CASE
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t encode_blocks_dispatch(exmy_dtype_t dt, int W, const BlockArgs& args, bool scaled, hipStream_t stream) {
  if (dt == EXMY_F16) return scaled ? dispatch_w<f16_t, true>(W, args, stream) : dispatch_w<f16_t, false>(W, args, stream);
  if (scaled)
    return dt == EXMY_F32 ? dispatch_w<float, true>(W, args, stream) : dispatch_w<uint16_t, true>(W, args, stream);
  return dt == EXMY_F32 ? dispatch_w<float, false>(W, args, stream) : dispatch_w<uint16_t, false>(W, args, stream);
}

}  // namespace exmy
