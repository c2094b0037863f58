// Host-side dispatch of the one-pass metadata + encode kernels (see exmy_encode_kernel.hpp).
#include "exmy_encode_kernel.hpp"
#include "exmy_launch.hpp"

namespace exmy {

namespace {

// Blocks of up to 64 groups (a power of two): flat tiles of the encoder's shape.
template <typename T>
struct Small;
template <>
struct Small<uint16_t> {
  static constexpr int kBlock = 64, kUnroll = 4;
};
template <>
struct Small<f16_t> : Small<uint16_t> {};
template <>
struct Small<float> {
  static constexpr int kBlock = 128, kUnroll = 1;
};

// Longer blocks: a workgroup per block, sized so that the block fills at least half of it, every lane holding
// kLoadsPerLane 16-byte loads in registers; blocks beyond 256 x kLoadsPerLane loads stay in a 256-lane
// workgroup with 8 or 16 loads per lane (measured: more lanes per workgroup instead are slower).
constexpr int kLoadsPerLane = 4;
// Longer blocks still: the workgroup walks the block twice, the second time out of the L2 cache (workgroups of
// 512 x 16 or 1024 x 8 register-held loads were measured no faster).
constexpr uint64_t kMaxTwoPassLoads = 8192;  // 128 KiB per block; beyond, two launches are as fast

template <typename T, int W, int kBlock, int kLoads>
hipError_t launch_team(const BlockArgs& args, hipStream_t stream) {
  constexpr int kUnroll = kLoads / (sizeof(T) == 4 ? 2 : 1);
  hipLaunchKernelGGL((enc::encode_blocks_auto_team_kernel<T, W, kBlock, kUnroll, true>),
                     grid_for_flat_tiles(args.n_blocks, 1), dim3(kBlock), 0, stream, args);
  return hipGetLastError();
}

template <typename T, int W>
hipError_t launch(BlockArgs args, hipStream_t stream) {
  constexpr uint32_t kGroupLoads = sizeof(T) == 4 ? 2 : 1;
  args.bi = make_block_index(args.block_groups);
  if (args.bi.log2 != kNotPow2 && args.block_groups <= 64) {
    using S = Small<T>;
    const uint64_t tile = (uint64_t)S::kBlock * S::kUnroll;
    const uint64_t tiles = ((args.n + 7) / 8 + tile - 1) / tile;
    hipLaunchKernelGGL((enc::encode_blocks_auto_small_kernel<T, W, S::kBlock, S::kUnroll, true>),
                       grid_for_flat_tiles(tiles, 1), dim3(S::kBlock), 0, stream, args);
    return hipGetLastError();
  }
  const uint64_t loads = (uint64_t)args.block_groups * kGroupLoads;  // 16-byte loads per block
  if (loads <= 64 * 2) return launch_team<T, W, 64, 2>(args, stream);
  if (loads <= 64 * kLoadsPerLane) return launch_team<T, W, 64, kLoadsPerLane>(args, stream);
  if (loads <= 128 * kLoadsPerLane) return launch_team<T, W, 128, kLoadsPerLane>(args, stream);
  // the 192-lane forms are there for rows of 5504 and 11008 elements, which would idle a third of the next
  // power of two (-10 to -15 % for bf16; with 16 loads per lane, rows of 22016, the idle third costs nothing)
  if (loads <= 192 * kLoadsPerLane) return launch_team<T, W, 192, kLoadsPerLane>(args, stream);
  if (loads <= 256 * kLoadsPerLane) return launch_team<T, W, 256, kLoadsPerLane>(args, stream);
  if (loads <= 192 * 8) return launch_team<T, W, 192, 8>(args, stream);
  if (loads <= 256 * 8) return launch_team<T, W, 256, 8>(args, stream);
  if (loads <= 256 * 16) return launch_team<T, W, 256, 16>(args, stream);
  if (loads <= kMaxTwoPassLoads) {
    constexpr int kUnroll = sizeof(T) == 4 ? 1 : 2;
    hipLaunchKernelGGL((enc::encode_blocks_auto_twopass_kernel<T, W, 256, kUnroll, true>),
                       grid_for_flat_tiles(args.n_blocks, 1), dim3(256), 0, stream, args);
    return hipGetLastError();
  }
  return hipErrorNotSupported;  // the caller falls back to two launches
}

template <typename T>
hipError_t dispatch_w(int W, const BlockArgs& args, hipStream_t stream) {
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

bool encode_blocks_auto_fits(exmy_dtype_t dt, uint32_t block_groups) {
  const uint64_t loads = (uint64_t)block_groups * (dt == EXMY_F32 ? 2 : 1);
  const bool pow2 = (block_groups & (block_groups - 1)) == 0;
  if (pow2 && block_groups <= 64) return true;
  return block_groups > 64 && loads <= kMaxTwoPassLoads;  // short odd-sized blocks would idle most of a workgroup
}

hipError_t encode_blocks_auto_dispatch(exmy_dtype_t dt, int W, const BlockArgs& args, hipStream_t stream) {
  if (dt == EXMY_F16) return dispatch_w<f16_t>(W, args, stream);
  return dt == EXMY_F32 ? dispatch_w<float>(W, args, stream) : dispatch_w<uint16_t>(W, args, stream);
}

}  // namespace exmy
