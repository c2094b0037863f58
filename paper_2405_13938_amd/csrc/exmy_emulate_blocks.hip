// Host-side dispatch of the per-block-metadata emulation and block-maximum-exponent
// kernels (see exmy_emulate_kernel.hpp).
#include "exmy_emulate_kernel.hpp"
#include "exmy_launch.hpp"

namespace exmy {

namespace {

constexpr int kBlock = 128;
constexpr int kUnroll = 1;

template <typename T, bool kScaled>
hipError_t launch_emulate(BlockArgs args, bool wide_format, hipStream_t stream) {
  constexpr uint64_t kVecsPerGroup = sizeof(T) == 4 ? 2 : 1;
  const uint64_t tile_vecs = (uint64_t)kBlock * kUnroll;
  const uint64_t tiles = (args.n / (16 / sizeof(T)) + tile_vecs - 1) / tile_vecs;
  args.bi = make_block_index(args.block_groups * kVecsPerGroup);
  hipLaunchKernelGGL((emu::emulate_blocks_kernel<T, kBlock, kUnroll, true, kScaled>), grid_for_flat_tiles(tiles, 1),
                     dim3(kBlock), 0, stream, args, wide_format);
  return hipGetLastError();
}

// Block maxima: the lanes of a wavefront combine blocks of up to 64 vectors (a
// power of two); blocks of up to kWaveRowVecs vectors get a wavefront each, longer
// ones a workgroup each.
constexpr int kMaxBlock = 256;
constexpr int kMaxUnroll = 4;
constexpr uint64_t kWaveRowVecs = 1024;

template <typename T, bool kScale>
hipError_t launch_max_exp(BlockArgs args, hipStream_t stream) {
  constexpr int kPer = 16 / sizeof(T);
  constexpr uint64_t kVecsPerGroup = sizeof(T) == 4 ? 2 : 1;
  args.bi = make_block_index(args.block_groups * kVecsPerGroup);
  if (args.bi.log2 != kNotPow2 && args.bi.size <= 64) {
    const uint64_t vecs = (args.n + kPer - 1) / kPer;
    const uint64_t tile_vecs = (uint64_t)kMaxBlock * kMaxUnroll;
    hipLaunchKernelGGL((emu::block_max_exp_small_kernel<T, kMaxBlock, kMaxUnroll, kScale>),
                       grid_for_flat_tiles((vecs + tile_vecs - 1) / tile_vecs, 1), dim3(kMaxBlock), 0,
                       stream, args);
  } else if (args.bi.size <= kWaveRowVecs) {
    constexpr int kTeams = kMaxBlock / 64;
    hipLaunchKernelGGL((emu::block_max_exp_team_kernel<T, kMaxBlock, 64, kScale>),
                       dim3(grid_for_chunks(args.n_blocks, kTeams, kMaxBlock)), dim3(kMaxBlock), 0, stream, args);
  } else {
    hipLaunchKernelGGL((emu::block_max_exp_team_kernel<T, kMaxBlock, kMaxBlock, kScale>),
                       dim3(grid_for_chunks(args.n_blocks, 1, kMaxBlock)), dim3(kMaxBlock), 0, stream, args);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t emulate_blocks_dispatch(exmy_dtype_t dt, const BlockArgs& args, bool wide_format, bool scaled,
                                   hipStream_t stream) {
  if (dt == EXMY_F16)
    return scaled ? launch_emulate<f16_t, true>(args, wide_format, stream)
                  : launch_emulate<f16_t, false>(args, wide_format, stream);
  if (scaled)
    return dt == EXMY_F32 ? launch_emulate<float, true>(args, wide_format, stream)
                          : launch_emulate<uint16_t, true>(args, wide_format, stream);
  return dt == EXMY_F32 ? launch_emulate<float, false>(args, wide_format, stream)
                        : launch_emulate<uint16_t, false>(args, wide_format, stream);
}

hipError_t block_max_exp_dispatch(exmy_dtype_t dt, const BlockArgs& args, bool scale, hipStream_t stream) {
  if (dt == EXMY_F16) return scale ? launch_max_exp<f16_t, true>(args, stream) : launch_max_exp<f16_t, false>(args, stream);
  if (scale)
    return dt == EXMY_F32 ? launch_max_exp<float, true>(args, stream) : launch_max_exp<uint16_t, true>(args, stream);
  return dt == EXMY_F32 ? launch_max_exp<float, false>(args, stream) : launch_max_exp<uint16_t, false>(args, stream);
}

}  // namespace exmy
