// Host-side dispatch of the per-block-metadata emulation and block-maximum-exponent
// kernels (see exmy_emulate_kernel.hpp).
#include "exmy_emulate_kernel.hpp"
#include "exmy_launch.hpp"

namespace exmy {

namespace {

constexpr int kBlock = 128;
constexpr int kUnroll = 1;
static_assert(kBlock * kUnroll >= 2 * kSmallBlockGroups, "a tile holds whole small blocks");

template <typename T>
hipError_t launch_emulate(const BlockArgs& args, bool rows, bool wide_format, hipStream_t stream) {
  constexpr uint64_t kVecsPerGroup = sizeof(T) == 4 ? 2 : 1;
  const uint64_t tile_vecs = (uint64_t)kBlock * kUnroll;
  if (rows) {
    const uint64_t tiles = (args.block_groups * kVecsPerGroup + tile_vecs - 1) / tile_vecs;
    hipLaunchKernelGGL((emu::emulate_blocks_kernel<T, kBlock, kUnroll, true, true>),
                       grid_for_rows(tiles, args.n_blocks, kBlock), dim3(kBlock), 0, stream, args, wide_format);
  } else {
    const uint64_t tiles = (args.n / (16 / sizeof(T)) + tile_vecs - 1) / tile_vecs;
    hipLaunchKernelGGL((emu::emulate_blocks_kernel<T, kBlock, kUnroll, false, true>),
                       dim3(grid_for_chunks(tiles, 1, kBlock)), dim3(kBlock), 0, stream, args, wide_format);
  }
  return hipGetLastError();
}

// Block maxima: a wavefront's butterfly covers blocks of up to 64 vectors; longer
// blocks get a workgroup each.
constexpr int kMaxBlock = 256;

template <typename T>
hipError_t launch_max_exp(const BlockArgs& args, bool rows, hipStream_t stream) {
  constexpr int kPer = 16 / sizeof(T);
  constexpr uint64_t kVecsPerGroup = sizeof(T) == 4 ? 2 : 1;
  if (rows || args.block_groups * kVecsPerGroup > 64) {
    hipLaunchKernelGGL((emu::block_max_exp_kernel<T, kMaxBlock, true>), grid_for_rows(1, args.n_blocks, kMaxBlock),
                       dim3(kMaxBlock), 0, stream, args);
  } else {
    const uint64_t vecs = (args.n + kPer - 1) / kPer;
    const uint64_t blocks = (vecs + kMaxBlock - 1) / kMaxBlock;
    hipLaunchKernelGGL((emu::block_max_exp_kernel<T, kMaxBlock, false>), dim3(grid_for_chunks(blocks, 1, kMaxBlock)),
                       dim3(kMaxBlock), 0, stream, args);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t emulate_blocks_dispatch(exmy_dtype_t dt, const BlockArgs& args, bool rows, bool wide_format,
                                   hipStream_t stream) {
  return dt == EXMY_F32 ? launch_emulate<float>(args, rows, wide_format, stream)
                        : launch_emulate<uint16_t>(args, rows, wide_format, stream);
}

hipError_t block_max_exp_dispatch(exmy_dtype_t dt, const BlockArgs& args, bool rows, hipStream_t stream) {
  return dt == EXMY_F32 ? launch_max_exp<float>(args, rows, stream) : launch_max_exp<uint16_t>(args, rows, stream);
}

}  // namespace exmy
