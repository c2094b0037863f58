// Host-side dispatch of the emulation kernels (see exmy_emulate_kernel.hpp).
#include "exmy_emulate_kernel.hpp"
#include "exmy_launch.hpp"

namespace exmy {

namespace {

// Launch shape, from a sweep on MI355X (1 GiB tensors, rotating buffers).
constexpr int kBlock = 128;
constexpr int kUnroll = 1;
constexpr bool kNT = true;

template <typename T, bool kWide>
hipError_t launch_emulate(void* data, uint64_t n, const FormatConsts& fc, const TensorConsts& tc,
                          hipStream_t stream) {
  constexpr int kPer = 16 / sizeof(T);
  const uint64_t tile_vecs = (uint64_t)kBlock * kUnroll;
  const uint64_t tiles = (n / kPer + tile_vecs - 1) / tile_vecs;
  const dim3 grid = grid_for_flat_tiles(tiles, 1);
  hipLaunchKernelGGL((emu::emulate_kernel<T, kBlock, kUnroll, kWide, kNT>), grid, dim3(kBlock), 0, stream,
                     static_cast<T*>(data), n, fc, tc);
  return hipGetLastError();
}

}  // namespace

hipError_t emulate_dispatch(exmy_dtype_t dt, bool wide, void* data, uint64_t n, const FormatConsts& fc,
                            const TensorConsts& tc, hipStream_t stream) {
  if (dt == EXMY_F32)
    return wide ? launch_emulate<float, true>(data, n, fc, tc, stream)
                : launch_emulate<float, false>(data, n, fc, tc, stream);
  if (dt == EXMY_F16)
    return wide ? launch_emulate<f16_t, true>(data, n, fc, tc, stream)
                : launch_emulate<f16_t, false>(data, n, fc, tc, stream);
  return wide ? launch_emulate<uint16_t, true>(data, n, fc, tc, stream)
              : launch_emulate<uint16_t, false>(data, n, fc, tc, stream);
}

}  // namespace exmy
