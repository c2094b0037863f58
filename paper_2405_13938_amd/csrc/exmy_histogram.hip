// Host-side dispatch of the exponent histogram kernels (see exmy_histogram_kernel.hpp).
#include "exmy_histogram_kernel.hpp"
#include "exmy_launch.hpp"

namespace exmy {

namespace {

// Launch shape, from a sweep on MI355X (1 GiB tensors).
constexpr int kBlock = 256;
constexpr int kUnroll = 4;
constexpr int kCopies = 32;
constexpr int kBlocksPerCU = 2;  // 4 measured 3-4 % slower: twice the blocks fold twice the bins into the same 256 global words at the end
constexpr bool kNT = true;

template <typename T>
hipError_t launch_histogram(const void* src, uint64_t n, uint64_t* hist, hipStream_t stream) {
  constexpr int kPer = 16 / sizeof(T);
  const uint64_t tile_vecs = (uint64_t)kBlock * kUnroll;
  const uint64_t tiles = (n / kPer + tile_vecs - 1) / tile_vecs;
  const uint32_t grid = grid_for_tiles(tiles, kBlocksPerCU);
  hipLaunchKernelGGL((hist::histogram_kernel<T, kBlock, kUnroll, kCopies, kNT>), dim3(grid), dim3(kBlock), 0, stream,
                     static_cast<const T*>(src), n, reinterpret_cast<unsigned long long*>(hist));
  return hipGetLastError();
}

}  // namespace

hipError_t histogram_dispatch(exmy_dtype_t dt, const void* src, uint64_t n, uint64_t* hist, hipStream_t stream) {
  if (dt == EXMY_F32) return launch_histogram<float>(src, n, hist, stream);
  if (dt == EXMY_F16) return launch_histogram<f16_t>(src, n, hist, stream);
  return launch_histogram<uint16_t>(src, n, hist, stream);
}

}  // namespace exmy
