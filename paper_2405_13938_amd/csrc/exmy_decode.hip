// Host-side dispatch of the fused decode kernels (see exmy_decode_kernel.hpp).
#include "exmy_decode_kernel.hpp"
#include "exmy_launch.hpp"

namespace exmy {

namespace {

// Launch shapes, from a sweep of block size x units per lane x tiles per block x
// non-temporal stores on MI355X over 32 MiB, 86 MiB and 1 GiB tensors.
template <typename T>
struct Shape;
template <>
struct Shape<uint16_t> {
  static constexpr int kBlock = 128;
  static constexpr int kUnroll = 2;
  static constexpr bool kNT = true;
};
template <>
struct Shape<f16_t> : Shape<uint16_t> {};
template <>
struct Shape<float> {
  static constexpr int kBlock = 256;
  static constexpr int kUnroll = 2;
  static constexpr bool kNT = true;
};

// W = 3 (2-bit and 1-bit planes): whole tiles pass through an LDS image, +7 % (bf16) to +10 % (fp32); at W = 1 and 2
// the image measured between -10 % and +5 %, from W = 5 up +-1 %.
struct StagedShape {
  static constexpr int kBlock = 256;
  static constexpr int kUnroll = 2;
};

template <typename T, int W>
hipError_t launch_decode(bool x8, const BatchArgs& args, uint64_t n_max, hipStream_t stream) {
  constexpr uint64_t E = 16 / sizeof(T);  // a unit = one lane's 16 bytes of output
  const uint64_t units = (n_max + E - 1) / E;  // the elements after the last whole unit included
  if constexpr (W == 3) {
    using S = StagedShape;
    const uint64_t tile_units = (uint64_t)S::kBlock * S::kUnroll;
    hipLaunchKernelGGL((dec::decode_kernel<T, W, S::kBlock, S::kUnroll, false, true, true>),
                       grid_for_flat_tiles((units + tile_units - 1) / tile_units, args.count), dim3(S::kBlock), 0, stream,
                       args);
    return hipGetLastError();
  }
  using S = Shape<T>;
  // Up to 7 bits a lane reads so little of each plane that a workgroup of the usual size touches only 128-512
  // bytes of the narrow ones: 512 lanes there (+4-7 % for bf16, +3-5 % for fp32 up to 6 bits; from 8 bits up the
  // larger workgroup measured 1-5 % slower).
  constexpr int kBlock = W <= 7 ? 512 : S::kBlock;
  const uint64_t tile_units = (uint64_t)kBlock * S::kUnroll;
  const dim3 grid = grid_for_flat_tiles((units + tile_units - 1) / tile_units, args.count);
  if constexpr (W >= 9) {  // X = 8 needs at least 9 bits
    if (x8) {
      hipLaunchKernelGGL((dec::decode_kernel<T, W, kBlock, S::kUnroll, true, S::kNT>), grid, dim3(kBlock), 0, stream, args);
      return hipGetLastError();
    }
  }
  hipLaunchKernelGGL((dec::decode_kernel<T, W, kBlock, S::kUnroll, false, S::kNT>), grid, dim3(kBlock), 0, stream, args);
  return hipGetLastError();
}

template <typename T>
hipError_t dispatch_w(int W, bool x8, const BatchArgs& args, uint64_t n_max, hipStream_t stream) {
  switch (W) {
#define EXMY_CASE(w) \
  case w:            \
    return launch_decode<T, w>(x8, args, n_max, stream);
    EXMY_CASE(1) EXMY_CASE(2) EXMY_CASE(3) EXMY_CASE(4) EXMY_CASE(5) EXMY_CASE(6) EXMY_CASE(7) EXMY_CASE(8)
    EXMY_CASE(9) EXMY_CASE(10) EXMY_CASE(11) EXMY_CASE(12) EXMY_CASE(13) EXMY_CASE(14) EXMY_CASE(15) EXMY_CASE(16)
  }
  if constexpr (sizeof(T) == 4) {  // only fp32 holds formats wider than 16 bits
    switch (W) {
      EXMY_CASE(17) EXMY_CASE(18) EXMY_CASE(19) EXMY_CASE(20) EXMY_CASE(21) EXMY_CASE(22) EXMY_CASE(23) EXMY_CASE(24)
      EXMY_CASE(25) EXMY_CASE(26) EXMY_CASE(27) EXMY_CASE(28) EXMY_CASE(29) EXMY_CASE(30) EXMY_CASE(31)
    }
  }
#undef EXMY_CASE
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t decode_dispatch(exmy_dtype_t dt, int W, bool x8, const BatchArgs& args, uint64_t n_max,
                           hipStream_t stream) {
  if (dt == EXMY_F32) return dispatch_w<float>(W, x8, args, n_max, stream);
  if (dt == EXMY_F16) return dispatch_w<f16_t>(W, x8, args, n_max, stream);
  return dispatch_w<uint16_t>(W, x8, args, n_max, stream);
}

}  // namespace exmy
