// Host-side dispatch of the two's complement kernels (see exmy_int_kernel.hpp).
#include "exmy_int_kernel.hpp"
#include "exmy_launch.hpp"

namespace exmy {

namespace {

// Tile shapes of the sign-magnitude codec.
template <typename T>
struct Shape;
template <>
struct Shape<uint16_t> {
  static constexpr int kEncBlock = 64, kEncUnroll = 2, kDecBlock = 128, kDecUnroll = 2;
};
template <>
struct Shape<f16_t> : Shape<uint16_t> {};
template <>
struct Shape<float> {
  static constexpr int kEncBlock = 128, kEncUnroll = 1, kDecBlock = 256, kDecUnroll = 2;
};
constexpr int kEmuBlock = 128;

template <typename T, int W>
hipError_t launch_encode(const void* src, void* dst, uint64_t n, const IntConsts& ic, hipStream_t stream) {
  using S = Shape<T>;
  const uint64_t tile = (uint64_t)S::kEncBlock * S::kEncUnroll;
  const uint64_t tiles = (n / 8 + tile - 1) / tile;
  hipLaunchKernelGGL((twos::encode_int_kernel<T, W, S::kEncBlock, S::kEncUnroll>),
                     grid_for_flat_tiles(tiles, 1), dim3(S::kEncBlock), 0, stream, src, dst, n, ic);
  return hipGetLastError();
}

template <typename T, int W>
hipError_t launch_decode(const void* src, void* dst, uint64_t n, const IntConsts& ic, hipStream_t stream) {
  using S = Shape<T>;
  const uint64_t tile = (uint64_t)S::kDecBlock * S::kDecUnroll;
  const uint64_t tiles = (n / (16 / sizeof(T)) + tile - 1) / tile;
  hipLaunchKernelGGL((twos::decode_int_kernel<T, W, S::kDecBlock, S::kDecUnroll>),
                     grid_for_flat_tiles(tiles, 1), dim3(S::kDecBlock), 0, stream, src, dst, n, ic);
  return hipGetLastError();
}

template <typename T, bool kEncode>
hipError_t dispatch_w(int W, const void* src, void* dst, uint64_t n, const IntConsts& ic, hipStream_t stream) {
  switch (W) {
#define EXMY_CASE(w)                                                                   \
  case w:                                                                              \
    return kEncode ? launch_encode<T, w>(src, dst, n, ic, stream) : launch_decode<T, w>(src, dst, n, ic, stream);
    EXMY_CASE(2) EXMY_CASE(3) EXMY_CASE(4) EXMY_CASE(5) EXMY_CASE(6) EXMY_CASE(7) EXMY_CASE(8) EXMY_CASE(9)
    EXMY_CASE(10) EXMY_CASE(11) EXMY_CASE(12) EXMY_CASE(13) EXMY_CASE(14) EXMY_CASE(15) EXMY_CASE(16)
#undef EXMY_CASE
  }
  return hipErrorInvalidValue;
}

template <typename T>
hipError_t launch_emulate(void* data, uint64_t n, const IntConsts& ic, hipStream_t stream) {
  const uint64_t tiles = (n / (16 / sizeof(T)) + kEmuBlock - 1) / kEmuBlock;
  hipLaunchKernelGGL((twos::emulate_int_kernel<T, kEmuBlock>), grid_for_flat_tiles(tiles, 1),
                     dim3(kEmuBlock), 0, stream, data, n, ic);
  return hipGetLastError();
}

}  // namespace

hipError_t encode_int_dispatch(exmy_dtype_t dt, int W, const void* src, void* dst, uint64_t n, const IntConsts& ic,
                               hipStream_t stream) {
  if (dt == EXMY_F16) return dispatch_w<f16_t, true>(W, src, dst, n, ic, stream);
  return dt == EXMY_F32 ? dispatch_w<float, true>(W, src, dst, n, ic, stream)
                        : dispatch_w<uint16_t, true>(W, src, dst, n, ic, stream);
}

hipError_t decode_int_dispatch(exmy_dtype_t dt, int W, const void* src, void* dst, uint64_t n, const IntConsts& ic,
                               hipStream_t stream) {
  if (dt == EXMY_F16) return dispatch_w<f16_t, false>(W, src, dst, n, ic, stream);
  return dt == EXMY_F32 ? dispatch_w<float, false>(W, src, dst, n, ic, stream)
                        : dispatch_w<uint16_t, false>(W, src, dst, n, ic, stream);
}

hipError_t emulate_int_dispatch(exmy_dtype_t dt, void* data, uint64_t n, const IntConsts& ic, hipStream_t stream) {
  if (dt == EXMY_F16) return launch_emulate<f16_t>(data, n, ic, stream);
  return dt == EXMY_F32 ? launch_emulate<float>(data, n, ic, stream) : launch_emulate<uint16_t>(data, n, ic, stream);
}

}  // namespace exmy
