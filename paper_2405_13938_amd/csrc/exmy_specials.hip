// Host-side dispatch of the kernels with reserved NaN / Inf code points (see exmy_specials_kernel.hpp).
#include "exmy_launch.hpp"
#include "exmy_specials_kernel.hpp"

namespace exmy {

namespace {

// Tile shapes of the per-tensor codec.
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
  static constexpr int kEncBlock = 64, kEncUnroll = 1, kDecBlock = 256, kDecUnroll = 2;
};

template <typename T, int W>
hipError_t launch(bool decode, bool wide, const void* src, void* dst, uint64_t n, const FormatConsts& fc,
                  const TensorConsts& tc, const SpecialConsts& sc, hipStream_t stream) {
  using S = Shape<T>;
  if (decode) {
    const uint64_t tile = (uint64_t)S::kDecBlock * S::kDecUnroll;
    const uint64_t tiles = (n / (16 / sizeof(T)) + tile - 1) / tile;
    hipLaunchKernelGGL((spec::decode_specials_kernel<T, W, S::kDecBlock, S::kDecUnroll>),
                       grid_for_flat_tiles(tiles, 1), dim3(S::kDecBlock), 0, stream, src, dst, n, fc, tc, sc);
    return hipGetLastError();
  }
  const uint64_t tile = (uint64_t)S::kEncBlock * S::kEncUnroll;
  const uint64_t tiles = (n / 8 + tile - 1) / tile;
  const dim3 grid = grid_for_flat_tiles(tiles, 1), block(S::kEncBlock);
  if (wide)
    hipLaunchKernelGGL((spec::encode_specials_kernel<T, W, S::kEncBlock, S::kEncUnroll, true>), grid, block, 0, stream, src, dst, n, fc, tc, sc);
  else
    hipLaunchKernelGGL((spec::encode_specials_kernel<T, W, S::kEncBlock, S::kEncUnroll, false>), grid, block, 0, stream, src, dst, n, fc, tc, sc);
  return hipGetLastError();
}

template <typename T>
hipError_t dispatch_w(int W, bool decode, bool wide, const void* src, void* dst, uint64_t n, const FormatConsts& fc,
                      const TensorConsts& tc, const SpecialConsts& sc, hipStream_t stream) {
  switch (W) {
#define EXMY_CASE(w) \
  case w:            \
    return launch<T, w>(decode, wide, src, dst, n, fc, tc, sc, stream);
    EXMY_CASE(2) EXMY_CASE(3) EXMY_CASE(4) EXMY_CASE(5) EXMY_CASE(6) EXMY_CASE(7) EXMY_CASE(8) EXMY_CASE(9)
    EXMY_CASE(10) EXMY_CASE(11) EXMY_CASE(12) EXMY_CASE(13) EXMY_CASE(14) EXMY_CASE(15) EXMY_CASE(16)
#undef EXMY_CASE
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t specials_dispatch(exmy_dtype_t dt, int W, bool decode, bool wide, const void* src, void* dst, uint64_t n,
                             const FormatConsts& fc, const TensorConsts& tc, const SpecialConsts& sc,
                             hipStream_t stream) {
  if (dt == EXMY_F16) return dispatch_w<f16_t>(W, decode, wide, src, dst, n, fc, tc, sc, stream);
  return dt == EXMY_F32 ? dispatch_w<float>(W, decode, wide, src, dst, n, fc, tc, sc, stream)
                        : dispatch_w<uint16_t>(W, decode, wide, src, dst, n, fc, tc, sc, stream);
}

}  // namespace exmy
