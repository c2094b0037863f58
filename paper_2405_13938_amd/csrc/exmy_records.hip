// Host-side dispatch of the record-layout kernels (see exmy_records_kernel.hpp).
#include "exmy_launch.hpp"
#include "exmy_records_kernel.hpp"

namespace exmy {

namespace {

template <typename T>
struct Shape {
  static constexpr int kBlock = 128;
  static constexpr int kUnroll = sizeof(T) == 4 ? 1 : 2;
};

template <typename T, int W>
hipError_t launch(bool decode, bool flag, const void* src, void* dst, uint64_t n, const FormatConsts& fc,
                  const TensorConsts& tc, hipStream_t stream) {
  using S = Shape<T>;
  const uint64_t tile_groups = (uint64_t)S::kBlock * S::kUnroll;
  const uint64_t tiles = ((n + 7) / 8 + tile_groups - 1) / tile_groups;
  const dim3 grid = grid_for_flat_tiles(tiles, 1), block(S::kBlock);
  if (decode) {  // flag: X = 8
    const uint8_t* s = static_cast<const uint8_t*>(src);
    T* d = static_cast<T*>(dst);
    if (flag)
      hipLaunchKernelGGL((rec::decode_records_kernel<T, W, S::kBlock, S::kUnroll, true>), grid, block, 0, stream, s, d, n, fc, tc);
    else
      hipLaunchKernelGGL((rec::decode_records_kernel<T, W, S::kBlock, S::kUnroll, false>), grid, block, 0, stream, s, d, n, fc, tc);
  } else {  // flag: the fp64 rounding path
    uint8_t* d = static_cast<uint8_t*>(dst);
    if (flag)
      hipLaunchKernelGGL((rec::encode_records_kernel<T, W, S::kBlock, S::kUnroll, true>), grid, block, 0, stream, src, d, n, fc, tc);
    else
      hipLaunchKernelGGL((rec::encode_records_kernel<T, W, S::kBlock, S::kUnroll, false>), grid, block, 0, stream, src, d, n, fc, tc);
  }
  return hipGetLastError();
}

template <typename T>
hipError_t dispatch_w(int W, bool decode, bool flag, const void* src, void* dst, uint64_t n, const FormatConsts& fc,
                      const TensorConsts& tc, hipStream_t stream) {
  switch (W) {  // 8 and 16 have a single plane: their records are the planar form, which the caller uses
#define EXMY_CASE(w) \
  case w:            \
    return launch<T, w>(decode, flag, src, dst, n, fc, tc, stream);
    EXMY_CASE(1) EXMY_CASE(2) EXMY_CASE(3) EXMY_CASE(4) EXMY_CASE(5) EXMY_CASE(6) EXMY_CASE(7)
    EXMY_CASE(9) EXMY_CASE(10) EXMY_CASE(11) EXMY_CASE(12) EXMY_CASE(13) EXMY_CASE(14) EXMY_CASE(15)
#undef EXMY_CASE
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t records_dispatch(exmy_dtype_t dt, int W, bool decode, bool flag, const void* src, void* dst, uint64_t n,
                            const FormatConsts& fc, const TensorConsts& tc, hipStream_t stream) {
  if (dt == EXMY_F16) return dispatch_w<f16_t>(W, decode, flag, src, dst, n, fc, tc, stream);
  return dt == EXMY_F32 ? dispatch_w<float>(W, decode, flag, src, dst, n, fc, tc, stream)
                        : dispatch_w<uint16_t>(W, decode, flag, src, dst, n, fc, tc, stream);
}

}  // namespace exmy
