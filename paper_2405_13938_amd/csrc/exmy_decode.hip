// Host-side dispatch of the fused decode kernels (see exmy_decode_kernel.hpp).
#include "exmy_decode_kernel.hpp"
#include "exmy_launch.hpp"

namespace exmy {

namespace {

// Launch shapes (lanes per workgroup, 16-byte units per lane, whole tiles through an LDS image or not), from a
// sweep on MI355X over 1 GiB tensors of every width: what a lane reads of each plane is so little (1-16 bytes per
// unit) that the best shape follows the plane mix rather than the output, by up to 17 % (fp32 at 1 bit).
struct Shape {
  int block, unroll;
  bool stage;
};
template <typename T>
constexpr Shape shape_of(int W) {
  if (sizeof(T) == 4) {
    if (W <= 2) return {256, 1, false};
    if (W == 3) return {1024, 2, false};
    if (W <= 15) return {512, 2, false};
    if (W == 16) return {1024, 1, false};
    return {256, 2, false};
  }
  if (W == 1) return {256, 1, false};
  if (W == 2) return {256, 4, false};
  if (W == 3) return {256, 2, true};  // 2-bit and 1-bit planes: +7 % through the image
  if (W <= 7) return {512, 2, false};
  if (W <= 10 || W == 16) return {128, 2, false};
  return {256, 1, false};
}

template <typename T, int W>
hipError_t launch_decode(bool x8, const BatchArgs& args, uint64_t n_max, hipStream_t stream) {
  constexpr uint64_t E = 16 / sizeof(T);  // a unit = one lane's 16 bytes of output
  constexpr Shape S = shape_of<T>(W);
  const uint64_t units = (n_max + E - 1) / E;  // the elements after the last whole unit included
  const uint64_t tile_units = (uint64_t)S.block * S.unroll;
  const dim3 grid = grid_for_flat_tiles((units + tile_units - 1) / tile_units, args.count);
  if constexpr (W >= 9) {  // X = 8 needs at least 9 bits
    if (x8) {
      hipLaunchKernelGGL((dec::decode_kernel<T, W, S.block, S.unroll, true, true, S.stage>), grid, dim3(S.block), 0, stream, args);
      return hipGetLastError();
    }
  }
  hipLaunchKernelGGL((dec::decode_kernel<T, W, S.block, S.unroll, false, true, S.stage>), grid, dim3(S.block), 0, stream, args);
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
