// Host-side dispatch of the fused encode kernels (see exmy_encode_kernel.hpp).
#include "exmy_encode_kernel.hpp"
#include "exmy_launch.hpp"

namespace exmy {

namespace {

// Launch shapes, from a sweep of block size x groups per lane x tiles per block x
// non-temporal loads on MI355X over 32 MiB, 86 MiB and 1 GiB tensors (back-to-back
// launches on rotating buffers): one tile per block, two bf16 groups or one fp32
// group per lane.  The histogram variant uses large resident blocks that walk chunks
// of 8 tiles and fold their LDS bins into the global bins once, at the end.
constexpr int kHistBlocksPerCU = 2;

template <typename T, bool kHist>
struct Shape;
template <bool kHist>
struct Shape<uint16_t, kHist> {
  static constexpr int kBlock = kHist ? 512 : 64;
  static constexpr int kUnroll = 2;
  static constexpr int kChunk = kHist ? 8 : 1;
  static constexpr bool kNT = true;
};
template <bool kHist>
struct Shape<f16_t, kHist> : Shape<uint16_t, kHist> {};
template <bool kHist>
struct Shape<float, kHist> {
  static constexpr int kBlock = kHist ? 512 : 64;
  static constexpr int kUnroll = kHist ? 2 : 1;
  static constexpr int kChunk = kHist ? 8 : 1;
  static constexpr bool kNT = true;
};

template <typename T, int W, bool kWide, bool kHist>
hipError_t launch_encode(const BatchArgs& args, uint64_t n_max, hipStream_t stream) {
  using S = Shape<T, kHist>;
  const uint64_t tile_groups = (uint64_t)S::kBlock * S::kUnroll;
  if constexpr (!kHist) {  // one tile per workgroup: the loop-free kernel
    static_assert(S::kChunk == 1, "the flat kernel takes one tile per workgroup");
    const uint64_t tiles = ((n_max + 7) / 8 + tile_groups - 1) / tile_groups;  // the ragged last group included
    hipLaunchKernelGGL((enc::encode_flat_kernel<T, W, S::kBlock, S::kUnroll, kWide, S::kNT>),
                       grid_for_flat_tiles(tiles, args.count), dim3(S::kBlock), 0, stream, args);
    return hipGetLastError();
  } else {
    const uint64_t tiles = (n_max / 8 + tile_groups - 1) / tile_groups;
    // Every workgroup ends by folding its non-empty bins into the same 256 global words, and those additions
    // queue up behind each other (about 1.25 ns each): with a workgroup per chunk a 1 GiB tensor would make 90 000
    // of them, as long as the conversion itself.  Two resident workgroups per compute unit stride over the chunks
    // instead and fold once each (+8-10 %; one per unit is too few to hide the loads, 3-6 measured the same as 2).
    uint32_t gx = grid_for_chunks(tiles, S::kChunk, S::kBlock);
    const uint32_t resident = (uint32_t)compute_units() * kHistBlocksPerCU;
    if (gx > resident) gx = resident;
    const dim3 grid(gx, args.count);
    hipLaunchKernelGGL((enc::encode_kernel<T, W, S::kBlock, S::kUnroll, S::kChunk, kWide, kHist, S::kNT>), grid,
                       dim3(S::kBlock), 0, stream, args);
    return hipGetLastError();
  }
}

template <typename T, bool kWide, bool kHist>
hipError_t dispatch_w(int W, const BatchArgs& args, uint64_t n_max, hipStream_t stream) {
  switch (W) {
#define EXMY_CASE(w) \
  case w:            \
    return launch_encode<T, w, kWide, kHist>(args, n_max, stream);
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

hipError_t encode_dispatch(exmy_dtype_t dt, int W, bool wide, bool with_hist, const BatchArgs& args, uint64_t n_max,
                           hipStream_t stream) {
  if (dt == EXMY_F32) {
    if (with_hist) return wide ? dispatch_w<float, true, true>(W, args, n_max, stream)
                               : dispatch_w<float, false, true>(W, args, n_max, stream);
    return wide ? dispatch_w<float, true, false>(W, args, n_max, stream)
                : dispatch_w<float, false, false>(W, args, n_max, stream);
  }
  if (dt == EXMY_F16) {
    if (with_hist) return wide ? dispatch_w<f16_t, true, true>(W, args, n_max, stream)
                               : dispatch_w<f16_t, false, true>(W, args, n_max, stream);
    return wide ? dispatch_w<f16_t, true, false>(W, args, n_max, stream)
                : dispatch_w<f16_t, false, false>(W, args, n_max, stream);
  }
  if (with_hist) return wide ? dispatch_w<uint16_t, true, true>(W, args, n_max, stream)
                             : dispatch_w<uint16_t, false, true>(W, args, n_max, stream);
  return wide ? dispatch_w<uint16_t, true, false>(W, args, n_max, stream)
              : dispatch_w<uint16_t, false, false>(W, args, n_max, stream);
}

}  // namespace exmy
