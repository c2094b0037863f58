// W = 32: e8m23, the fp32 layout itself (Table 1 lists e8mY as fp32 / bf16 with fewer
// mantissa bits; max_exp is 255, the identity exponent map).  The power-of-2
// decomposition (Section 2.2.2) has the single segment 32, whose 32-byte group word is
// the group's 8 codes in element order: the packed form is the array of codes, padded
// with zero codes to a whole group.  A code is the element's own bit pattern unless the
// element is Inf / NaN, which take the largest finite magnitude under their sign (all
// codes are finite); a code with exponent field 255 decodes to that same value.  Encode
// and decode are therefore one function of 32-bit words.
#include "exmy_launch.hpp"

namespace exmy {

namespace {

__device__ __forceinline__ uint32_t finite_code(uint32_t u) { return (u & 0x80000000u) | min(u & 0x7FFFFFFFu, 0x7F7FFFFFu); }

// Grid: x strides over tiles of kBlock * kUnroll 16-byte vectors, y = tensor of the batch.
// n_out: words to write (encode: n rounded up to a whole group; decode: n).
template <int kBlock, int kUnroll, bool kDecode>
__global__ __launch_bounds__(kBlock) void codes32_kernel(const BatchArgs batch) {
  constexpr uint32_t TV = kBlock * kUnroll;
  const TensorArgs& ta = batch.t[blockIdx.y];
  const uint64_t n = ta.n;
  const uint64_t V = n / 4;  // whole vectors of input
  const uint32_t tiles = (uint32_t)((V + TV - 1) / TV);
  const uint32_t lane_off = threadIdx.x * 16;
  for (uint32_t tile = flat_tile(), once = 1; once && tile < tiles; once = 0) {
    const uint64_t v0 = (uint64_t)tile * TV;
    const rsrc_t in = make_rsrc(static_cast<const uint4*>(ta.src) + v0);
    const rsrc_t out = make_rsrc(static_cast<uint4*>(ta.dst) + v0);
    const uint64_t left = V - v0;
    const uint32_t rem = left < TV ? (uint32_t)left : TV;
    uint4 v[kUnroll];
#pragma unroll
    for (int r = 0; r < kUnroll; ++r)
      if (r * kBlock + threadIdx.x < rem) v[r] = load16<true>(in, lane_off, r * kBlock * 16);
#pragma unroll
    for (int r = 0; r < kUnroll; ++r)
      if (r * kBlock + threadIdx.x < rem)
        store16<true>(out, lane_off, r * kBlock * 16,
                      make_uint4(finite_code(v[r].x), finite_code(v[r].y), finite_code(v[r].z), finite_code(v[r].w)));
  }
  // The words after the last whole vector: the rest of the tensor and, for encode, the zero codes that
  // complete the last group.
  if (flat_tile() == 0 && threadIdx.x < 8) {
    const uint64_t i = V * 4 + threadIdx.x;
    const uint64_t end = kDecode ? n : (n + 7) / 8 * 8;
    if (i < end) static_cast<uint32_t*>(ta.dst)[i] = i < n ? finite_code(static_cast<const uint32_t*>(ta.src)[i]) : 0u;
  }
}

// Launch shape, from a sweep of workgroup size x vectors per lane on 1 GiB: the smallest workgroup with one
// vector per lane copies fastest (6.75 TB/s; 256 lanes x 2 vectors: 5.97).
constexpr int kBlock = 64;
constexpr int kUnroll = 1;

}  // namespace

hipError_t codes32_dispatch(bool decode, const BatchArgs& args, uint64_t n_max, hipStream_t stream) {
  const uint64_t tiles = (n_max / 4 + kBlock * kUnroll - 1) / (kBlock * kUnroll);
  const dim3 grid = grid_for_flat_tiles(tiles, args.count);
  if (decode)
    hipLaunchKernelGGL((codes32_kernel<kBlock, kUnroll, true>), grid, dim3(kBlock), 0, stream, args);
  else
    hipLaunchKernelGGL((codes32_kernel<kBlock, kUnroll, false>), grid, dim3(kBlock), 0, stream, args);
  return hipGetLastError();
}

}  // namespace exmy
