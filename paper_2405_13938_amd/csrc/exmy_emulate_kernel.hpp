// In-place emulation (Section 2.1): every element is replaced by the eXmY value
// nearest to it, kept in its own type; NaN and Inf are left untouched.
//
// One lane handles 16-byte vectors; a tile is kBlock * kUnroll vectors, one block
// per tile, launched in address order (see the encoder for why).
#pragma once

#include "exmy_common.hpp"

namespace exmy {
namespace emu {

// fp32 bits of the emulated value of the element with fp32-position bits u.
//
// Same rounding as the encoder (magic addend with the ulp of the target
// quantum), but the rounded magnitude is recovered as a float by subtracting
// the addend again instead of being re-biased into a code.
template <bool kWide>
__device__ __forceinline__ uint32_t emulate_bits(uint32_t u, const FormatConsts& fc, const TensorConsts& tc) {
  const uint32_t a0 = u & 0x7FFFFFFFu;
  const uint32_t a = min(a0, tc.sat_bits);
  const uint32_t te = max(a, tc.emin_bits) & 0x7F800000u;
  uint32_t r;
  if constexpr (!kWide) {
    const float m = as_f32(te) * fc.magic_scale;
    const float s = as_f32(a) + m;
    r = as_u32(s - m);
  } else {
    const uint32_t hi = ((te >> 23) + (uint32_t)fc.wide_exp) << 20;
    const double m = __hiloint2double((int)hi, 0);
    const double s = (double)as_f32(a) + m;
    r = as_u32((float)(s - m));
  }
  r |= u & 0x80000000u;
  return a0 >= 0x7F800000u ? u : r;  // Inf / NaN pass through
}

template <typename T, bool kWide>
__device__ __forceinline__ uint4 emulate_vector(uint4 v, const FormatConsts& fc, const TensorConsts& tc) {
  uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    if constexpr (sizeof(T) == 4) {
      w[k] = emulate_bits<kWide>(w[k], fc, tc);
    } else {
      const uint32_t lo = emulate_bits<kWide>(w[k] << 16, fc, tc);
      const uint32_t hi = emulate_bits<kWide>(w[k] & 0xFFFF0000u, fc, tc);
      w[k] = __builtin_amdgcn_perm(hi, lo, 0x07060302u);
    }
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

template <typename T, int kBlock, int kUnroll, bool kWide, bool kNT>
__global__ __launch_bounds__(kBlock) void emulate_kernel(T* __restrict__ data, uint64_t n, FormatConsts fc,
                                                          TensorConsts tc) {
  constexpr int kPer = 16 / sizeof(T);  // elements per 16-byte vector
  constexpr uint32_t TV = kBlock * kUnroll;
  static_assert(TV * kPer >= 512, "tile counts must fit 32 bits for n <= 2^40");
  const uint64_t V = n / kPer;  // whole vectors
  const uint32_t full_tiles = (uint32_t)(V / TV);
  const uint32_t rem = (uint32_t)(V - (uint64_t)full_tiles * TV);
  const uint32_t tiles = full_tiles + (rem ? 1u : 0u);
  const uint32_t lane_off = threadIdx.x * 16;

  for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const rsrc_t buf = make_rsrc(reinterpret_cast<uint4*>(data) + (uint64_t)tile * TV);
    uint4 v[kUnroll];
    if (tile < full_tiles) {
#pragma unroll
      for (int r = 0; r < kUnroll; ++r) v[r] = load16<kNT>(buf, lane_off, r * kBlock * 16);
#pragma unroll
      for (int r = 0; r < kUnroll; ++r) store16<kNT>(buf, lane_off, r * kBlock * 16, emulate_vector<T, kWide>(v[r], fc, tc));
    } else {
#pragma unroll
      for (int r = 0; r < kUnroll; ++r)
        if (r * kBlock + threadIdx.x < rem) v[r] = load16<kNT>(buf, lane_off, r * kBlock * 16);
#pragma unroll
      for (int r = 0; r < kUnroll; ++r)
        if (r * kBlock + threadIdx.x < rem)
          store16<kNT>(buf, lane_off, r * kBlock * 16, emulate_vector<T, kWide>(v[r], fc, tc));
    }
  }

  // Elements past the last whole 16-byte vector.
  if (blockIdx.x == 0 && threadIdx.x < kPer) {
    const uint64_t i = V * kPer + threadIdx.x;
    if (i < n) {
      if constexpr (sizeof(T) == 4) {
        uint32_t* p = reinterpret_cast<uint32_t*>(data) + i;
        *p = emulate_bits<kWide>(*p, fc, tc);
      } else {
        uint16_t* p = reinterpret_cast<uint16_t*>(data) + i;
        *p = (uint16_t)(emulate_bits<kWide>((uint32_t)*p << 16, fc, tc) >> 16);
      }
    }
  }
}

}  // namespace emu
}  // namespace exmy
