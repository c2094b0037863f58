// Reserved code points for NaN and Inf (Section 5: values encoded for training need
// an encoding for them, which the paper leaves open).  Two conventions, those of the
// float types in use: IEEE 754 style (the top exponent code is reserved: mantissa 0
// is Inf, anything else NaN) and NaN only (the all-ones magnitude code is NaN, there
// is no Inf).  Finite elements are rounded as always and saturate to the largest
// finite value, which the host passes as the format's saturation bound; a NaN takes
// the all-ones magnitude code under its own sign; Inf takes the Inf code, or (NaN
// only) saturates.  The kernels are the flat per-tensor ones; since Inf / NaN are rare,
// a wavefront first asks whether any of its lanes holds one (a maximum over the lane's
// elements and one ballot) and only then runs the two compares and two selects per
// element that place or read the reserved codes.
#pragma once

#include "exmy_common.hpp"
#include "exmy_decode_kernel.hpp"
#include "exmy_encode_kernel.hpp"

namespace exmy {

namespace spec {

template <int W, bool kWide, class Dst>
__device__ __forceinline__ void encode_group(const uint32_t u[8], const FormatConsts& fc, const TensorConsts& tc,
                                             const SpecialConsts& sc, const Dst& pd, uint32_t lane_group,
                                             uint32_t tile_group) {
  uint32_t f[8];
  uint32_t top = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    top = max(top, u[j] & 0x7FFFFFFFu);
    f[j] = magnitude_code_left<kWide>(u[j], fc, tc);  // Inf / NaN come out saturated: replaced below
  }
  if (__builtin_amdgcn_ballot_w64(top >= 0x7F800000u) != 0) {  // some lane of the wavefront holds an Inf or a NaN
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t a = u[j] & 0x7FFFFFFFu;
      f[j] = a == 0x7F800000u ? sc.inf_left : f[j];
      f[j] = a > 0x7F800000u ? sc.nan_left : f[j];
    }
  }
  if constexpr ((W & 1) == 0) {  // even W: the sign rides at bit 31
#pragma unroll
    for (int j = 0; j < 8; ++j) f[j] |= u[j] & 0x80000000u;
  }
  enc::peel_planes<W, Planes<W>::count - 1>(f, u, pd, lane_group, tile_group);
}

template <typename T, int W, int kBlock, int kUnroll, bool kWide>
__global__ __launch_bounds__(kBlock) void encode_specials_kernel(const void* src_v, void* dst_v, uint64_t n,
                                                                  FormatConsts fc, TensorConsts tc, SpecialConsts sc) {
  constexpr uint32_t TG = kBlock * kUnroll;
  constexpr int kLoads = enc::TileRegs<T, kUnroll>::kLoads;
  static_assert(TG >= 64, "tile counts must fit 32 bits for n <= 2^40");
  const uint4* __restrict__ src4 = static_cast<const uint4*>(src_v);
  uint8_t* __restrict__ dst = static_cast<uint8_t*>(dst_v);
  const uint64_t G = (n + 7) / 8;
  const uint64_t Gfull = n / 8;
  const uint32_t full_tiles = (uint32_t)(Gfull / TG);
  const uint32_t rem_groups = (uint32_t)(Gfull - (uint64_t)full_tiles * TG);
  const uint32_t tiles = full_tiles + (rem_groups ? 1u : 0u);
  __shared__ __align__(16) uint8_t lds_stage[TG * W];
  const enc::PlaneStage<W, TG> stage{lds_stage};

  for (uint32_t tile = flat_tile(), once = 1; once && tile < tiles; once = 0) {
    const uint64_t g0 = (uint64_t)tile * TG;
    const rsrc_t src = make_rsrc(src4 + g0 * kLoads);
    enc::TileRegs<T, kUnroll> regs;
    if (tile < full_tiles) {  // a whole tile leaves through the LDS image, in 16-byte pieces
      enc::load_tile<T, kBlock, kUnroll, true, false>(src, 0, 0, regs);
#pragma unroll
      for (int r = 0; r < kUnroll; ++r) {
        uint32_t u[8];
        enc::group_bits<T, true>(regs.v[r], u);
        encode_group<W, kWide>(u, fc, tc, sc, stage, enc::row_slot<T, kBlock>(), r * kBlock);
      }
      enc::flush_stage<W, TG, kBlock>(stage, dst, G, g0);
      continue;
    }
    enc::PlaneDst<W> pd;
    enc::make_plane_dst<W>(dst, G, g0, pd);
    enc::load_tile<T, kBlock, kUnroll, true, true>(src, 0, rem_groups, regs);
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      if (r * kBlock + threadIdx.x < rem_groups) {
        uint32_t u[8];
        enc::group_bits<T>(regs.v[r], u);
        encode_group<W, kWide>(u, fc, tc, sc, pd, threadIdx.x, r * kBlock);
      }
    }
  }

  // Ragged last group, padded with +0 (code 0).
  if (Gfull != G && flat_tile() == 0 && threadIdx.x == 0) {
    uint32_t u[8];
    enc::ragged_group_bits<T>(src_v, Gfull * 8, n, u);
    enc::PlaneDst<W> pd;
    enc::make_plane_dst<W>(dst, G, Gfull, pd);
    encode_group<W, kWide>(u, fc, tc, sc, pd, 0, 0);
  }
}

// fp32 bit patterns of the unit's E elements: a finite code as always, a reserved one as
// Inf or the quiet NaN 0x7FC00000, under the code's sign.
template <int W, int E>
__device__ __forceinline__ void unit_bits(const dec::UnitWords<W>& uw, const FormatConsts& fc, const TensorConsts& tc,
                                          const SpecialConsts& sc, uint32_t b[E]) {
  uint32_t g[E];
  uint32_t top = 0;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    g[j] = dec::add_fields<W, 0>(uw, j, tc.dec_bias, fc);
    top = max(top, g[j]);
  }
  if (__builtin_amdgcn_ballot_w64(top > sc.g_last) != 0) {  // some lane of the wavefront holds a reserved code
#pragma unroll
    for (int j = 0; j < E; ++j) {
      uint32_t mag = finish_magnitude(min(g[j], sc.g_last), tc);  // the clamp keeps NaN patterns (X = 8) out of the float ops
      mag = g[j] > sc.g_last ? 0x7FC00000u : mag;
      b[j] = g[j] == sc.g_inf ? 0x7F800000u : mag;
    }
  } else {
#pragma unroll
    for (int j = 0; j < E; ++j) b[j] = finish_magnitude(g[j], tc);
  }
  constexpr int PT = Planes<W>::count - 1;
  constexpr int ST = Planes<W>::seg(PT);
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const int bit = ST * j + ST - 1;  // the sign: top bit of the top plane's field
    const uint32_t sgn = uw.w[PT][bit / 32] << (31 - bit % 32);
    b[j] |= sgn & 0x80000000u;
  }
}

template <typename T, int W>
__device__ __forceinline__ void decode_unit(const dec::UnitWords<W>& uw, const FormatConsts& fc, const TensorConsts& tc,
                                            const SpecialConsts& sc, rsrc_t out, uint32_t lane_unit,
                                            uint32_t tile_unit) {
  constexpr int E = 16 / sizeof(T);
  uint32_t b[E];
  unit_bits<W, E>(uw, fc, tc, sc, b);
  if constexpr (sizeof(T) == 4) {
    store16<true>(out, lane_unit * 16, tile_unit * 16, make_uint4(b[0], b[1], b[2], b[3]));
  } else {
    // finite values are exact in the 16-bit type; Inf and the quiet NaN convert to its own Inf and quiet NaN
    // (fp16: by the hardware conversion; bf16: by taking the upper half)
    uint4 o;
    o.x = pack_elems<T, false>(b[0], b[1]);
    o.y = pack_elems<T, false>(b[2], b[3]);
    o.z = pack_elems<T, false>(b[4], b[5]);
    o.w = pack_elems<T, false>(b[6], b[7]);
    store16<true>(out, lane_unit * 16, tile_unit * 16, o);
  }
}

template <typename T, int W, int kBlock, int kUnroll>
__global__ __launch_bounds__(kBlock) void decode_specials_kernel(const void* src_v, void* dst_v, uint64_t n,
                                                                  FormatConsts fc, TensorConsts tc, SpecialConsts sc) {
  constexpr uint32_t TU = kBlock * kUnroll;
  constexpr int E = 16 / sizeof(T);
  static_assert(TU % 2 == 0 && TU * E >= 512, "tiles start on a byte of the 1-bit plane; tile counts fit 32 bits");
  const uint8_t* __restrict__ src = static_cast<const uint8_t*>(src_v);
  T* __restrict__ dst = static_cast<T*>(dst_v);
  const uint64_t G = (n + 7) / 8;
  const uint64_t Ufull = n / E;
  const uint32_t full_tiles = (uint32_t)(Ufull / TU);
  const uint32_t rem_units = (uint32_t)(Ufull - (uint64_t)full_tiles * TU);
  const uint32_t tiles = full_tiles + (rem_units ? 1u : 0u);

  for (uint32_t tile = flat_tile(), once = 1; once && tile < tiles; once = 0) {
    const uint64_t u0 = (uint64_t)tile * TU;
    dec::PlaneSrc<W> ps;
    dec::make_plane_src<W, E>(src, G, u0, ps);
    const rsrc_t out = make_rsrc(reinterpret_cast<uint4*>(dst) + u0);
    dec::TileWords<W, kUnroll> tw;
    if (tile < full_tiles) {
      dec::load_tile<W, E, kBlock, kUnroll, false>(ps, 0, 0, tw);
#pragma unroll
      for (int r = 0; r < kUnroll; ++r) decode_unit<T, W>(tw.u[r], fc, tc, sc, out, threadIdx.x, r * kBlock);
    } else {
      dec::load_tile<W, E, kBlock, kUnroll, true>(ps, 0, rem_units, tw);
#pragma unroll
      for (int r = 0; r < kUnroll; ++r)
        if (r * kBlock + threadIdx.x < rem_units) decode_unit<T, W>(tw.u[r], fc, tc, sc, out, threadIdx.x, r * kBlock);
    }
  }

  // The n % E elements after the last whole unit, one lane each.
  if (flat_tile() == 0 && threadIdx.x < E) {
    const uint64_t i = Ufull * E + threadIdx.x;
    if (i < n) {
      dec::PlaneSrc<W> ps;
      dec::make_plane_src<W, 8>(src, G, i / 8, ps);
      dec::UnitWords<W> uw;
      dec::load_unit<W, 8>(ps, 0, 0, uw);
      uint32_t all[8];  // the whole group that holds the element
      unit_bits<W, 8>(uw, fc, tc, sc, all);
      uint32_t b = 0;
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if ((int)(i % 8) == j) b = all[j];
      if constexpr (sizeof(T) == 4)
        reinterpret_cast<uint32_t*>(dst)[i] = b;
      else
        reinterpret_cast<uint16_t*>(dst)[i] = to_elem<T>(b);
    }
  }
}

}  // namespace spec
}  // namespace exmy
