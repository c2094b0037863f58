// Two's complement reading of the X = 0 formats (Section 2 "Format": e0m3 used as
// int4 represents [-8, 7]): the W = 1 + Y bits of a code are a two's complement
// integer k in [-2^Y, 2^Y - 1] and the value is k quanta, the quantum being that
// of e0mY with the same max_exp, 2^(max_exp + 1 - 127 - Y).
//
// Same tiles, loads, plane layout and launch order as the sign-magnitude codec;
// only the per-element arithmetic differs, and every plane (the 1-bit one of an
// odd W too) is peeled from the code itself.
#pragma once

#include "exmy_decode_kernel.hpp"
#include "exmy_encode_kernel.hpp"

namespace exmy {
namespace twos {

// k = round-half-even(|x| / quantum), clamped to 2^Y - 1 (x >= 0) or 2^Y (x < 0),
// as the fp32 bits of |x| + magic (k sits in the low Y + 1 bits): all magnitudes
// that survive the clamp lie under 2^emin8 or exactly on it, so one magic addend
// with the ulp of the quantum serves every element.  Inf / NaN patterns clamp
// like large values, to the side of their sign bit.
__device__ __forceinline__ float rounded_sum(uint32_t u, const IntConsts& ic) {
  const uint32_t smask = (uint32_t)((int32_t)u >> 31);
  const uint32_t sat = ic.sat_pos_bits + (smask & ic.neg_extra);  // negatives reach one quantum further
  const uint32_t a = min(u & 0x7FFFFFFFu, sat);
  return as_f32(a) + ic.magic;
}

// The code, left-aligned in 32 bits (two's complement in the top W bits, zeros below).
__device__ __forceinline__ uint32_t code_left(uint32_t u, const IntConsts& ic) {
  const uint32_t kl = as_u32(rounded_sum(u, ic)) << ic.left_shift;  // keeps the low W = Y + 1 bits of the sum
  const uint32_t smask = (uint32_t)((int32_t)u >> 31);
  return (kl ^ smask) - smask;                                       // negate where the sign bit is set
}

template <int W, int P, class Dst>
__device__ __forceinline__ void peel_all(uint32_t f[8], const Dst& pd, uint32_t lane_group, uint32_t tile_group) {
  constexpr int S = Planes<W>::seg(P);
  uint32_t word[4];
  enc::plane_word_from_top<S>(f, word);
  enc::put_plane_word<W, P>(pd, lane_group, tile_group, word);
  if constexpr (P > 0) {
#pragma unroll
    for (int j = 0; j < 8; ++j) f[j] <<= S;
    peel_all<W, P - 1>(f, pd, lane_group, tile_group);
  }
}

template <int W, class Dst>
__device__ __forceinline__ void encode_group(const uint32_t u[8], const IntConsts& ic, const Dst& pd,
                                             uint32_t lane_group, uint32_t tile_group) {
  uint32_t f[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) f[j] = code_left(u[j], ic);
  peel_all<W, Planes<W>::count - 1>(f, pd, lane_group, tile_group);
}

template <typename T, int W, int kBlock, int kUnroll>
__global__ __launch_bounds__(kBlock) void encode_int_kernel(const void* src_v, void* dst_v, uint64_t n, IntConsts ic) {
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
        encode_group<W>(u, ic, stage, enc::row_slot<T, kBlock>(), r * kBlock);
      }
      enc::flush_stage<W, TG, kBlock>(stage, dst, G, g0);
      continue;
    }
    enc::PlaneDst<W> pd;
    enc::make_plane_dst<W>(dst, G, g0, pd);
    const uint32_t rem = rem_groups;
    enc::load_tile<T, kBlock, kUnroll, true, true>(src, 0, rem, regs);
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      if (r * kBlock + threadIdx.x < rem) {
        uint32_t u[8];
        enc::group_bits<T>(regs.v[r], u);
        encode_group<W>(u, ic, pd, threadIdx.x, r * kBlock);
      }
    }
  }

  // Ragged last group, padded with +0 (code 0).
  if (Gfull != G && flat_tile() == 0 && threadIdx.x == 0) {
    const T* __restrict__ src = static_cast<const T*>(src_v);
    uint32_t u[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint64_t i = Gfull * 8 + j;
      u[j] = 0;
      if (i < n) {
        if constexpr (sizeof(T) == 4)
          u[j] = reinterpret_cast<const uint32_t*>(src)[i];
        else
          u[j] = elem_bits<T>(reinterpret_cast<const uint16_t*>(src)[i]);
      }
    }
    enc::PlaneDst<W> pd;
    enc::make_plane_dst<W>(dst, G, Gfull, pd);
    encode_group<W>(u, ic, pd, 0, 0);
  }
}

// fp32 bits of the value of element j of a unit: k = (low Y bits) - (top bit << Y), times the quantum.
template <int W>
__device__ __forceinline__ uint32_t element_bits(const dec::UnitWords<W>& uw, int j, const FormatConsts& fc_right,
                                                 const IntConsts& ic) {
  const uint32_t low = dec::add_fields<W, 0>(uw, j, 0u, fc_right);  // fc_right.exp_shift = 0: fields at their code positions
  constexpr int PT = Planes<W>::count - 1;
  constexpr int ST = Planes<W>::seg(PT);
  const int bit = ST * j + ST - 1;
  const uint32_t top = (uw.w[PT][bit / 32] >> (bit % 32)) & 1u;
  const int32_t k = (int32_t)low - (int32_t)(top << (W - 1));
  return as_u32((float)k * ic.quantum);  // exact: |k| <= 2^Y fits the container's significand
}

template <typename T, int W>
__device__ __forceinline__ void decode_unit(const dec::UnitWords<W>& uw, const FormatConsts& fc_right,
                                            const IntConsts& ic, rsrc_t out, uint32_t lane_unit, uint32_t tile_unit) {
  constexpr int E = 16 / sizeof(T);
  uint32_t b[E];
#pragma unroll
  for (int j = 0; j < E; ++j) b[j] = element_bits<W>(uw, j, fc_right, ic);
  if constexpr (sizeof(T) == 4) {
    store16<true>(out, lane_unit * 16, tile_unit * 16, make_uint4(b[0], b[1], b[2], b[3]));
  } else {
    uint4 o;
    o.x = pack_elems<T>(b[0], b[1]);
    o.y = pack_elems<T>(b[2], b[3]);
    o.z = pack_elems<T>(b[4], b[5]);
    o.w = pack_elems<T>(b[6], b[7]);
    store16<true>(out, lane_unit * 16, tile_unit * 16, o);
  }
}

template <typename T, int W, int kBlock, int kUnroll>
__global__ __launch_bounds__(kBlock) void decode_int_kernel(const void* src_v, void* dst_v, uint64_t n, IntConsts ic) {
  constexpr uint32_t TU = kBlock * kUnroll;
  constexpr int E = 16 / sizeof(T);
  static_assert(TU % 2 == 0 && TU * E >= 512, "tiles start on a byte of the 1-bit plane; tile counts fit 32 bits");
  const uint8_t* __restrict__ src = static_cast<const uint8_t*>(src_v);
  T* __restrict__ dst = static_cast<T*>(dst_v);
  FormatConsts fc_right = {};
  fc_right.exp_shift = 0;
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
    const uint32_t rem = tile < full_tiles ? TU : rem_units;
    dec::TileWords<W, kUnroll> tw;
    dec::load_tile<W, E, kBlock, kUnroll, true>(ps, 0, rem, tw);
#pragma unroll
    for (int r = 0; r < kUnroll; ++r)
      if (r * kBlock + threadIdx.x < rem) decode_unit<T, W>(tw.u[r], fc_right, ic, out, threadIdx.x, r * kBlock);
  }

  // The n % E elements after the last whole unit, one lane each.
  if (flat_tile() == 0 && threadIdx.x < E) {
    const uint64_t i = Ufull * E + threadIdx.x;
    if (i < n) {
      dec::PlaneSrc<W> ps;
      dec::make_plane_src<W, 8>(src, G, i / 8, ps);
      dec::UnitWords<W> uw;
      dec::load_unit<W, 8>(ps, 0, 0, uw);
      uint32_t b = 0;
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if ((int)(i % 8) == j) b = element_bits<W>(uw, j, fc_right, ic);
      if constexpr (sizeof(T) == 4)
        reinterpret_cast<uint32_t*>(dst)[i] = b;
      else
        reinterpret_cast<uint16_t*>(dst)[i] = to_elem<T>(b);
    }
  }
}

// In-place emulation: the rounded, clamped magnitude comes back out of the sum by
// subtracting the magic addend; a zero result is +0 (k = 0 has one encoding);
// Inf / NaN pass through (Section 2.1).
__device__ __forceinline__ uint32_t emulate_bits(uint32_t u, const IntConsts& ic) {
  const float r = rounded_sum(u, ic) - ic.magic;
  const uint32_t rb = as_u32(r);
  const uint32_t out = rb ? (rb | (u & 0x80000000u)) : 0u;
  return (u & 0x7FFFFFFFu) >= 0x7F800000u ? u : out;
}

template <typename T, int kBlock>
__global__ __launch_bounds__(kBlock) void emulate_int_kernel(void* data_v, uint64_t n, IntConsts ic) {
  constexpr int kPer = 16 / sizeof(T);
  T* __restrict__ data = static_cast<T*>(data_v);
  const uint64_t V = n / kPer;
  const uint32_t tiles = (uint32_t)((V + kBlock - 1) / kBlock);
  for (uint32_t tile = flat_tile(), once = 1; once && tile < tiles; once = 0) {
    const uint64_t v0 = (uint64_t)tile * kBlock;
    if (v0 + threadIdx.x >= V) continue;
    const rsrc_t buf = make_rsrc(reinterpret_cast<uint4*>(data) + v0);
    const uint4 v = load16<true>(buf, threadIdx.x * 16, 0);
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if constexpr (sizeof(T) == 4) {
        w[k] = emulate_bits(w[k], ic);
      } else {
        const uint32_t lo = emulate_bits(lo_elem_bits<T>(w[k]), ic);
        const uint32_t hi = emulate_bits(hi_elem_bits<T>(w[k]), ic);
        const uint32_t pair = pack_elems<T>(lo, hi);
        w[k] = kIsF16<T> ? keep_nonfinite_halves(w[k], pair) : pair;
      }
    }
    store16<true>(buf, threadIdx.x * 16, 0, make_uint4(w[0], w[1], w[2], w[3]));
  }
  if (flat_tile() == 0 && threadIdx.x < kPer) {
    const uint64_t i = V * kPer + threadIdx.x;
    if (i < n) {
      if constexpr (sizeof(T) == 4) {
        uint32_t* p = reinterpret_cast<uint32_t*>(data) + i;
        *p = emulate_bits(*p, ic);
      } else {
        uint16_t* p = reinterpret_cast<uint16_t*>(data) + i;
        const uint32_t u = elem_bits<T>(*p);
        if ((u & 0x7FFFFFFFu) < 0x7F800000u) *p = to_elem<T>(emulate_bits(u, ic));  // Inf / NaN stay as they are
      }
    }
  }
}

}  // namespace twos
}  // namespace exmy
