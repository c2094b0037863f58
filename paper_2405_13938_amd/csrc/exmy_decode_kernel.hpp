// Fused decode: power-of-2 planes -> eXmY codes (Section 2.2.2, Fig. 2 read right
// to left) -> bf16 / fp32 values (Section 2.2.1 "and vice versa").
//
// One lane produces one 16-byte store: a whole group of 8 bf16 values, or half a
// group (4 values) of fp32, so that the lanes of a wavefront always write one
// contiguous span.  The lane reads just the part of each plane word that holds
// its elements (S bytes per plane for a group, S/2 for half a group; two lanes
// share a byte of a 1-bit plane).  The code itself is never assembled: each
// plane field is extracted and added straight into the fp32 bit pattern at the
// position it has there.  Tiles, chunks and launch order are as in the encoder.
#pragma once

#include "exmy_common.hpp"

namespace exmy {
namespace dec {

// The plane bits of the E consecutive elements one lane decodes (E = 8 or 4):
// plane p uses w[p][0 .. ceil(E*S/32)).
template <int W>
struct UnitWords {
  uint32_t w[Planes<W>::count][4];
};

// The source of one chunk: a descriptor per plane, based at the plane bits of the
// chunk's first unit (a unit is E elements; chunks start on even units).
template <int W>
struct PlaneSrc {
  rsrc_t plane[Planes<W>::count];
};

template <int W, int E, int P = 0>
__device__ __forceinline__ void make_plane_src(const uint8_t* src, uint64_t G, uint64_t u0, PlaneSrc<W>& ps) {
  if constexpr (P < Planes<W>::count) {
    constexpr uint64_t kBits = E * Planes<W>::seg(P);
    constexpr uint64_t LO = Planes<W>::lo(P);
    ps.plane[P] = make_rsrc(src + (G * LO + (u0 * kBits) / 8));
    make_plane_src<W, E, P + 1>(src, G, u0, ps);
  }
}

// Plane bits of the unit number tile_unit + lane_unit of the chunk (tile_unit is
// wave-uniform and even).
template <int W, int E, int P = 0>
__device__ __forceinline__ void load_unit(const PlaneSrc<W>& ps, uint32_t lane_unit, uint32_t tile_unit,
                                          UnitWords<W>& uw) {
  if constexpr (P < Planes<W>::count) {
    constexpr int S = Planes<W>::seg(P);
    constexpr int kBits = E * S;  // plane bits per unit: 128, 64, 32, 16, 8 or 4
    const rsrc_t r = ps.plane[P];
    if constexpr (kBits == 128) {
      const uint4 o = load16<false>(r, lane_unit * 16, tile_unit * 16);
      uw.w[P][0] = o.x; uw.w[P][1] = o.y; uw.w[P][2] = o.z; uw.w[P][3] = o.w;
    } else if constexpr (kBits == 64) {
      const u32x2_t o = __builtin_amdgcn_raw_buffer_load_b64(r, lane_unit * 8, tile_unit * 8, 0);
      uw.w[P][0] = o.x; uw.w[P][1] = o.y;
    } else if constexpr (kBits == 32) {
      uw.w[P][0] = __builtin_amdgcn_raw_buffer_load_b32(r, lane_unit * 4, tile_unit * 4, 0);
    } else if constexpr (kBits == 16) {
      uw.w[P][0] = __builtin_amdgcn_raw_buffer_load_b16(r, lane_unit * 2, tile_unit * 2, 0);
    } else if constexpr (kBits == 8) {
      uw.w[P][0] = __builtin_amdgcn_raw_buffer_load_b8(r, lane_unit, tile_unit, 0);
    } else {  // 4 bits: the low or high nibble of a byte shared with the neighbouring lane
      uw.w[P][0] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b8(r, lane_unit >> 1, tile_unit >> 1, 0) >> (4 * (lane_unit & 1));
    }
    load_unit<W, E, P + 1>(ps, lane_unit, tile_unit, uw);
  }
}

// Add the magnitude bits that plane P holds for element j of the unit into g, at
// the place they have in the fp32 pattern.  The top plane's most significant bit
// is the sign and is left out here.
template <int W, int P>
__device__ __forceinline__ uint32_t add_fields(const UnitWords<W>& uw, int j, uint32_t g, const FormatConsts& fc) {
  if constexpr (P < Planes<W>::count) {
    constexpr int S = Planes<W>::seg(P);
    constexpr int LO = Planes<W>::lo(P);
    constexpr bool top = P == Planes<W>::count - 1;
    constexpr int width = top ? S - 1 : S;
    if constexpr (width > 0) {
      const int bit = S * j;
      const uint32_t field = __builtin_amdgcn_ubfe(uw.w[P][bit / 32], bit % 32, width);
      g = lshl_add(field, fc.exp_shift + LO, g);
    }
    return add_fields<W, P + 1>(uw, j, g, fc);
  } else {
    return g;
  }
}

// fp32 bit pattern of element j of the unit.
template <int W, bool kX8>
__device__ __forceinline__ uint32_t element_bits(const UnitWords<W>& uw, int j, const FormatConsts& fc,
                                                 const TensorConsts& tc) {
  uint32_t g = add_fields<W, 0>(uw, j, tc.dec_bias, fc);
  if constexpr (kX8) g = min(g, fc.g_clamp);  // exponent code 255 is not a value: largest finite instead
  const uint32_t mag = finish_magnitude(g, tc);
  constexpr int PT = Planes<W>::count - 1;
  constexpr int ST = Planes<W>::seg(PT);
  const int bit = ST * j + ST - 1;  // the sign: top bit of the top plane's field
  const uint32_t s = uw.w[PT][bit / 32] << (31 - bit % 32);
  return (s & 0x80000000u) | mag;
}

// The 16 bytes of one unit's values.
// kScaled (float scaling): every value is multiplied by `scale` on the way out and the real product is
// rounded once into T (see settle_scaled_product); short_scale (wave-uniform): the scales are bf16 values.
template <typename T, int W, bool kX8, bool kScaled = false>
__device__ __forceinline__ uint4 unit_values(const UnitWords<W>& uw, const FormatConsts& fc, const TensorConsts& tc,
                                             float scale = 1.0f, bool short_scale = false) {
  constexpr int E = 16 / sizeof(T);
  uint32_t b[E];
#pragma unroll
  for (int j = 0; j < E; ++j) b[j] = element_bits<W, kX8>(uw, j, fc, tc);
  if constexpr (kScaled) {
    float p[E];
#pragma unroll
    for (int j = 0; j < E; ++j) p[j] = as_f32(b[j]) * scale;  // scale > 0: the product keeps the sign
    if constexpr (sizeof(T) == 4) {
      return make_uint4(as_u32(p[0]), as_u32(p[1]), as_u32(p[2]), as_u32(p[3]));
    } else {
      if (__builtin_amdgcn_ballot_w64(scaled_products_suspect<T, E>(p, short_scale)) != 0) {
        asm volatile("");  // a real branch: the compiler must not settle every product and select
        const float s_mant = __builtin_amdgcn_frexp_mantf(scale);
        const int s_exp = __builtin_amdgcn_frexp_expf(scale);
#pragma unroll
        for (int j = 0; j < E; ++j)
          p[j] = settle_scaled_product(p[j], as_f32(b[j]), s_mant, s_exp, scaled_product_low_bits_clear<T>(p[j]));
      }
      if constexpr (kIsF16<T>)
        return make_uint4(pack_elems<T, false>(as_u32(p[0]), as_u32(p[1])), pack_elems<T, false>(as_u32(p[2]), as_u32(p[3])),
                          pack_elems<T, false>(as_u32(p[4]), as_u32(p[5])), pack_elems<T, false>(as_u32(p[6]), as_u32(p[7])));
      else  // bf16: rounded pair by pair by the conversion instruction
        return make_uint4(round_pack_bf16(p[0], p[1]), round_pack_bf16(p[2], p[3]), round_pack_bf16(p[4], p[5]),
                          round_pack_bf16(p[6], p[7]));
    }
  } else if constexpr (sizeof(T) == 4) {
    return make_uint4(b[0], b[1], b[2], b[3]);
  } else {
    // every value is exact in the 16-bit type: keep the upper halves / convert exactly
    uint4 o;
    o.x = pack_elems<T>(b[0], b[1]);
    o.y = pack_elems<T>(b[2], b[3]);
    o.z = pack_elems<T>(b[4], b[5]);
    o.w = pack_elems<T>(b[6], b[7]);
    return o;
  }
}

// Values of one unit, stored to 16-byte vector lane_unit + tile_unit of `out`.
template <typename T, int W, bool kX8, bool kNT, bool kScaled = false>
__device__ __forceinline__ void decode_unit(const UnitWords<W>& uw, const FormatConsts& fc, const TensorConsts& tc,
                                            rsrc_t out, uint32_t lane_unit, uint32_t tile_unit, float scale = 1.0f,
                                            bool short_scale = false) {
  store16<kNT>(out, lane_unit * 16, tile_unit * 16, unit_values<T, W, kX8, kScaled>(uw, fc, tc, scale, short_scale));
}

// A lane of a narrow format reads 1-3 bytes per plane straight from memory.  Whole tiles
// can instead come through an LDS image (see tile_piece_address) filled with 16-byte
// loads, which pays at W = 3 only (see the launcher).
template <int W, int kTileGroups, int kBlock>
__device__ __forceinline__ void load_image(const uint8_t* __restrict__ src, uint64_t G, uint64_t g0, uint8_t* lds) {
  constexpr uint32_t kPieces = kTileGroups * W / 16;
#pragma unroll
  for (uint32_t c0 = 0; c0 < kPieces; c0 += kBlock) {
    const uint32_t c = c0 + threadIdx.x;
    if (kPieces % kBlock == 0 || c < kPieces) {
      const u32x4_t w = __builtin_nontemporal_load(
          reinterpret_cast<const plane_piece_t*>(tile_piece_address<W, kTileGroups>(const_cast<uint8_t*>(src), G, g0, c * 16)));
      *reinterpret_cast<uint4*>(lds + c * 16) = make_uint4(w.x, w.y, w.z, w.w);
    }
  }
}

// Unit `unit` of the tile from its image, laid out as load_unit leaves it.
template <int W, int E, int kTileGroups, int P = 0>
__device__ __forceinline__ void image_unit(const uint8_t* lds, uint32_t unit, UnitWords<W>& uw) {
  if constexpr (P < Planes<W>::count) {
    constexpr int S = Planes<W>::seg(P);
    constexpr int kBits = E * S;  // of plane P per unit
    constexpr int LO = Planes<W>::lo(P);  // as a constant: the call itself would run its loop on the scalar unit
    const uint8_t* p = lds + kTileGroups * LO + unit * kBits / 8;
    if constexpr (kBits == 128) {
      const uint4 v = *reinterpret_cast<const uint4*>(p);
      uw.w[P][0] = v.x; uw.w[P][1] = v.y; uw.w[P][2] = v.z; uw.w[P][3] = v.w;
    } else if constexpr (kBits == 64) {
      const uint2 v = *reinterpret_cast<const uint2*>(p);
      uw.w[P][0] = v.x; uw.w[P][1] = v.y;
    } else if constexpr (kBits == 32) {
      uw.w[P][0] = *reinterpret_cast<const uint32_t*>(p);
    } else if constexpr (kBits == 16) {
      uw.w[P][0] = *reinterpret_cast<const uint16_t*>(p);
    } else if constexpr (kBits == 8) {
      uw.w[P][0] = *p;
    } else {  // 4 bits: a nibble of the byte shared with the neighbouring unit
      uw.w[P][0] = (uint32_t)*p >> (4 * (unit & 1u));
    }
    image_unit<W, E, kTileGroups, P + 1>(lds, unit, uw);
  }
}

template <int W, int kUnroll>
struct TileWords {
  UnitWords<W> u[kUnroll];
};

// Loads of the tile whose first unit, relative to the chunk, is tile_unit (wave-
// uniform, even).  kGuard: only the first `rem` units of the tile exist.
template <int W, int E, int kBlock, int kUnroll, bool kGuard>
__device__ __forceinline__ void load_tile(const PlaneSrc<W>& ps, uint32_t tile_unit, uint32_t rem,
                                          TileWords<W, kUnroll>& tw) {
#pragma unroll
  for (int r = 0; r < kUnroll; ++r) {
    if (!kGuard || r * kBlock + threadIdx.x < rem) load_unit<W, E>(ps, threadIdx.x, tile_unit + r * kBlock, tw.u[r]);
  }
}

template <typename T, int W, int kBlock, int kUnroll, bool kX8, bool kNT, bool kGuard>
__device__ __forceinline__ void decode_tile(const TileWords<W, kUnroll>& tw, rsrc_t out, uint32_t tile_unit,
                                            uint32_t rem, const FormatConsts& fc, const TensorConsts& tc) {
  if constexpr (!kGuard) {
    // a whole tile: all values first, then its stores back to back (+1 % over storing each unit as it is ready)
    uint4 o[kUnroll];
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) o[r] = unit_values<T, W, kX8>(tw.u[r], fc, tc);
    asm volatile("" ::: "memory");  // keeps the compiler from moving a store up between the conversions
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) store16<kNT>(out, threadIdx.x * 16, (tile_unit + r * kBlock) * 16, o[r]);
    return;
  }
#pragma unroll
  for (int r = 0; r < kUnroll; ++r) {
    if (!kGuard || r * kBlock + threadIdx.x < rem)
      decode_unit<T, W, kX8, kNT>(tw.u[r], fc, tc, out, threadIdx.x, tile_unit + r * kBlock);
  }
}

// One element straight from memory (the few elements after the last whole unit).
template <int W, bool kX8>
__device__ __forceinline__ uint32_t element_bits_slow(const uint8_t* __restrict__ src, uint64_t G, uint64_t idx,
                                                      const FormatConsts& fc, const TensorConsts& tc) {
  PlaneSrc<W> ps;
  make_plane_src<W, 8>(src, G, idx / 8, ps);  // the whole group that holds the element
  UnitWords<W> uw;
  load_unit<W, 8>(ps, 0, 0, uw);
  uint32_t b = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j)
    if ((int)(idx % 8) == j) b = element_bits<W, kX8>(uw, j, fc, tc);
  return b;
}

// Grid: x (and z, for tensors of more than gridDim.x tiles) = tile, one per workgroup and no loop (see
// enc::encode_flat_kernel for what the loop-free form saves); y = tensor of the batch.  Workgroups past a
// tensor's last tile find nothing to do; the workgroup of the tile after the last whole one takes the
// partial tile and the few elements after the last whole unit.
// kStage: whole tiles read their plane bytes through an LDS image.
template <typename T, int W, int kBlock, int kUnroll, bool kX8, bool kNT, bool kStage = false>
__global__ __launch_bounds__(kBlock) void decode_kernel(const BatchArgs batch) {
  constexpr uint32_t TU = kBlock * kUnroll;
  static_assert(TU % 2 == 0, "a tile must start on a byte of the 1-bit plane");
  static_assert(TU * (16 / sizeof(T)) >= 512, "tile counts must fit 32 bits for n <= 2^40");
  const TensorArgs& ta = batch.t[blockIdx.y];
  const uint8_t* __restrict__ src = static_cast<const uint8_t*>(ta.src);
  T* __restrict__ dst = static_cast<T*>(ta.dst);
  const uint64_t n = ta.n;
  const FormatConsts fc = batch.fc;
  const TensorConsts tc = ta.tc;
  constexpr int E = 16 / sizeof(T);  // elements per lane
  const uint64_t G = (n + 7) / 8;
  const uint64_t Ufull = n / E;  // units with all E elements present
  const uint32_t full_tiles = (uint32_t)(Ufull / TU);
  constexpr uint32_t TG = TU * E / 8;  // groups of a tile
  __shared__ __align__(16) uint8_t lds_image[kStage ? TG * W : 16];
  const uint32_t tile = blockIdx.z * gridDim.x + blockIdx.x;
  if (tile > full_tiles) return;
  const uint64_t u0 = (uint64_t)tile * TU;  // first unit of the tile (even)
  const rsrc_t out = make_rsrc(reinterpret_cast<uint4*>(dst) + u0);

  if (tile < full_tiles) {
    if constexpr (kStage) {
      load_image<W, TG, kBlock>(src, G, u0 * E / 8, lds_image);
      __syncthreads();
#pragma unroll
      for (int r = 0; r < kUnroll; ++r) {
        UnitWords<W> uw;
        image_unit<W, E, TG>(lds_image, r * kBlock + threadIdx.x, uw);
        decode_unit<T, W, kX8, kNT>(uw, fc, tc, out, threadIdx.x, r * kBlock);
      }
    } else {
      PlaneSrc<W> ps;
      make_plane_src<W, E>(src, G, u0, ps);
      TileWords<W, kUnroll> tw;
      load_tile<W, E, kBlock, kUnroll, false>(ps, 0, 0, tw);
      decode_tile<T, W, kBlock, kUnroll, kX8, kNT, false>(tw, out, 0, 0, fc, tc);
    }
    return;
  }

  const uint32_t rem_units = (uint32_t)(Ufull - (uint64_t)full_tiles * TU);
  if (rem_units) {
    PlaneSrc<W> ps;
    make_plane_src<W, E>(src, G, u0, ps);
    TileWords<W, kUnroll> tw;
    load_tile<W, E, kBlock, kUnroll, true>(ps, 0, rem_units, tw);
    decode_tile<T, W, kBlock, kUnroll, kX8, kNT, true>(tw, out, 0, rem_units, fc, tc);
  }
  // The n % E elements after the last whole unit, one lane each.
  if (threadIdx.x < E) {
    const uint64_t i = Ufull * E + threadIdx.x;
    if (i < n) {
      const uint32_t b = element_bits_slow<W, kX8>(src, G, i, fc, tc);
      if constexpr (sizeof(T) == 4)
        reinterpret_cast<uint32_t*>(dst)[i] = b;
      else
        reinterpret_cast<uint16_t*>(dst)[i] = to_elem<T>(b);
    }
  }
}

// ---------------------------------------------------------------------------
// Per-block metadata: flat tiles with a per-lane metadata lookup, as in the
// encoder.  A unit is one lane's 16 bytes of output (E elements).

// One unit under its block's metadatum.  try_uniform: look first for a metadatum common to the
// wavefront, whose constants are then derived once on the scalar unit (see wave_uniform).
template <typename T, int W, bool kNT>
__device__ __forceinline__ void decode_unit_meta(const UnitWords<W>& uw, uint32_t me, const FormatConsts& fc,
                                                 const BlockConsts& bc, rsrc_t out, uint32_t lane_unit,
                                                 uint32_t tile_unit, bool try_uniform) {
  uint32_t first;
  if (try_uniform && wave_uniform(me, first))
    decode_unit<T, W, false, kNT>(uw, fc, derive_tc(first, bc), out, lane_unit, tile_unit);
  else
    decode_unit<T, W, false, kNT>(uw, fc, derive_tc(me, bc), out, lane_unit, tile_unit);
}

// kScaled: per-block fp32 scales and the max_exp = 127 format instead of per-block
// metadata bytes.
template <typename T, int W, int kBlock, int kUnroll, bool kNT, bool kScaled>
__global__ __launch_bounds__(kBlock) void decode_blocks_kernel(const BlockArgs args) {
  constexpr uint32_t TU = kBlock * kUnroll;
  constexpr int E = 16 / sizeof(T);
  const uint8_t* __restrict__ src = static_cast<const uint8_t*>(args.src);
  T* __restrict__ dst = static_cast<T*>(args.dst);
  const uint8_t* __restrict__ meta = args.meta;
  const uint64_t n = args.n;
  const FormatConsts fc = args.fc;
  const BlockConsts bc = args.bc;
  const BlockIndex bi = args.bi;  // in units
  const uint64_t G = (n + 7) / 8;
  const uint64_t Ufull = n / E;
  const uint32_t full_tiles = (uint32_t)(Ufull / TU);
  const uint32_t rem_units = (uint32_t)(Ufull - (uint64_t)full_tiles * TU);
  const uint32_t tiles = full_tiles + (rem_units ? 1u : 0u);
  // at most 16 blocks per wavefront; 16-bit elements only: +2-3 % there, while the fp32 kernel (4 elements per lane,
  // less arithmetic per byte) lost 6 % to the second copy of its code
  const bool try_uniform = sizeof(T) == 2 && bi.size >= 4;

  for (uint32_t tile = flat_tile(), once = 1; once && tile < tiles; once = 0) {
    const uint64_t u0 = (uint64_t)tile * TU;  // even
    uint64_t blk0;
    uint32_t off;
    tile_first_block(u0, bi, blk0, off);
    PlaneSrc<W> ps;
    make_plane_src<W, E>(src, G, u0, ps);
    const rsrc_t out = make_rsrc(reinterpret_cast<uint4*>(dst) + u0);
    const rsrc_t mt = kScaled ? make_rsrc(scale_address(args, blk0)) : make_rsrc(meta + blk0);
    TileWords<W, kUnroll> tw;
    uint32_t me[kUnroll];  // the block's metadatum, or the bits of its scale
    if (tile < full_tiles) {
      load_tile<W, E, kBlock, kUnroll, false>(ps, 0, 0, tw);
#pragma unroll
      for (int r = 0; r < kUnroll; ++r)
        me[r] = load_block_datum<kScaled>(mt, lane_block<TU>(off + r * kBlock + threadIdx.x, bi), args.scale_log2_bytes);
#pragma unroll
      for (int r = 0; r < kUnroll; ++r) {
        if constexpr (kScaled)
          decode_unit<T, W, false, kNT, true>(tw.u[r], fc, args.tc127, out, threadIdx.x, r * kBlock, as_f32(me[r]),
                                              args.scale_log2_bytes == 1);
        else
          decode_unit_meta<T, W, kNT>(tw.u[r], me[r], fc, bc, out, threadIdx.x, r * kBlock, try_uniform);
      }
    } else {
      load_tile<W, E, kBlock, kUnroll, true>(ps, 0, rem_units, tw);
#pragma unroll
      for (int r = 0; r < kUnroll; ++r)
        me[r] = (r * kBlock + threadIdx.x < rem_units)
                    ? load_block_datum<kScaled>(mt, lane_block<TU>(off + r * kBlock + threadIdx.x, bi), args.scale_log2_bytes)
                    : 0u;
#pragma unroll
      for (int r = 0; r < kUnroll; ++r) {
        if (r * kBlock + threadIdx.x < rem_units) {
          if constexpr (kScaled)
            decode_unit<T, W, false, kNT, true>(tw.u[r], fc, args.tc127, out, threadIdx.x, r * kBlock, as_f32(me[r]),
                                              args.scale_log2_bytes == 1);
          else
            decode_unit_meta<T, W, kNT>(tw.u[r], me[r], fc, bc, out, threadIdx.x, r * kBlock, try_uniform);
        }
      }
    }
  }

  // The n % E elements after the last whole unit belong to the last block.
  if (flat_tile() == 0 && threadIdx.x < E) {
    const uint64_t i = Ufull * E + threadIdx.x;
    if (i < n) {
      uint32_t b;
      if constexpr (kScaled) {
        b = element_bits_slow<W, false>(src, G, i, fc, args.tc127);
        b = scaled_product_bits<T>(b, as_f32(load_scale_bits(args, args.n_blocks - 1)));
      } else {
        b = element_bits_slow<W, false>(src, G, i, fc, derive_tc(meta[args.n_blocks - 1], bc));
      }
      if constexpr (sizeof(T) == 4)
        reinterpret_cast<uint32_t*>(dst)[i] = b;
      else
        reinterpret_cast<uint16_t*>(dst)[i] = to_elem<T>(b);
    }
  }
}

}  // namespace dec
}  // namespace exmy
