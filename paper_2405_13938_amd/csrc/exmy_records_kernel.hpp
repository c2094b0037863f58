// Records: the plane words of Section 2.2.2 / Fig. 2 in another order.  Instead of
// one array per power-of-2 segment, the words of one group follow each other,
// widest segment first, as one record of W bytes, and the records follow each
// other in group order ("8 values in W bytes"): one stream instead of popcount(W),
// and a shard of the tensor is one byte range.  Not a layout of the paper.
//
// A lane still owns whole groups and forms (or consumes) the same plane words as
// the planar kernels.  A record starts at byte W * group, which no aligned store
// wider than a byte can reach for odd W, so a workgroup tile of kBlock * kUnroll
// groups passes through LDS: lanes move their records byte by byte on the LDS
// side, and the tile's kBlock * kUnroll * W contiguous bytes move between LDS and
// memory in 16-byte pieces (a tile starts on a multiple of 16 bytes because
// kBlock * kUnroll is a multiple of 16).
#pragma once

#include <type_traits>

#include "exmy_common.hpp"
#include "exmy_decode_kernel.hpp"
#include "exmy_encode_kernel.hpp"
#include "exmy_rows_kernel.hpp"

namespace exmy {
namespace rec {

// Bytes [lo(P), lo(P) + S) of a record hold the word of plane P.
template <int W, int P = 0>
__device__ __forceinline__ void put_record(uint8_t* rec, const rows::LaneWords<W, 1>& lw) {
  if constexpr (P < Planes<W>::count) {
    constexpr int S = Planes<W>::seg(P);
    constexpr int LO = Planes<W>::lo(P);
#pragma unroll
    for (int b = 0; b < S; ++b) rec[LO + b] = (uint8_t)(lw.w[P][b / 4] >> (8 * (b % 4)));
    put_record<W, P + 1>(rec, lw);
  }
}

// The plane bits of E consecutive elements of a record's group (E = 8: the group; E = 4:
// its half number `part`), laid out as the planar decoder's unit: plane P in the low
// E * S bits of uw.w[P].
template <int W, int E, int P = 0>
__device__ __forceinline__ void get_record(const uint8_t* rec, int part, dec::UnitWords<W>& uw) {
  if constexpr (P < Planes<W>::count) {
    constexpr int S = Planes<W>::seg(P);
    constexpr int LO = Planes<W>::lo(P);
    constexpr int kBits = E * S;
    if constexpr (kBits >= 8) {
      constexpr int kBytes = kBits / 8;
#pragma unroll
      for (int k = 0; k < (kBytes + 3) / 4; ++k) uw.w[P][k] = 0;
#pragma unroll
      for (int b = 0; b < kBytes; ++b) uw.w[P][b / 4] |= (uint32_t)rec[LO + part * kBytes + b] << (8 * (b % 4));
    } else {  // 4 bits: a nibble of the 1-bit plane's byte
      uw.w[P][0] = (uint32_t)rec[LO] >> (4 * part);
    }
    get_record<W, E, P + 1>(rec, part, uw);
  }
}

// The tile's `bytes` bytes between LDS and memory at `mem`: 16-byte pieces, then
// the few bytes of a last partial piece (only the last tile of a tensor has one).
template <int kBlock, bool kToMemory>
__device__ __forceinline__ void move_tile_bytes(uint8_t* lds, uint8_t* mem, uint32_t bytes) {
  const rsrc_t r = make_rsrc(mem);
  const uint32_t pieces = bytes / 16;
  for (uint32_t c = threadIdx.x; c < pieces; c += kBlock) {
    if constexpr (kToMemory)
      store16<true>(r, c * 16, 0, *reinterpret_cast<const uint4*>(lds + c * 16));
    else
      *reinterpret_cast<uint4*>(lds + c * 16) = load16<true>(r, c * 16, 0);
  }
  for (uint32_t b = pieces * 16 + threadIdx.x; b < bytes; b += kBlock) {
    if constexpr (kToMemory)
      mem[b] = lds[b];
    else
      lds[b] = mem[b];
  }
}

template <typename T, int W, int kBlock, int kUnroll, bool kWide>
__global__ __launch_bounds__(kBlock) void encode_records_kernel(const void* __restrict__ src_v, uint8_t* __restrict__ dst,
                                                                 uint64_t n, FormatConsts fc, TensorConsts tc) {
  constexpr uint32_t TG = kBlock * kUnroll;
  static_assert(TG % 16 == 0, "a tile must start on a multiple of 16 bytes");
  constexpr int kLoads = enc::TileRegs<T, kUnroll>::kLoads;
  __shared__ __align__(16) uint8_t lds[TG * W];
  const uint4* __restrict__ src4 = static_cast<const uint4*>(src_v);
  const uint64_t G = (n + 7) / 8;  // groups, the last one possibly ragged
  const uint64_t Gfull = n / 8;
  const uint32_t tiles = (uint32_t)((G + TG - 1) / TG);
  const uint32_t all_tiles = (uint32_t)(G / TG), full_tiles = (uint32_t)(Gfull / TG);
  const uint32_t rem_all = (uint32_t)(G - (uint64_t)all_tiles * TG), rem_whole = (uint32_t)(Gfull - (uint64_t)full_tiles * TG);

  for (uint32_t tile = flat_tile(), once = 1; once && tile < tiles; once = 0) {
    const uint64_t g0 = (uint64_t)tile * TG;
    const uint32_t here = units_in_tile(tile, all_tiles, rem_all, TG);        // groups of this tile
    const uint32_t whole = units_in_tile(tile, full_tiles, rem_whole, TG);   // of them, with all 8 elements
    const rsrc_t src = make_rsrc(src4 + g0 * kLoads);
    enc::TileRegs<T, kUnroll> regs;
    auto body = [&](auto guard) {
      constexpr bool kGuard = decltype(guard)::value;
      enc::load_tile<T, kBlock, kUnroll, true, kGuard>(src, 0, whole, regs);
#pragma unroll
      for (int r = 0; r < kUnroll; ++r) {
        const uint32_t jl = r * kBlock + (kGuard ? threadIdx.x : enc::row_slot<T, kBlock>());
        if (!kGuard || jl < here) {
          uint32_t u[8];
          if (!kGuard || jl < whole)
            enc::group_bits<T, !kGuard>(regs.v[r], u);
          else
            enc::ragged_group_bits<T>(src_v, (g0 + jl) * 8, n, u);
          uint32_t f[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const uint32_t m = magnitude_code_left<kWide>(u[j], fc, tc);
            f[j] = (W & 1) ? m : ((u[j] & 0x80000000u) | m);  // even W: the sign rides at bit 31
          }
          rows::LaneWords<W, 1> lw;
          rows::peel_column<W, 1, Planes<W>::count - 1>(f, u, 0, lw);
          put_record<W>(lds + jl * W, lw);
        }
      }
    };
    if (tile < full_tiles)
      body(std::false_type{});
    else
      body(std::true_type{});
    __syncthreads();
    move_tile_bytes<kBlock, true>(lds, dst + g0 * W, here * W);
    __syncthreads();  // the next tile overwrites the LDS bytes
  }
}

// A lane produces one 16-byte store, as in the planar decoder: a whole group of 16-bit
// values, or half a group of fp32 (the two lanes of a group read the same record).
template <typename T, int W, int kBlock, int kUnroll, bool kX8>
__global__ __launch_bounds__(kBlock) void decode_records_kernel(const uint8_t* __restrict__ src, T* __restrict__ dst,
                                                                 uint64_t n, FormatConsts fc, TensorConsts tc) {
  constexpr uint32_t TG = kBlock * kUnroll;
  static_assert(TG % 16 == 0, "a tile must start on a multiple of 16 bytes");
  constexpr int E = 16 / sizeof(T);  // elements per store
  constexpr int kPerGroup = 8 / E;   // stores per group
  __shared__ __align__(16) uint8_t lds[TG * W];
  const uint64_t G = (n + 7) / 8;
  const uint64_t Gfull = n / 8;
  const uint32_t tiles = (uint32_t)((G + TG - 1) / TG);
  const uint32_t all_tiles = (uint32_t)(G / TG), full_tiles = (uint32_t)(Gfull / TG);
  const uint32_t rem_all = (uint32_t)(G - (uint64_t)all_tiles * TG), rem_whole = (uint32_t)(Gfull - (uint64_t)full_tiles * TG);

  for (uint32_t tile = flat_tile(), once = 1; once && tile < tiles; once = 0) {
    const uint64_t g0 = (uint64_t)tile * TG;
    const uint32_t here = units_in_tile(tile, all_tiles, rem_all, TG);
    const uint32_t whole = units_in_tile(tile, full_tiles, rem_whole, TG);
    move_tile_bytes<kBlock, false>(lds, const_cast<uint8_t*>(src) + g0 * W, here * W);
    __syncthreads();
    const rsrc_t out = make_rsrc(reinterpret_cast<uint4*>(dst) + g0 * kPerGroup);
#pragma unroll
    for (int r = 0; r < kUnroll * kPerGroup; ++r) {
      const uint32_t ul = r * kBlock + threadIdx.x;  // store of the tile
      const uint32_t jl = ul / kPerGroup;            // its group
      const int half = ul % kPerGroup;
      if (jl < here) {
        dec::UnitWords<W> uw;
        get_record<W, E>(lds + jl * W, half, uw);
        uint32_t b[E];
#pragma unroll
        for (int j = 0; j < E; ++j) b[j] = dec::element_bits<W, kX8>(uw, j, fc, tc);
        if (jl < whole) {
          if constexpr (sizeof(T) == 4) {
            store16<true>(out, ul * 16, 0, make_uint4(b[0], b[1], b[2], b[3]));
          } else {
            uint4 o;
            o.x = pack_elems<T>(b[0], b[1]);
            o.y = pack_elems<T>(b[2], b[3]);
            o.z = pack_elems<T>(b[4], b[5]);
            o.w = pack_elems<T>(b[6], b[7]);
            store16<true>(out, ul * 16, 0, o);
          }
        } else {  // the ragged last group of the tensor
#pragma unroll
          for (int j = 0; j < E; ++j) {
            const uint64_t i = (g0 + jl) * 8 + half * E + j;
            if (i < n) {
              if constexpr (sizeof(T) == 4)
                reinterpret_cast<uint32_t*>(dst)[i] = b[j];
              else
                reinterpret_cast<uint16_t*>(dst)[i] = to_elem<T>(b[j]);
            }
          }
        }
      }
    }
    __syncthreads();  // the next tile overwrites the LDS bytes
  }
}

}  // namespace rec
}  // namespace exmy
