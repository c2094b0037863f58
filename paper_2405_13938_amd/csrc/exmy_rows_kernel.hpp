// Codec with packing along rows (Section 2.2.2, Fig. 2: an array of shape (8R, C)
// becomes, per power-of-2 segment, an array of shape (R, C)): the 8 elements of a
// group are the 8 rows of one row block at one column of a row-major matrix.
//
// One lane owns kCols adjacent columns (16 bytes of every row: 8 bf16 or 4 fp32
// values) of one row block: eight 16-byte loads, one per row, each contiguous
// over the wavefront; kCols adjacent words of every plane, written (or read) as
// one contiguous piece of kCols * S bytes.  A row block is cols / kCols such lane
// places, and the lane places of the whole matrix, row block after row block, are
// the words of every plane in address order.
//
// Two ways to cut them into workgroup tiles of kBlock places:
//  - by row block (wide matrices): a tile is kBlock * kCols columns of one row block,
//    the last tile of a row block partly idle.  A tile sees at most 8 metadata, all
//    wave-uniform, so the constants of the 8 rows stay in SGPRs;
//  - folded (kFold; narrow matrices, and widths that would leave much of the last
//    tile idle): a tile is kBlock consecutive places whatever row blocks they fall
//    into, so a 128-column bf16 matrix (16 places per row block) puts 4 row blocks
//    into a wavefront and every lane works.  The planes are still written as one
//    contiguous run per tile, the source is read as runs of one matrix row each,
//    and per-row metadata are per-lane values.
//
// Metadata: one max_exp for the tensor, or one per row of the matrix (Section
// 2.2.1: the (R, 1) metadata tensor).
#pragma once

#include "exmy_decode_kernel.hpp"
#include "exmy_encode_kernel.hpp"

namespace exmy {

namespace rows {

using enc::plane_word_from_top;

// fp32-position bits of column c of a 16-byte row piece.
template <typename T>
__device__ __forceinline__ uint32_t column_bits(const uint4& v, int c) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  if constexpr (sizeof(T) == 4) return w[c];
  return (c & 1) ? hi_elem_bits<T>(w[c / 2]) : lo_elem_bits<T>(w[c / 2]);
}

// Plane words of a lane: plane P holds kCols words of S bytes, packed into
// dwords in column order.
template <int W, int kCols>
struct LaneWords {
  uint32_t w[Planes<W>::count][kCols * 4];  // plane P uses the first kCols * S / 4 (at least 1)
};

// Place the word of column c (from plane_word_from_top) into the lane's piece of plane P.
template <int W, int kCols, int P>
__device__ __forceinline__ void put_word(LaneWords<W, kCols>& lw, int c, const uint32_t word[4]) {
  constexpr int S = Planes<W>::seg(P);
  if constexpr (S >= 4) {
#pragma unroll
    for (int k = 0; k < S / 4; ++k) lw.w[P][c * (S / 4) + k] = word[k];
  } else if constexpr (S == 2) {
    if (c & 1)
      lw.w[P][c / 2] |= word[0] << 16;
    else
      lw.w[P][c / 2] = word[0] & 0xFFFFu;
  } else {
    if (c & 3)
      lw.w[P][c / 4] |= (word[0] & 0xFFu) << (8 * (c & 3));
    else
      lw.w[P][c / 4] = word[0] & 0xFFu;
  }
}

// Peel the planes of column c off the left-aligned codes f (sign plane of an odd W from u).
template <int W, int kCols, int P>
__device__ __forceinline__ void peel_column(uint32_t f[8], const uint32_t u[8], int c, LaneWords<W, kCols>& lw) {
  constexpr int S = Planes<W>::seg(P);
  constexpr bool sign_plane = (W & 1) && P == Planes<W>::count - 1;
  uint32_t word[4];
  if constexpr (sign_plane) {
    plane_word_from_top<S>(u, word);
  } else {
    plane_word_from_top<S>(f, word);
    if constexpr (P > 0) {
#pragma unroll
      for (int j = 0; j < 8; ++j) f[j] <<= S;
    }
  }
  put_word<W, kCols, P>(lw, c, word);
  if constexpr (P > 0) peel_column<W, kCols, P - 1>(f, u, c, lw);
}

// Store (kStore) or load the lane's piece of every plane: kCols * S bytes at byte
// offset lane * kCols * S of the plane descriptor.
template <int W, int kCols, bool kStore, int P = 0>
__device__ __forceinline__ void move_words(LaneWords<W, kCols>& lw, const rsrc_t* plane, uint32_t lane) {
  if constexpr (P < Planes<W>::count) {
    constexpr int S = Planes<W>::seg(P);
    constexpr int kBytes = kCols * S;  // 4 ... 128
    const uint32_t off = lane * kBytes;
    const rsrc_t r = plane[P];
    if constexpr (kBytes >= 16) {
#pragma unroll
      for (int k = 0; k < kBytes / 16; ++k) {
        if constexpr (kStore) {
          store16<false>(r, off, k * 16, make_uint4(lw.w[P][4 * k], lw.w[P][4 * k + 1], lw.w[P][4 * k + 2], lw.w[P][4 * k + 3]));
        } else {
          const uint4 v = load16<false>(r, off, k * 16);
          lw.w[P][4 * k] = v.x; lw.w[P][4 * k + 1] = v.y; lw.w[P][4 * k + 2] = v.z; lw.w[P][4 * k + 3] = v.w;
        }
      }
    } else if constexpr (kBytes == 8) {
      if constexpr (kStore) {
        const u32x2_t o = {lw.w[P][0], lw.w[P][1]};
        __builtin_amdgcn_raw_buffer_store_b64(o, r, off, 0, 0);
      } else {
        const u32x2_t v = __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, 0);
        lw.w[P][0] = v.x; lw.w[P][1] = v.y;
      }
    } else {
      static_assert(kBytes == 4, "a lane's piece of a plane is at least one dword");
      if constexpr (kStore)
        __builtin_amdgcn_raw_buffer_store_b32(lw.w[P][0], r, off, 0, 0);
      else
        lw.w[P][0] = __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 0);
    }
    move_words<W, kCols, kStore, P + 1>(lw, plane, lane);
  }
}

// Plane descriptors based at the plane words of (row block rb, column col0).
template <int W, int P = 0>
__device__ __forceinline__ void make_plane_rsrc(uint8_t* packed, uint64_t R, uint32_t cols, uint64_t rb, uint32_t col0,
                                                rsrc_t* plane) {
  if constexpr (P < Planes<W>::count) {
    constexpr uint64_t S = Planes<W>::seg(P);
    constexpr uint64_t LO = Planes<W>::lo(P);
    plane[P] = make_rsrc(packed + (R * cols * LO + (rb * cols + col0) * S));
    make_plane_rsrc<W, P + 1>(packed, R, cols, rb, col0, plane);
  }
}

// Where a lane works: its row block, its byte offset in the source from row 0 of
// row block rb0, and the tile's base (rb0, col0) in the (R, cols) plane arrays.
struct LanePlace {
  uint64_t rb0;
  uint64_t rb;
  uint32_t col0;
  uint32_t src_off;
  bool inside;
};

// kFold: a.tiles divides by the places per row block; else by the tiles per row block.
template <typename T, int kBlock, bool kFold>
__device__ __forceinline__ LanePlace lane_place(uint64_t tile, const RowsArgs& a, uint64_t R) {
  constexpr uint32_t kCols = 16 / sizeof(T);
  LanePlace p;
  uint32_t first;
  if constexpr (kFold) {
    tile_first_block(tile * kBlock, a.tiles, p.rb0, first);  // first: the tile's first place inside row block rb0
    const uint32_t j = first + threadIdx.x;
    const uint32_t d = lane_block<kBlock>(j, a.tiles);  // row blocks that start in between
    p.rb = p.rb0 + d;
    p.col0 = first * kCols;
    p.src_off = d * 8u * a.cols * (uint32_t)sizeof(T) + (j - d * a.tiles.size) * 16u;
    p.inside = p.rb < R;
  } else {
    tile_first_block(tile, a.tiles, p.rb0, first);  // first: the tile's number inside row block rb0
    p.rb = p.rb0;
    p.col0 = first * kBlock * kCols;
    p.src_off = p.col0 * (uint32_t)sizeof(T) + threadIdx.x * 16u;
    p.inside = p.col0 + threadIdx.x * kCols < a.cols;
  }
  return p;
}

// Metadata bytes of the 8 rows of a lane's row block, clamped later by derive_tc.
// Not folded: lane l fetches the byte of row 8 rb + (l & 7), one load for the whole
// (wave-uniform) block, and metadatum j is read from lane j - every lane of the
// wavefront must call load() and get().  Folded: a lane fetches its own 8 bytes.
template <bool kPerRow, bool kFold>
struct RowMetadata {
  uint32_t mv[kFold ? 8 : 1];
  __device__ __forceinline__ void load(const RowsArgs& a, const LanePlace& p) {
    if constexpr (!kPerRow) return;
    if constexpr (kFold) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const uint64_t row = 8 * p.rb + (uint32_t)j;
        mv[j] = p.inside && row < a.rows ? a.meta[row] : a.bc.meta_lo;
      }
    } else {
      const uint64_t row = 8 * p.rb + (threadIdx.x & 7u);
      mv[0] = row < a.rows ? a.meta[row] : a.bc.meta_lo;
    }
  }
  __device__ __forceinline__ uint32_t get(int j) const {
    if constexpr (kFold)
      return mv[j];
    else
      return (uint32_t)__builtin_amdgcn_readlane(mv[0], j);
  }
};

// Constants of the 8 rows (wave-uniform results unless folded).
//
// A metadatum so large that the fp32 rounding addend 2^(ec-127+23-Y) would overflow
// (max_exp > 231 + Y; values beyond 2^104) is handled without the fp64 variant: the
// row's values are multiplied by 2^-64 and its metadatum lowered by 64.  That is
// exact for every value that does not flush to zero anyway: in such a row the
// subnormal quantum is above 2^-46, while only values under 2^-62 underflow.
template <bool kPerRow, bool kFold>
__device__ __forceinline__ void row_constants(const RowsArgs& a, const RowMetadata<kPerRow, kFold>& md,
                                              TensorConsts tc[8], float pre[8], bool& any_pre) {
  bool lane_pre = false;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    pre[j] = 1.0f;
    if constexpr (kPerRow) {
      uint32_t me = min(max(md.get(j), a.bc.meta_lo), a.bc.meta_hi);
      if (me > a.bc.wide_above) {
        me -= 64u;
        pre[j] = as_f32((127u - 64u) << 23);
        lane_pre = true;
      }
      tc[j] = derive_tc(me, a.bc);
    } else {
      tc[j] = a.tc;
    }
  }
  any_pre = kFold ? __builtin_amdgcn_ballot_w64(lane_pre) != 0 : lane_pre;
}

// kPre: multiply row j by pre[j] first (see row_constants).
template <typename T, int W, int kCols, bool kWide, bool kPre>
__device__ __forceinline__ void encode_columns(const uint4 v[8], const FormatConsts& fc, const TensorConsts tc[8],
                                               const float pre[8], LaneWords<W, kCols>& lw) {
#pragma unroll
  for (int c = 0; c < kCols; ++c) {
    uint32_t u[8], f[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      u[j] = column_bits<T>(v[j], c);
      const uint32_t a = kPre ? as_u32(as_f32(u[j]) * pre[j]) : u[j];
      const uint32_t m = magnitude_code_left<kWide>(a, fc, tc[j]);
      f[j] = (W & 1) ? m : ((u[j] & 0x80000000u) | m);
    }
    peel_column<W, kCols, Planes<W>::count - 1>(f, u, c, lw);
  }
}

// kWide: per-tensor metadata only (per-row metadata never needs the fp64 variant, see row_constants).
// One tile per workgroup, tile = flat_tile().
template <typename T, int W, int kBlock, bool kPerRow, bool kWide, bool kFold>
__global__ __launch_bounds__(kBlock) void encode_rows_kernel(const RowsArgs args) {
  constexpr int kCols = 16 / sizeof(T);
  const uint8_t* __restrict__ src = static_cast<const uint8_t*>(args.src);
  uint8_t* __restrict__ dst = static_cast<uint8_t*>(args.dst);
  const FormatConsts fc = args.fc;
  const uint32_t cols = args.cols;
  const uint64_t R = (args.rows + 7) / 8;
  const uint32_t row_bytes = cols * (uint32_t)sizeof(T);

  const LanePlace p = lane_place<T, kBlock, kFold>(die_ranged_tile(args.xcd_chunk), args, R);
  if (p.rb0 >= R) return;  // workgroups past the last tile of a rounded-up grid
  RowMetadata<kPerRow, kFold> md;
  md.load(args, p);
  if (!kFold && !p.inside) return;  // folded: idle lanes stay for the ballot in row_constants
  const uint64_t left = p.inside ? args.rows - 8 * p.rb : 0;
  const uint32_t nrows = left < 8 ? (uint32_t)left : 8u;
  const rsrc_t in = make_rsrc(src + 8 * p.rb0 * cols * sizeof(T));
  uint4 v[8];
  if (args.xcd_chunk) {  // lines shared with the neighbouring tile: leave them in the L2 cache for it
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = j < (int)nrows ? load16<false>(in, p.src_off, j * row_bytes) : make_uint4(0, 0, 0, 0);
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = j < (int)nrows ? load16<true>(in, p.src_off, j * row_bytes) : make_uint4(0, 0, 0, 0);
  }  // rows past the end hold zero codes
  TensorConsts tc[8];
  float pre[8];
  bool any_pre;
  row_constants<kPerRow, kFold>(args, md, tc, pre, any_pre);
  if (kFold && !p.inside) return;
  LaneWords<W, kCols> lw;
  if constexpr (kPerRow) {
    if (any_pre)
      encode_columns<T, W, kCols, false, true>(v, fc, tc, pre, lw);
    else
      encode_columns<T, W, kCols, false, false>(v, fc, tc, pre, lw);
  } else {
    encode_columns<T, W, kCols, kWide, false>(v, fc, tc, pre, lw);
  }
  rsrc_t plane[Planes<W>::count];
  make_plane_rsrc<W>(dst, R, cols, p.rb0, p.col0, plane);
  move_words<W, kCols, true>(lw, plane, threadIdx.x);
}

// The plane bits of column c of the lane, in the form element_bits reads (a unit of 8 elements).
template <int W, int kCols, int P = 0>
__device__ __forceinline__ void column_unit(const LaneWords<W, kCols>& lw, int c, dec::UnitWords<W>& uw) {
  if constexpr (P < Planes<W>::count) {
    constexpr int S = Planes<W>::seg(P);
    if constexpr (S >= 4) {
#pragma unroll
      for (int k = 0; k < S / 4; ++k) uw.w[P][k] = lw.w[P][c * (S / 4) + k];
    } else if constexpr (S == 2) {
      uw.w[P][0] = lw.w[P][c / 2] >> (16 * (c & 1));
    } else {
      uw.w[P][0] = lw.w[P][c / 4] >> (8 * (c & 3));
    }
    column_unit<W, kCols, P + 1>(lw, c, uw);
  }
}

template <typename T, int W, int kBlock, bool kPerRow, bool kX8, bool kFold>
__global__ __launch_bounds__(kBlock) void decode_rows_kernel(const RowsArgs args) {
  constexpr int kCols = 16 / sizeof(T);
  uint8_t* __restrict__ src = static_cast<uint8_t*>(const_cast<void*>(args.src));
  uint8_t* __restrict__ dst = static_cast<uint8_t*>(args.dst);
  const FormatConsts fc = args.fc;
  const uint32_t cols = args.cols;
  const uint64_t R = (args.rows + 7) / 8;
  const uint32_t row_bytes = cols * (uint32_t)sizeof(T);

  const LanePlace p = lane_place<T, kBlock, kFold>(die_ranged_tile(args.xcd_chunk), args, R);
  if (p.rb0 >= R) return;
  RowMetadata<kPerRow, kFold> md;
  md.load(args, p);
  TensorConsts tc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) tc[j] = kPerRow ? derive_tc(md.get(j), args.bc) : args.tc;
  if (!p.inside) return;
  const uint64_t left = args.rows - 8 * p.rb;
  const uint32_t nrows = left < 8 ? (uint32_t)left : 8u;
  rsrc_t plane[Planes<W>::count];
  make_plane_rsrc<W>(src, R, cols, p.rb0, p.col0, plane);
  LaneWords<W, kCols> lw;
  move_words<W, kCols, false>(lw, plane, threadIdx.x);

  uint32_t o[8][4];  // the lane's 16 bytes of every row
#pragma unroll
  for (int c = 0; c < kCols; ++c) {
    dec::UnitWords<W> uw;
    column_unit<W, kCols>(lw, c, uw);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t b = dec::element_bits<W, kX8>(uw, j, fc, tc[j]);
      if constexpr (sizeof(T) == 4) {
        o[j][c] = b;
      } else {  // every value is exact in the 16-bit type: pair it with its neighbour
        if (c & 1)
          o[j][c / 2] = pack_elems<T>(o[j][c / 2], b);
        else
          o[j][c / 2] = b;
      }
    }
  }
  const rsrc_t out = make_rsrc(dst + 8 * p.rb0 * cols * sizeof(T));
  if (args.xcd_chunk) {  // lines shared with the neighbouring tile: let the L2 cache merge the two parts
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (j < (int)nrows) store16<false>(out, p.src_off, j * row_bytes, make_uint4(o[j][0], o[j][1], o[j][2], o[j][3]));
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (j < (int)nrows) store16<true>(out, p.src_off, j * row_bytes, make_uint4(o[j][0], o[j][1], o[j][2], o[j][3]));
  }
}

}  // namespace rows
}  // namespace exmy
