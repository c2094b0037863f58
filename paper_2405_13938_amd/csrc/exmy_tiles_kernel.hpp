// Blocks that are columns or 2-D tiles: the block shapes of Section 2 "Block Size"
// that are not runs of consecutive elements.
//
// The matrix is row-major and its codes are packed in its flat memory order, so the
// conversion kernels are the flat per-block kernels with a different metadata
// lookup: workgroup tiles run flat over the matrix, and every lane finds the
// metadatum of the 2-D tile its own run of elements lies in (see TileIndex).  A
// tile whose width is a multiple of 8 gives one metadatum per lane and step; with
// columns (width 1) every element has its own, read as the bytes that follow each
// other in the metadata row (kColumns).
//
// The maximum-exponent kernel walks 2-D regions instead: the lanes of a workgroup
// lie along matrix rows and step down the rows of one tile row, so that the
// reduction along a column stays in a lane's registers.
#pragma once

#include <type_traits>

#include "exmy_common.hpp"
#include "exmy_decode_kernel.hpp"
#include "exmy_emulate_kernel.hpp"
#include "exmy_encode_kernel.hpp"

namespace exmy {
namespace tiles {

// Metadata of one unit: a byte (2-D tiles), or kBytes consecutive bytes, one per
// element (columns), in one or two dwords.
template <int kBytes>
struct UnitMeta {
  uint32_t w[kBytes > 4 ? 2 : 1];
};

template <bool kColumns, int kElems>
__device__ __forceinline__ UnitMeta<kColumns ? kElems : 1> load_unit_meta(rsrc_t mt, uint32_t offset) {
  UnitMeta<kColumns ? kElems : 1> m;
  if constexpr (!kColumns) {
    m.w[0] = __builtin_amdgcn_raw_buffer_load_b8(mt, offset, 0, 0);
  } else if constexpr (kElems == 8) {
    const u32x2_t v = __builtin_amdgcn_raw_buffer_load_b64(mt, offset, 0, 0);
    m.w[0] = v.x;
    m.w[1] = v.y;
  } else {
    static_assert(kElems == 4, "units are 4 or 8 elements");
    m.w[0] = __builtin_amdgcn_raw_buffer_load_b32(mt, offset, 0, 0);
  }
  return m;
}

template <int kBytes>
__device__ __forceinline__ uint32_t meta_byte(const UnitMeta<kBytes>& m, int j) {
  return __builtin_amdgcn_ubfe(m.w[j / 4], 8 * (j % 4), 8);
}

// One metadatum per element: deriving a block's constants for every element would
// cost more than its conversion.  Instead the element is scaled by the power of two
// 2^(kRefExp - max_exp), converted with the constants of max_exp = kRefExp, and (on
// the way back) scaled by 2^(max_exp - kRefExp).  The format at max_exp is the
// format at kRefExp times that power of two, and the scalings are exact wherever
// it matters: kRefExp is high enough that every value of the reference format, and
// every value within a quarter of its quantum, is a normal float (2^X + Y + 1 <=
// 152 <= kRefExp), so a scaled element that loses bits to underflow lies far below
// half a quantum and rounds to zero either way; one that overflows lies far above
// the largest value and saturates either way; Inf and NaN stay what they are.
// kRefExp + 23 - Y <= 254 keeps the reference format on the fp32 rounding path.
constexpr uint32_t kRefExp = 160;

__device__ __forceinline__ TensorConsts reference_consts(BlockConsts bc) {
  bc.meta_lo = 0;  // kRefExp is taken as it is, whatever range the container allows for real metadata
  bc.meta_hi = 255;
  return derive_tc(kRefExp, bc);
}

// kRefExp - max_exp (kBack: max_exp - kRefExp) for element j of the unit, max_exp read as the nearest valid value.
// Two instructions: the subtraction takes the byte straight out of the metadata dword through its operand's
// byte select, and one median clamps the difference (max_exp in [lo, hi] <=> kRefExp - max_exp in
// [kRefExp - hi, kRefExp - lo]); extracting, clamping with a maximum and a minimum and subtracting took five.
template <bool kBack, int kBytes>
__device__ __forceinline__ int ref_shift(const UnitMeta<kBytes>& m, int j, const BlockConsts& bc) {
  const uint32_t w = m.w[j / 4], ref = kRefExp;
  int d;
  if (!kBack) {
    if (j % 4 == 0) asm("v_sub_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0" : "=v"(d) : "v"(ref), "v"(w));
    if (j % 4 == 1) asm("v_sub_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(d) : "v"(ref), "v"(w));
    if (j % 4 == 2) asm("v_sub_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2" : "=v"(d) : "v"(ref), "v"(w));
    if (j % 4 == 3) asm("v_sub_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(d) : "v"(ref), "v"(w));
  } else {
    if (j % 4 == 0) asm("v_sub_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_0 src1_sel:DWORD" : "=v"(d) : "v"(w), "v"(ref));
    if (j % 4 == 1) asm("v_sub_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_1 src1_sel:DWORD" : "=v"(d) : "v"(w), "v"(ref));
    if (j % 4 == 2) asm("v_sub_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_2 src1_sel:DWORD" : "=v"(d) : "v"(w), "v"(ref));
    if (j % 4 == 3) asm("v_sub_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_3 src1_sel:DWORD" : "=v"(d) : "v"(w), "v"(ref));
  }
  const int lo = kBack ? (int)bc.meta_lo - (int)kRefExp : (int)kRefExp - (int)bc.meta_hi;
  const int hi = kBack ? (int)bc.meta_hi - (int)kRefExp : (int)kRefExp - (int)bc.meta_lo;
  int r;
  asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(d), "s"(lo), "v"(hi));
  return r;
}

// fp32 bits of |x| * 2^shift for the element with fp32-position bits u.
__device__ __forceinline__ uint32_t scaled_magnitude(uint32_t u, int shift) {
  return as_u32(ldexpf(__builtin_fabsf(as_f32(u)), shift));
}

// ---------------------------------------------------------------- encode

// One group whose 8 elements have a metadatum each.
template <int W, class Dst>
__device__ __forceinline__ void encode_group_each(const uint32_t u[8], const UnitMeta<8>& me, const FormatConsts& fc,
                                                  const BlockConsts& bc, const TensorConsts& tc_ref, const Dst& pd,
                                                  uint32_t lane_group, uint32_t tile_group) {
  uint32_t f[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const uint32_t m = magnitude_code_left<false>(scaled_magnitude(u[j], ref_shift<false>(me, j, bc)), fc, tc_ref);
    f[j] = (W & 1) ? m : ((u[j] & 0x80000000u) | m);
  }
  enc::peel_planes<W, Planes<W>::count - 1>(f, u, pd, lane_group, tile_group);
}

// A unit is one group of 8 elements.  n = rows * cols is a multiple of 8.
template <typename T, int W, int kBlock, int kUnroll, bool kNT, bool kColumns>
__global__ __launch_bounds__(kBlock) void encode_tiles_kernel(const TileArgs args) {
  constexpr uint32_t TG = kBlock * kUnroll;
  constexpr int kLoads = enc::TileRegs<T, kUnroll>::kLoads;
  const uint4* __restrict__ src4 = static_cast<const uint4*>(args.src);
  uint8_t* __restrict__ dst = static_cast<uint8_t*>(args.dst);
  const FormatConsts fc = args.fc;
  const BlockConsts bc = args.bc;
  const TileIndex ti = args.ti;  // in groups
  const TensorConsts tc_ref = reference_consts(bc);
  const uint64_t G = args.rows * args.cols / 8;
  const uint32_t full_tiles = (uint32_t)(G / TG);
  const uint32_t rem_groups = (uint32_t)(G - (uint64_t)full_tiles * TG);
  const uint32_t tiles = full_tiles + (rem_groups ? 1u : 0u);
  __shared__ __align__(16) uint8_t lds_stage[TG * W];
  const enc::PlaneStage<W, TG> stage{lds_stage};

  for (uint32_t tile = flat_tile(), once = 1; once && tile < tiles; once = 0) {
    const uint64_t g0 = (uint64_t)tile * TG;
    const TileStart ts = tile_start<TG, kColumns>(g0, ti);
    const rsrc_t src = make_rsrc(src4 + g0 * kLoads);
    const rsrc_t mt = make_rsrc(args.meta + ts.meta_row);
    enc::PlaneDst<W> pd;
    enc::make_plane_dst<W>(dst, G, g0, pd);
    enc::TileRegs<T, kUnroll> regs;
    UnitMeta<kColumns ? 8 : 1> me[kUnroll];
    // whole tiles take the path without bounds checks and write their plane words through the LDS stage
    auto body = [&](auto guard, const auto& out) {
      constexpr bool kGuard = decltype(guard)::value;
      enc::load_tile<T, kBlock, kUnroll, kNT, kGuard>(src, 0, rem_groups, regs);
      const uint32_t slot = kGuard ? threadIdx.x : enc::row_slot<T, kBlock>();  // the lane's group of a tile row
#pragma unroll
      for (int r = 0; r < kUnroll; ++r)
        if (!kGuard || r * kBlock + slot < rem_groups)
          me[r] = load_unit_meta<kColumns, 8>(mt, tile_meta_offset<TG, kColumns>(r * kBlock + slot, ti, ts));
#pragma unroll
      for (int r = 0; r < kUnroll; ++r) {
        if (!kGuard || r * kBlock + slot < rem_groups) {  // the rounding-variant vote is among the lanes that get here
          uint32_t u[8];
          enc::group_bits<T, !kGuard>(regs.v[r], u);
          if constexpr (kColumns)
            encode_group_each<W>(u, me[r], fc, bc, tc_ref, out, slot, r * kBlock);
          else
            enc::encode_group_meta<W>(u, me[r].w[0], fc, bc, out, slot, r * kBlock);
        }
      }
    };
    if (tile < full_tiles) {
      body(std::false_type{}, stage);
      enc::flush_stage<W, TG, kBlock>(stage, dst, G, g0);
    } else {
      body(std::true_type{}, pd);
    }
  }
}

// ---------------------------------------------------------------- decode

// Values of one unit whose elements have a metadatum each.
template <typename T, int W, bool kNT>
__device__ __forceinline__ void decode_unit_each(const dec::UnitWords<W>& uw, const FormatConsts& fc,
                                                 const BlockConsts& bc, const TensorConsts& tc_ref,
                                                 const UnitMeta<16 / sizeof(T)>& me, rsrc_t out, uint32_t lane_unit,
                                                 uint32_t tile_unit) {
  constexpr int E = 16 / sizeof(T);
  uint32_t b[E];
#pragma unroll
  for (int j = 0; j < E; ++j)  // the sign rides through the scaling
    b[j] = as_u32(ldexpf(as_f32(dec::element_bits<W, false>(uw, j, fc, tc_ref)), ref_shift<true>(me, j, bc)));
  if constexpr (sizeof(T) == 4) {
    store16<kNT>(out, lane_unit * 16, tile_unit * 16, make_uint4(b[0], b[1], b[2], b[3]));
  } else {
    uint4 o;
    o.x = pack_elems<T>(b[0], b[1]);
    o.y = pack_elems<T>(b[2], b[3]);
    o.z = pack_elems<T>(b[4], b[5]);
    o.w = pack_elems<T>(b[6], b[7]);
    store16<kNT>(out, lane_unit * 16, tile_unit * 16, o);
  }
}

// A unit is one lane's 16 bytes of output (E elements).
template <typename T, int W, int kBlock, int kUnroll, bool kNT, bool kColumns>
__global__ __launch_bounds__(kBlock) void decode_tiles_kernel(const TileArgs args) {
  constexpr uint32_t TU = kBlock * kUnroll;
  constexpr int E = 16 / sizeof(T);
  const uint8_t* __restrict__ src = static_cast<const uint8_t*>(args.src);
  T* __restrict__ dst = static_cast<T*>(args.dst);
  const FormatConsts fc = args.fc;
  const BlockConsts bc = args.bc;
  const TileIndex ti = args.ti;  // in units
  const TensorConsts tc_ref = reference_consts(bc);
  const uint64_t n = args.rows * args.cols;
  const uint64_t G = n / 8;
  const uint64_t U = n / E;
  const uint32_t full_tiles = (uint32_t)(U / TU);
  const uint32_t rem_units = (uint32_t)(U - (uint64_t)full_tiles * TU);
  const uint32_t tiles = full_tiles + (rem_units ? 1u : 0u);

  for (uint32_t tile = flat_tile(), once = 1; once && tile < tiles; once = 0) {
    const uint64_t u0 = (uint64_t)tile * TU;  // even
    const TileStart ts = tile_start<TU, kColumns>(u0, ti);
    dec::PlaneSrc<W> ps;
    dec::make_plane_src<W, E>(src, G, u0, ps);
    const rsrc_t out = make_rsrc(reinterpret_cast<uint4*>(dst) + u0);
    const rsrc_t mt = make_rsrc(args.meta + ts.meta_row);
    dec::TileWords<W, kUnroll> tw;
    UnitMeta<kColumns ? E : 1> me[kUnroll];
    auto body = [&](auto guard) {
      constexpr bool kGuard = decltype(guard)::value;
      dec::load_tile<W, E, kBlock, kUnroll, kGuard>(ps, 0, rem_units, tw);
#pragma unroll
      for (int r = 0; r < kUnroll; ++r)
        if (!kGuard || r * kBlock + threadIdx.x < rem_units)
          me[r] = load_unit_meta<kColumns, E>(mt, tile_meta_offset<TU, kColumns>(r * kBlock + threadIdx.x, ti, ts));
#pragma unroll
      for (int r = 0; r < kUnroll; ++r) {
        if (!kGuard || r * kBlock + threadIdx.x < rem_units) {
          if constexpr (kColumns)
            decode_unit_each<T, W, kNT>(tw.u[r], fc, bc, tc_ref, me[r], out, threadIdx.x, r * kBlock);
          else
            dec::decode_unit<T, W, false, kNT>(tw.u[r], fc, derive_tc(me[r].w[0], bc), out, threadIdx.x, r * kBlock);
        }
      }
    };
    if (tile < full_tiles)
      body(std::false_type{});
    else
      body(std::true_type{});
  }
}

// ---------------------------------------------------------------- emulate

// In emulation the scaling would be needed twice (there and back), which costs more
// than deriving the element's own constants.
template <typename T, bool kWide>
__device__ __forceinline__ uint4 emulate_vector_each_as(uint4 v, const UnitMeta<16 / sizeof(T)>& me,
                                                        const FormatConsts& fc, const BlockConsts& bc) {
  uint32_t w[4] = {v.x, v.y, v.z, v.w};
  if constexpr (sizeof(T) == 2 && !kIsF16<T>) {  // bf16: signs per pair, Inf / NaN only where a wavefront holds one (see emulate_vector)
    uint32_t out[4];
    uint32_t top = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint32_t lo = emu::emulate_magnitude<kWide>((w[k] << 16) & 0x7FFFFFFFu, fc, derive_tc(meta_byte(me, 2 * k), bc));
      const uint32_t hi = emu::emulate_magnitude<kWide>(w[k] & 0x7FFF0000u, fc, derive_tc(meta_byte(me, 2 * k + 1), bc));
      out[k] = bit_select(0x7FFF7FFFu, pack_elems<T>(lo, hi), w[k]);
      top = max_pair_keys(top, w[k] & 0x7FFF7FFFu);
    }
    if (__builtin_amdgcn_ballot_w64(((top + 0x00800080u) & 0x80008000u) != 0) != 0) {
#pragma unroll
      for (int k = 0; k < 4; ++k) out[k] = keep_nonfinite_bf16(w[k], out[k]);
    }
    return make_uint4(out[0], out[1], out[2], out[3]);
  }
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    if constexpr (sizeof(T) == 4) {
      w[k] = emu::emulate_bits<kWide>(w[k], fc, derive_tc(meta_byte(me, k), bc));
    } else {
      const uint32_t lo = emu::emulate_bits<kWide>(lo_elem_bits<T>(w[k]), fc, derive_tc(meta_byte(me, 2 * k), bc));
      const uint32_t hi = emu::emulate_bits<kWide>(hi_elem_bits<T>(w[k]), fc, derive_tc(meta_byte(me, 2 * k + 1), bc));
      const uint32_t pair = pack_elems<T>(lo, hi);
      w[k] = kIsF16<T> ? keep_nonfinite_halves(w[k], pair) : pair;
    }
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// The rounding variant is chosen for a whole wavefront at once, as in emulate_vector_meta.
template <typename T>
__device__ __forceinline__ uint4 emulate_vector_each(uint4 v, const UnitMeta<16 / sizeof(T)>& me, bool wide_format,
                                                     const FormatConsts& fc, const BlockConsts& bc) {
  constexpr int E = 16 / sizeof(T);
  bool wide = wide_format;
#pragma unroll
  for (int j = 0; j < E; ++j) wide |= meta_byte(me, j) > bc.wide_above;
  if (__builtin_amdgcn_ballot_w64(wide) != 0) return emulate_vector_each_as<T, true>(v, me, fc, bc);
  return emulate_vector_each_as<T, false>(v, me, fc, bc);
}

// A unit is one 16-byte vector.  wide_format: the format itself needs the fp64 path.
template <typename T, int kBlock, int kUnroll, bool kNT, bool kColumns>
__global__ __launch_bounds__(kBlock) void emulate_tiles_kernel(const TileArgs args, bool wide_format) {
  constexpr int E = 16 / sizeof(T);
  constexpr uint32_t TV = kBlock * kUnroll;
  T* __restrict__ data = static_cast<T*>(const_cast<void*>(args.src));
  const FormatConsts fc = args.fc;
  const BlockConsts bc = args.bc;
  const TileIndex ti = args.ti;  // in vectors
  const uint64_t V = args.rows * args.cols / E;
  const uint32_t lane_off = threadIdx.x * 16;
  const uint32_t tiles = (uint32_t)((V + TV - 1) / TV);

  for (uint32_t tile = flat_tile(), once = 1; once && tile < tiles; once = 0) {
    const uint64_t v0 = (uint64_t)tile * TV;
    const TileStart ts = tile_start<TV, kColumns>(v0, ti);
    const rsrc_t buf = make_rsrc(reinterpret_cast<uint4*>(data) + v0);
    const rsrc_t mt = make_rsrc(args.meta + ts.meta_row);
    const uint64_t left = V - v0;
    const uint32_t rem = left < TV ? (uint32_t)left : TV;
    uint4 v[kUnroll];
    UnitMeta<kColumns ? E : 1> me[kUnroll];
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      if (r * kBlock + threadIdx.x < rem) {
        v[r] = load16<kNT>(buf, lane_off, r * kBlock * 16);
        me[r] = load_unit_meta<kColumns, E>(mt, tile_meta_offset<TV, kColumns>(r * kBlock + threadIdx.x, ti, ts));
      }
    }
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      if (r * kBlock + threadIdx.x < rem) {
        if constexpr (kColumns)
          store16<kNT>(buf, lane_off, r * kBlock * 16, emulate_vector_each<T>(v[r], me[r], wide_format, fc, bc));
        else
          store16<kNT>(buf, lane_off, r * kBlock * 16, emu::emulate_vector_meta<T>(v[r], me[r].w[0], wide_format, fc, bc, true));
      }
    }
  }
}

// ---------------------------------------------------------------- maximum exponent

// Clears the whole 4-byte words of the `bytes` metadata bytes at p (4-byte aligned)
// before the maximum kernel folds into them.  The 1-3 bytes of a last partial word
// are not touched here: tile_max_exp_tail_kernel writes them.
template <int kBlock>
__global__ __launch_bounds__(kBlock) void clear_words_kernel(uint8_t* __restrict__ p, uint64_t bytes) {
  const uint64_t words = bytes / 4;
  const uint64_t first = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  for (uint64_t i = first; i < words; i += (uint64_t)gridDim.x * kBlock) reinterpret_cast<uint32_t*>(p)[i] = 0u;
}

// Byte-wise maximum of two words.
__device__ __forceinline__ uint32_t max_bytes(uint32_t a, uint32_t b) {
  uint32_t r = 0;
#pragma unroll
  for (int k = 0; k < 4; ++k) r |= max((a >> (8 * k)) & 0xFFu, (b >> (8 * k)) & 0xFFu) << (8 * k);
  return r;
}

// *p = byte-wise max(*p, mine); other workgroups fold into the same word at the
// same time.  Every failed exchange means another workgroup raised a byte, and
// bytes only grow, so the loop ends.
__device__ __forceinline__ void atomic_max_bytes(uint32_t* p, uint32_t mine) {
  uint32_t old = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  for (;;) {
    const uint32_t want = max_bytes(old, mine);
    if (want == old) return;
    const uint32_t seen = atomicCAS(p, old, want);
    if (seen == old) return;
    old = seen;
  }
}

// Launch geometry of the maximum kernel (host and device agree through these).
// The kBlock lanes of a workgroup form `lanes_y` rows of `lanes_x` lanes: lane
// (lx, ly) reads vector lx of its column strip in matrix rows ly, ly + lanes_y, ...
// of its row chunk.  A region is one column strip x one chunk of `chunk_rows`
// matrix rows of one tile row.
struct MaxGeometry {
  uint32_t vpr;          // 16-byte vectors per matrix row
  uint32_t lanes_x_log2;
  uint32_t row_steps;    // matrix rows per lane and region (a multiple of 4)
  uint32_t chunk_rows;   // matrix rows per region: lanes_y * row_steps
  uint32_t strips;       // column strips per matrix row
  uint32_t chunks;       // row chunks per tile row
  uint64_t tile_rows_n;  // tile rows
  uint64_t regions;      // strips * chunks * tile_rows_n
  BlockIndex tcv;        // tile width in vectors (2-D tiles only)
  // The metadata array is folded into with 32-bit atomic operations.  When its size is not a multiple of 4
  // the last word would reach past its end, into memory that is not the library's to read or write: the
  // tiles of those 1-3 bytes are left out here (tail_word = index of that word, else ~0) and computed by
  // tile_max_exp_tail_kernel, one workgroup per tile, with byte stores.
  uint64_t tail_word;
};

// Slots of the workgroup's partial maxima in LDS: one per tile column that the
// strip touches (2-D tiles), or one per matrix column of the strip (columns).
constexpr int kMaxSlots = 256 * 8;

template <typename T, int kBlock, bool kColumns>
__global__ __launch_bounds__(kBlock) void tile_max_exp_kernel(const TileArgs args, const MaxGeometry geo) {
  constexpr int E = 16 / sizeof(T);
  constexpr int kBatch = 4;  // loads in flight per lane
  __shared__ int32_t slot[kMaxSlots];
  const u32x4_t* __restrict__ src4 = static_cast<const u32x4_t*>(args.src);
  const BlockConsts bc = args.bc;
  const uint32_t lanes_x = 1u << geo.lanes_x_log2;
  const uint32_t lanes_y = kBlock >> geo.lanes_x_log2;
  const uint32_t lx = threadIdx.x & (lanes_x - 1u);
  const uint32_t ly = threadIdx.x >> geo.lanes_x_log2;

  for (uint64_t region = blockIdx.x; region < geo.regions; region += gridDim.x) {
    // region -> (tile row, chunk, strip), strips fastest so that neighbouring workgroups read neighbouring columns
    const uint64_t per_tile_row = (uint64_t)geo.strips * geo.chunks;
    const uint64_t tb = region / per_tile_row;
    const uint32_t in_tile_row = (uint32_t)(region - tb * per_tile_row);
    const uint32_t chunk = in_tile_row / geo.strips;
    const uint32_t strip = in_tile_row - chunk * geo.strips;

    const uint64_t row_begin = tb * args.tile_rows + (uint64_t)chunk * geo.chunk_rows;
    const uint64_t band_end = min(args.rows, (tb + 1) * args.tile_rows);
    const uint64_t row_end = min(band_end, row_begin + geo.chunk_rows);
    const uint32_t cv0 = strip << geo.lanes_x_log2;            // first vector column of the strip
    const uint32_t cv = cv0 + lx;
    // tile columns that the strip touches (2-D tiles), or its matrix columns
    uint32_t first_slot_col, n_slots;
    if constexpr (kColumns) {
      first_slot_col = cv0 * E;
      n_slots = min(lanes_x, geo.vpr - cv0) * E;
    } else {
      uint64_t q;
      uint32_t r;
      tile_first_block(cv0, geo.tcv, q, r);
      first_slot_col = (uint32_t)q;
      const uint32_t last_cv = min(cv0 + lanes_x, geo.vpr) - 1u;
      tile_first_block(last_cv, geo.tcv, q, r);
      n_slots = (uint32_t)q - first_slot_col + 1u;
    }
    for (uint32_t i = threadIdx.x; i < n_slots; i += kBlock) slot[i] = kNoKey;
    __syncthreads();

    if (row_begin < row_end && cv < geo.vpr) {
      constexpr bool kPairs = kColumns && std::is_same<T, uint16_t>::value;  // bf16 columns: keys in packed pairs
      int32_t key[kColumns ? E : 1];
      uint32_t pairs[4] = {kNoPairKeys, kNoPairKeys, kNoPairKeys, kNoPairKeys};
#pragma unroll
      for (int e = 0; e < (kColumns ? E : 1); ++e) key[e] = kNoKey;
      for (uint32_t s0 = 0; s0 < geo.row_steps; s0 += kBatch) {
        uint4 v[kBatch];
        bool have[kBatch];
#pragma unroll
        for (int s = 0; s < kBatch; ++s) {
          const uint64_t row = row_begin + ly + (uint64_t)(s0 + s) * lanes_y;
          have[s] = row < row_end;
          if (have[s]) {
            const u32x4_t x = __builtin_nontemporal_load(src4 + (row * geo.vpr + cv));
            v[s] = make_uint4(x.x, x.y, x.z, x.w);
          }
        }
#pragma unroll
        for (int s = 0; s < kBatch; ++s) {
          if (have[s]) {
            if constexpr (kColumns) {
              const uint32_t w[4] = {v[s].x, v[s].y, v[s].z, v[s].w};
#pragma unroll
              for (int k = 0; k < 4; ++k) {
                if constexpr (kPairs) {
                  pairs[k] = max_pair_keys(pairs[k], pair_keys(w[k]));
                } else if constexpr (sizeof(T) == 4) {
                  key[k] = max(key[k], exp_key(w[k]));
                } else {
                  key[2 * k] = max(key[2 * k], exp_key(lo_elem_bits<T>(w[k])));
                  key[2 * k + 1] = max(key[2 * k + 1], exp_key(hi_elem_bits<T>(w[k])));
                }
              }
            } else {
              key[0] = max(key[0], emu::vector_exp_key<T>(v[s]));
            }
          }
        }
      }
      if constexpr (kPairs) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          key[2 * k] = (int32_t)(pairs[k] << 16);
          key[2 * k + 1] = (int32_t)(pairs[k] & 0xFFFF0000u);
        }
      }
      if constexpr (kColumns) {
#pragma unroll
        for (int e = 0; e < E; ++e) atomicMax(&slot[lx * E + e], key[e]);
      } else {
        uint64_t q;
        uint32_t r;
        tile_first_block(cv, geo.tcv, q, r);
        atomicMax(&slot[(uint32_t)q - first_slot_col], key[0]);
      }
    }
    __syncthreads();

    // Fold the slots into the metadata bytes of this tile row, a word at a time.
    if (row_begin < row_end) {
      const uint64_t t_first = tb * args.ti.meta_stride + first_slot_col;  // byte index of slot 0
      const uint64_t word_first = t_first / 4;
      const uint32_t n_words = (uint32_t)((t_first + n_slots - 1) / 4 - word_first) + 1u;
      for (uint32_t wd = threadIdx.x; wd < n_words; wd += kBlock) {
        if (word_first + wd == geo.tail_word) continue;
        uint32_t mine = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const uint64_t t = (word_first + wd) * 4 + k;
          if (t >= t_first && t < t_first + n_slots) mine |= meta_from_key(slot[(uint32_t)(t - t_first)], bc) << (8 * k);
        }
        atomic_max_bytes(reinterpret_cast<uint32_t*>(args.meta) + (word_first + wd), mine);
      }
    }
    __syncthreads();  // the slots are cleared again by the next region
  }
}

// The metadata of the tiles number first_tile + blockIdx.x (row-major over the tiles): one workgroup
// walks one whole 2-D tile and stores its byte, so no word is shared with anything.  Used for the tiles
// whose bytes lie in a last partial 4-byte word of the metadata array (see MaxGeometry::tail_word).
// lanes_x_log2: the workgroup's lanes form rows of 2^lanes_x_log2 lanes along the tile's 16-byte vectors.
template <typename T, int kBlock>
__global__ __launch_bounds__(kBlock) void tile_max_exp_tail_kernel(const TileArgs args, uint64_t first_tile,
                                                                   uint32_t lanes_x_log2) {
  constexpr int E = 16 / sizeof(T);
  constexpr int kBatch = 4;  // loads in flight per lane
  __shared__ int32_t wave_key[kBlock / 64];
  const u32x4_t* __restrict__ src4 = static_cast<const u32x4_t*>(args.src);
  const uint64_t tile = first_tile + blockIdx.x;
  const uint64_t tb = tile / args.tiles_along_row, tc = tile - tb * args.tiles_along_row;
  const uint64_t row_begin = tb * args.tile_rows, row_end = min(args.rows, row_begin + args.tile_rows);
  const uint64_t vpr = args.cols / E;
  const uint64_t cv_begin = tc * (args.tile_cols / E), cv_end = min(vpr, cv_begin + args.tile_cols / E);
  const uint32_t lanes_x = 1u << lanes_x_log2, lanes_y = kBlock >> lanes_x_log2;
  const uint32_t lx = threadIdx.x & (lanes_x - 1u), ly = threadIdx.x >> lanes_x_log2;
  int32_t key = kNoKey;
  for (uint64_t cv = cv_begin + lx; cv < cv_end; cv += lanes_x) {
    for (uint64_t row0 = row_begin + ly; row0 < row_end; row0 += (uint64_t)kBatch * lanes_y) {
      uint4 v[kBatch];
      bool have[kBatch];
#pragma unroll
      for (int s = 0; s < kBatch; ++s) {
        const uint64_t row = row0 + (uint64_t)s * lanes_y;
        have[s] = row < row_end;
        if (have[s]) {
          const u32x4_t x = __builtin_nontemporal_load(src4 + (row * vpr + cv));
          v[s] = make_uint4(x.x, x.y, x.z, x.w);
        }
      }
#pragma unroll
      for (int s = 0; s < kBatch; ++s)
        if (have[s]) key = max(key, emu::vector_exp_key<T>(v[s]));
    }
  }
  key = max_over_lanes(key, 6);
  if ((threadIdx.x & 63u) == 0) wave_key[threadIdx.x >> 6] = key;
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < kBlock / 64; ++w) key = max(key, wave_key[w]);
    args.meta[tile] = (uint8_t)meta_from_key(key, args.bc);
  }
}

}  // namespace tiles
}  // namespace exmy
