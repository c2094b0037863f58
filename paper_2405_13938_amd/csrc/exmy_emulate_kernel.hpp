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

// ---------------------------------------------------------------------------
// Per-block metadata: see the encoder for the two launch modes.  Work is counted
// in 16-byte vectors of kPer elements; blocks hold block_groups * 8 / kPer of them.

template <typename T>
__device__ __forceinline__ uint4 emulate_vector_meta(uint4 v, uint32_t me, bool wide_format, const FormatConsts& fc,
                                                     const BlockConsts& bc) {
  const TensorConsts tc = derive_tc(me, bc);
  if (__builtin_amdgcn_ballot_w64(wide_format || me > bc.wide_above) != 0) return emulate_vector<T, true>(v, fc, tc);
  return emulate_vector<T, false>(v, fc, tc);
}

// wide_format: the format itself needs the fp64 path (Y > 21), whatever the metadata.
template <typename T, int kBlock, int kUnroll, bool kRows, bool kNT>
__global__ __launch_bounds__(kBlock) void emulate_blocks_kernel(const BlockArgs args, bool wide_format) {
  constexpr int kPer = 16 / sizeof(T);
  constexpr int kVecsPerGroupLog2 = sizeof(T) == 4 ? 1 : 0;
  constexpr uint32_t TV = kBlock * kUnroll;
  T* __restrict__ data = static_cast<T*>(const_cast<void*>(args.src));
  const uint8_t* __restrict__ meta = args.meta;
  const uint64_t n = args.n;
  const FormatConsts fc = args.fc;
  const BlockConsts bc = args.bc;
  const uint64_t V = n / kPer;
  const uint32_t lane_off = threadIdx.x * 16;

  if constexpr (kRows) {
    const uint64_t row = blockIdx.y + (uint64_t)blockIdx.z * gridDim.y;
    if (row >= args.n_blocks) return;
    const uint32_t me = __builtin_amdgcn_readfirstlane((uint32_t)meta[row]);
    const uint32_t block_vecs = args.block_groups << kVecsPerGroupLog2;
    const uint64_t row_v0 = row * block_vecs;
    const uint64_t left = V - row_v0;
    const uint32_t row_vecs = left < block_vecs ? (uint32_t)left : block_vecs;
    const uint32_t tiles = (row_vecs + TV - 1) / TV;
    for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
      const rsrc_t buf = make_rsrc(reinterpret_cast<uint4*>(data) + row_v0 + (uint64_t)tile * TV);
      const uint32_t rem = row_vecs - tile * TV;  // >= TV on whole tiles
      uint4 v[kUnroll];
#pragma unroll
      for (int r = 0; r < kUnroll; ++r)
        if (r * kBlock + threadIdx.x < rem) v[r] = load16<kNT>(buf, lane_off, r * kBlock * 16);
#pragma unroll
      for (int r = 0; r < kUnroll; ++r)
        if (r * kBlock + threadIdx.x < rem)
          store16<kNT>(buf, lane_off, r * kBlock * 16, emulate_vector_meta<T>(v[r], me, wide_format, fc, bc));
    }
  } else {
    const uint32_t lg = args.block_groups_log2 + kVecsPerGroupLog2;
    const uint32_t tiles = (uint32_t)((V + TV - 1) / TV);
    for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
      const uint64_t v0 = (uint64_t)tile * TV;
      const rsrc_t buf = make_rsrc(reinterpret_cast<uint4*>(data) + v0);
      const rsrc_t mt = make_rsrc(meta + (v0 >> lg));
      const uint64_t left = V - v0;
      const uint32_t rem = left < TV ? (uint32_t)left : TV;
      uint4 v[kUnroll];
      uint32_t me[kUnroll];
#pragma unroll
      for (int r = 0; r < kUnroll; ++r) {
        if (r * kBlock + threadIdx.x < rem) {
          v[r] = load16<kNT>(buf, lane_off, r * kBlock * 16);
          me[r] = __builtin_amdgcn_raw_buffer_load_b8(mt, (r * kBlock + threadIdx.x) >> lg, 0, 0);
        }
      }
#pragma unroll
      for (int r = 0; r < kUnroll; ++r)
        if (r * kBlock + threadIdx.x < rem)
          store16<kNT>(buf, lane_off, r * kBlock * 16, emulate_vector_meta<T>(v[r], me[r], wide_format, fc, bc));
    }
  }

  // Elements past the last whole 16-byte vector belong to the last block.
  const bool last = kRows ? (blockIdx.y + (uint64_t)blockIdx.z * gridDim.y == args.n_blocks - 1) : true;
  if (last && blockIdx.x == 0 && threadIdx.x < kPer) {
    const uint64_t i = V * kPer + threadIdx.x;
    if (i < n) {
      const uint32_t me = meta[args.n_blocks - 1];
      const TensorConsts tc = derive_tc(me, bc);
      const bool wide = __builtin_amdgcn_ballot_w64(wide_format || me > bc.wide_above) != 0;
      if constexpr (sizeof(T) == 4) {
        uint32_t* p = reinterpret_cast<uint32_t*>(data) + i;
        *p = wide ? emulate_bits<true>(*p, fc, tc) : emulate_bits<false>(*p, fc, tc);
      } else {
        uint16_t* p = reinterpret_cast<uint16_t*>(data) + i;
        const uint32_t u = (uint32_t)*p << 16;
        *p = (uint16_t)((wide ? emulate_bits<true>(u, fc, tc) : emulate_bits<false>(u, fc, tc)) >> 16);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// "Maximum exponent before rounding" of every block (Section 2 "Metadata"): the
// largest biased exponent among the block's finite elements, clamped into the
// valid range.  Adding 1 to the exponent field turns Inf / NaN patterns negative
// as signed integers, so a signed maximum skips them.

template <typename T, typename V4>
__device__ __forceinline__ int32_t vector_exp_key(V4 v) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  int32_t m = (int32_t)0x80000000;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    if constexpr (sizeof(T) == 4) {
      m = max(m, (int32_t)((w[k] & 0x7FFFFFFFu) + 0x00800000u));
    } else {
      m = max(m, (int32_t)(((w[k] << 16) & 0x7FFFFFFFu) + 0x00800000u));
      m = max(m, (int32_t)((w[k] & 0x7FFF0000u) + 0x00800000u));
    }
  }
  return m;
}

template <typename T>
__device__ __forceinline__ int32_t element_exp_key(const T* p) {
  uint32_t u;
  if constexpr (sizeof(T) == 4)
    u = *reinterpret_cast<const uint32_t*>(p);
  else
    u = (uint32_t)*reinterpret_cast<const uint16_t*>(p) << 16;
  return (int32_t)((u & 0x7FFFFFFFu) + 0x00800000u);
}

__device__ __forceinline__ uint8_t key_to_meta(int32_t key, const BlockConsts& bc) {
  const uint32_t e = key > 0 ? ((uint32_t)key >> 23) - 1u : 0u;  // no finite element: exponent 0
  return (uint8_t)min(max(e, bc.meta_lo), bc.meta_hi);
}

template <typename T, int kBlock, bool kRows>
__global__ __launch_bounds__(kBlock) void block_max_exp_kernel(const BlockArgs args) {
  constexpr int kPer = 16 / sizeof(T);
  constexpr int kVecsPerGroupLog2 = sizeof(T) == 4 ? 1 : 0;
  const T* __restrict__ src = static_cast<const T*>(args.src);
  const uint4* __restrict__ src4 = static_cast<const uint4*>(args.src);
  uint8_t* __restrict__ meta = args.meta;
  const uint64_t n = args.n;
  const BlockConsts bc = args.bc;
  const uint64_t V = n / kPer;  // whole vectors

  if constexpr (kRows) {
    __shared__ int32_t part[kBlock / 64];
    const uint64_t row = blockIdx.y + (uint64_t)blockIdx.z * gridDim.y;
    if (row >= args.n_blocks) return;
    const uint32_t block_vecs = args.block_groups << kVecsPerGroupLog2;
    const uint64_t row_v0 = row * block_vecs;
    const uint64_t left = V - row_v0;
    const uint32_t row_vecs = left < block_vecs ? (uint32_t)left : block_vecs;
    const rsrc_t buf = make_rsrc(src4 + row_v0);
    int32_t m = (int32_t)0x80000000;
    for (uint32_t i = threadIdx.x; i < row_vecs; i += kBlock) m = max(m, vector_exp_key<T>(load16<true>(buf, i * 16, 0)));
    if (row == args.n_blocks - 1 && threadIdx.x < kPer) {  // elements past the last whole vector
      const uint64_t i = V * kPer + threadIdx.x;
      if (i < n) m = max(m, element_exp_key<T>(src + i));
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) m = max(m, __shfl_xor(m, d, 64));
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
      for (int w = 1; w < kBlock / 64; ++w) m = max(m, part[w]);
      meta[row] = key_to_meta(m, bc);
    }
  } else {
    // a block is 2^lg vectors, at most one wavefront wide: butterfly over its lanes
    const uint32_t lg = args.block_groups_log2 + kVecsPerGroupLog2;
    const uint64_t Vall = (n + kPer - 1) / kPer;  // the last vector may be partial
    for (uint64_t base = (uint64_t)blockIdx.x * kBlock; base < Vall; base += (uint64_t)gridDim.x * kBlock) {
      const uint64_t i = base + threadIdx.x;
      int32_t m = (int32_t)0x80000000;
      if (i < V) {
        m = vector_exp_key<T>(__builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(src4) + i));
      } else if (i < Vall) {
        for (uint64_t e = i * kPer; e < n; ++e) m = max(m, element_exp_key<T>(src + e));
      }
      for (uint32_t d = 1; d < (1u << lg); d <<= 1) m = max(m, __shfl_xor(m, (int)d, 64));
      if (i < Vall && (threadIdx.x & ((1u << lg) - 1u)) == 0) meta[i >> lg] = key_to_meta(m, bc);
    }
  }
}

}  // namespace emu
}  // namespace exmy
