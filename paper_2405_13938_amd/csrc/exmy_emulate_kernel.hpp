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
// Per-block metadata: flat tiles with a per-lane metadata lookup, as in the
// encoder.  Work is counted in 16-byte vectors of kPer elements.

template <typename T>
__device__ __forceinline__ uint4 emulate_vector_meta(uint4 v, uint32_t me, bool wide_format, const FormatConsts& fc,
                                                     const BlockConsts& bc) {
  const TensorConsts tc = derive_tc(me, bc);
  if (__builtin_amdgcn_ballot_w64(wide_format || me > bc.wide_above) != 0) return emulate_vector<T, true>(v, fc, tc);
  return emulate_vector<T, false>(v, fc, tc);
}

// wide_format: the format itself needs the fp64 path (Y > 21), whatever the metadata.
template <typename T, int kBlock, int kUnroll, bool kNT>
__global__ __launch_bounds__(kBlock) void emulate_blocks_kernel(const BlockArgs args, bool wide_format) {
  constexpr int kPer = 16 / sizeof(T);
  constexpr uint32_t TV = kBlock * kUnroll;
  T* __restrict__ data = static_cast<T*>(const_cast<void*>(args.src));
  const uint8_t* __restrict__ meta = args.meta;
  const uint64_t n = args.n;
  const FormatConsts fc = args.fc;
  const BlockConsts bc = args.bc;
  const BlockIndex bi = args.bi;  // in vectors
  const uint64_t V = n / kPer;
  const uint32_t lane_off = threadIdx.x * 16;
  const uint32_t tiles = (uint32_t)((V + TV - 1) / TV);

  for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const uint64_t v0 = (uint64_t)tile * TV;
    uint64_t blk0;
    uint32_t off;
    tile_first_block(v0, bi, blk0, off);
    const rsrc_t buf = make_rsrc(reinterpret_cast<uint4*>(data) + v0);
    const rsrc_t mt = make_rsrc(meta + blk0);
    const uint64_t left = V - v0;
    const uint32_t rem = left < TV ? (uint32_t)left : TV;
    uint4 v[kUnroll];
    uint32_t me[kUnroll];
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      if (r * kBlock + threadIdx.x < rem) {
        v[r] = load16<kNT>(buf, lane_off, r * kBlock * 16);
        me[r] = __builtin_amdgcn_raw_buffer_load_b8(mt, lane_block<TV>(off + r * kBlock + threadIdx.x, bi), 0, 0);
      }
    }
#pragma unroll
    for (int r = 0; r < kUnroll; ++r)
      if (r * kBlock + threadIdx.x < rem)
        store16<kNT>(buf, lane_off, r * kBlock * 16, emulate_vector_meta<T>(v[r], me[r], wide_format, fc, bc));
  }

  // Elements past the last whole 16-byte vector belong to the last block.
  if (blockIdx.x == 0 && threadIdx.x < kPer) {
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
// Maximum exponent of every block, "before rounding" or "after rounding"
// (Section 2 "Metadata"): the biased exponent of the block's largest finite
// magnitude, taken as it is or after that value is rounded to the mantissa width
// of the format's top binade, clamped into the valid range.  Adding 1 to the exponent field turns Inf / NaN patterns negative
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
  uint32_t a = key > 0 ? (uint32_t)key - 0x00800000u : 0u;  // bits of the largest finite magnitude (0 if none)
  a += bc.round_half + ((a >> bc.round_shift) & bc.round_odd);  // "after rounding"; may carry up to exponent 255
  return (uint8_t)min(max(a >> 23, bc.meta_lo), bc.meta_hi);
}

// Maximum over the 2^lg lanes (lg <= 6) that share all lane-index bits above the
// low lg; every lane of the wavefront must call it.  Steps inside a row of 16
// lanes are data-parallel-primitive moves: after the two quad permutes every
// lane of a quad holds the quad's maximum, so mirroring 8 and then 16 lanes
// brings in exactly the other half each time.
__device__ __forceinline__ int32_t max_over_lanes(int32_t m, uint32_t lg) {
  if (lg >= 1) m = max(m, __builtin_amdgcn_update_dpp(m, m, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
  if (lg >= 2) m = max(m, __builtin_amdgcn_update_dpp(m, m, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
  if (lg >= 3) m = max(m, __builtin_amdgcn_update_dpp(m, m, 0x141, 0xF, 0xF, false));  // row_half_mirror
  if (lg >= 4) m = max(m, __builtin_amdgcn_update_dpp(m, m, 0x140, 0xF, 0xF, false));  // row_mirror
  if (lg >= 5) m = max(m, __shfl_xor(m, 16, 64));
  if (lg >= 6) m = max(m, __shfl_xor(m, 32, 64));
  return m;
}

// Blocks of 2^lg vectors, lg <= 6: flat tiles of kBlock * kUnroll vectors, one
// vector per lane and step; the lanes of a block combine with a butterfly.
template <typename T, int kBlock, int kUnroll>
__global__ __launch_bounds__(kBlock) void block_max_exp_small_kernel(const BlockArgs args) {
  constexpr int kPer = 16 / sizeof(T);
  constexpr uint32_t TV = kBlock * kUnroll;
  const T* __restrict__ src = static_cast<const T*>(args.src);
  const uint4* __restrict__ src4 = static_cast<const uint4*>(args.src);
  uint8_t* __restrict__ meta = args.meta;
  const uint64_t n = args.n;
  const BlockConsts bc = args.bc;
  const uint32_t lg = args.bi.log2;  // of vectors per block
  const uint64_t V = n / kPer;                  // whole vectors
  const uint64_t Vall = (n + kPer - 1) / kPer;  // the last one may be partial
  const uint32_t tiles = (uint32_t)((Vall + TV - 1) / TV);
  for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const uint64_t v0 = (uint64_t)tile * TV;
    const rsrc_t buf = make_rsrc(src4 + v0);
    const uint64_t whole = V - (v0 < V ? v0 : V);  // whole vectors from v0 on
    int32_t m[kUnroll];
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      const uint32_t i = r * kBlock + threadIdx.x;
      m[r] = (int32_t)0x80000000;
      if (i < whole) {
        m[r] = vector_exp_key<T>(load16<true>(buf, i * 16, 0));
      } else if (v0 + i < Vall) {
        for (uint64_t e = (v0 + i) * kPer; e < n; ++e) m[r] = max(m[r], element_exp_key<T>(src + e));
      }
    }
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      const uint64_t i = v0 + r * kBlock + threadIdx.x;
      const int32_t mm = max_over_lanes(m[r], lg);
      if (i < Vall && (threadIdx.x & ((1u << lg) - 1u)) == 0) meta[i >> lg] = key_to_meta(mm, bc);
    }
  }
}

// Any other block size: a team of kTeam lanes per block, kTeam = 64 (a wavefront;
// blocks of up to about a thousand vectors) or kTeam = kBlock (the workgroup).
template <typename T, int kBlock, int kTeam>
__global__ __launch_bounds__(kBlock) void block_max_exp_team_kernel(const BlockArgs args) {
  static_assert(kTeam == 64 || kTeam == kBlock, "a team is a wavefront or the workgroup");
  constexpr int kPer = 16 / sizeof(T);
  constexpr uint32_t kTeams = kBlock / kTeam;
  __shared__ int32_t part[kBlock / 64];
  const T* __restrict__ src = static_cast<const T*>(args.src);
  const uint4* __restrict__ src4 = static_cast<const uint4*>(args.src);
  uint8_t* __restrict__ meta = args.meta;
  const uint64_t n = args.n;
  const BlockConsts bc = args.bc;
  const uint64_t V = n / kPer;  // whole vectors
  const uint32_t block_vecs = args.bi.size;
  const uint32_t team = kTeams > 1 ? __builtin_amdgcn_readfirstlane(threadIdx.x >> 6) : 0;
  const uint32_t lane = threadIdx.x % kTeam;

  for (uint64_t first = (uint64_t)blockIdx.x * kTeams; first < args.n_blocks; first += (uint64_t)gridDim.x * kTeams) {
    const uint64_t row = first + team;  // uniform over the team
    int32_t m = (int32_t)0x80000000;
    if (row < args.n_blocks) {
      const uint64_t row_v0 = row * block_vecs;
      const uint64_t left = V - row_v0;
      const uint32_t row_vecs = left < block_vecs ? (uint32_t)left : block_vecs;
      const rsrc_t buf = make_rsrc(src4 + row_v0);
      uint32_t i = lane;
      for (; i + 3 * kTeam < row_vecs; i += 4 * kTeam) {  // four loads in flight per lane
        const uint4 a = load16<true>(buf, i * 16, 0);
        const uint4 b = load16<true>(buf, (i + kTeam) * 16, 0);
        const uint4 c = load16<true>(buf, (i + 2 * kTeam) * 16, 0);
        const uint4 d = load16<true>(buf, (i + 3 * kTeam) * 16, 0);
        m = max(max(m, vector_exp_key<T>(a)), vector_exp_key<T>(b));
        m = max(max(m, vector_exp_key<T>(c)), vector_exp_key<T>(d));
      }
      for (; i < row_vecs; i += kTeam) m = max(m, vector_exp_key<T>(load16<true>(buf, i * 16, 0)));
      if (row == args.n_blocks - 1 && lane < kPer) {  // elements past the last whole vector
        const uint64_t e = V * kPer + lane;
        if (e < n) m = max(m, element_exp_key<T>(src + e));
      }
    }
    m = max_over_lanes(m, 6);
    if constexpr (kTeam == 64) {
      if (lane == 0 && row < args.n_blocks) meta[row] = key_to_meta(m, bc);
    } else {
      if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
      __syncthreads();
      if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kBlock / 64; ++w) m = max(m, part[w]);
        meta[row] = key_to_meta(m, bc);
      }
      __syncthreads();  // part is reused by the next block
    }
  }
}

}  // namespace emu
}  // namespace exmy
