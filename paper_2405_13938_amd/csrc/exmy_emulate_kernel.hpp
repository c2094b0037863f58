// In-place emulation (Section 2.1): every element is replaced by the eXmY value
// nearest to it, kept in its own type; NaN and Inf are left untouched.
//
// One lane handles 16-byte vectors; a tile is kBlock * kUnroll vectors, one block
// per tile, launched in address order (see the encoder for why).
#pragma once

#include <type_traits>

#include "exmy_common.hpp"

namespace exmy {
namespace emu {

// fp32 bits of the eXmY value nearest to the magnitude with fp32 bits a0 (sign
// clear); anything above the largest value, Inf and NaN patterns included, gives
// the largest value.
//
// Same rounding as the encoder (magic addend with the ulp of the target
// quantum), but the rounded magnitude is recovered as a float by subtracting
// the addend again instead of being re-biased into a code.
template <bool kWide>
__device__ __forceinline__ uint32_t emulate_magnitude(uint32_t a0, const FormatConsts& fc, const TensorConsts& tc) {
  const uint32_t a = min(a0, tc.sat_bits);
  const uint32_t te = max(a, tc.emin_bits) & 0x7F800000u;
  if constexpr (!kWide) {
    // (a + m) - m with m = te * magic_scale, a power of two: the product is exact, so two fused operations give
    // the same two roundings
    const float s = __builtin_fmaf(as_f32(te), fc.magic_scale, as_f32(a));
    return as_u32(__builtin_fmaf(-as_f32(te), fc.magic_scale, s));
  } else {
    const uint32_t hi = ((te >> 23) + (uint32_t)fc.wide_exp) << 20;
    const double m = __hiloint2double((int)hi, 0);
    const double s = (double)as_f32(a) + m;
    return as_u32((float)(s - m));
  }
}

// fp32 bits of the emulated value of the element with fp32-position bits u.
template <bool kWide>
__device__ __forceinline__ uint32_t emulate_bits(uint32_t u, const FormatConsts& fc, const TensorConsts& tc) {
  const uint32_t a0 = u & 0x7FFFFFFFu;
  const uint32_t r = emulate_magnitude<kWide>(a0, fc, tc) | (u & 0x80000000u);
  return a0 >= 0x7F800000u ? u : r;  // Inf / NaN pass through
}

template <typename T, bool kWide>
__device__ __forceinline__ uint4 emulate_vector(uint4 v, const FormatConsts& fc, const TensorConsts& tc) {
  uint32_t w[4] = {v.x, v.y, v.z, v.w};
  if constexpr (sizeof(T) == 2 && !kIsF16<T>) {
    // bf16: the magnitudes of a pair are rounded, packed, and put under the pair's own sign bits by one bit
    // select.  Inf / NaN (which the rounding saturates) are rare: a maximum over the vector's magnitudes and one
    // ballot tell whether any lane of the wavefront holds one, and only then are the original halves put back.
    uint32_t out[4];
    uint32_t top = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint32_t lo = emulate_magnitude<kWide>((w[k] << 16) & 0x7FFFFFFFu, fc, tc);
      const uint32_t hi = emulate_magnitude<kWide>(w[k] & 0x7FFF0000u, fc, tc);
      out[k] = bit_select(0x7FFF7FFFu, pack_elems<T>(lo, hi), w[k]);
      top = max_pair_keys(top, w[k] & 0x7FFF7FFFu);  // non-negative halves: the signed maximum orders them
    }
    if (__builtin_amdgcn_ballot_w64(((top + 0x00800080u) & 0x80008000u) != 0) != 0) {  // a half with exponent 255
#pragma unroll
      for (int k = 0; k < 4; ++k) out[k] = keep_nonfinite_bf16(w[k], out[k]);
    }
    return make_uint4(out[0], out[1], out[2], out[3]);
  }
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    if constexpr (sizeof(T) == 4) {
      w[k] = emulate_bits<kWide>(w[k], fc, tc);
    } else {
      const uint32_t lo = emulate_bits<kWide>(lo_elem_bits<T>(w[k]), fc, tc);
      const uint32_t hi = emulate_bits<kWide>(hi_elem_bits<T>(w[k]), fc, tc);
      const uint32_t pair = pack_elems<T>(lo, hi);
      w[k] = kIsF16<T> ? keep_nonfinite_halves(w[k], pair) : pair;
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

  for (uint32_t tile = flat_tile(), once = 1; once && tile < tiles; once = 0) {
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
  if (flat_tile() == 0 && threadIdx.x < kPer) {
    const uint64_t i = V * kPer + threadIdx.x;
    if (i < n) {
      if constexpr (sizeof(T) == 4) {
        uint32_t* p = reinterpret_cast<uint32_t*>(data) + i;
        *p = emulate_bits<kWide>(*p, fc, tc);
      } else {
        uint16_t* p = reinterpret_cast<uint16_t*>(data) + i;
        const uint32_t u = elem_bits<T>(*p);
        if ((u & 0x7FFFFFFFu) < 0x7F800000u) *p = to_elem<T>(emulate_bits<kWide>(u, fc, tc));  // Inf / NaN stay as they are
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Per-block metadata: flat tiles with a per-lane metadata lookup, as in the
// encoder.  Work is counted in 16-byte vectors of kPer elements.

// try_uniform: look for a metadatum common to the wavefront first (not worth the ballot for the shortest blocks).
template <typename T>
__device__ __forceinline__ uint4 emulate_vector_meta(uint4 v, uint32_t me, bool wide_format, const FormatConsts& fc,
                                                     const BlockConsts& bc, bool try_uniform) {
  uint32_t first;
  if (try_uniform && wave_uniform(me, first)) {
    const TensorConsts tc = derive_tc(first, bc);
    if (wide_format || first > bc.wide_above) return emulate_vector<T, true>(v, fc, tc);
    return emulate_vector<T, false>(v, fc, tc);
  }
  const TensorConsts tc = derive_tc(me, bc);
  if (__builtin_amdgcn_ballot_w64(wide_format || me > bc.wide_above) != 0) return emulate_vector<T, true>(v, fc, tc);
  return emulate_vector<T, false>(v, fc, tc);
}

// Float scaling: every element becomes the value, in the max_exp = 127 format, nearest its real quotient
// by the block's scale (see scaled_sums), times the scale, rounded once into the container (see
// settle_scaled_product).  Inf / NaN pass through.  f64 and short_scale are wave-uniform.
template <typename T>
__device__ __forceinline__ uint4 emulate_vector_scaled(uint4 v, uint32_t scale_bits, bool f64, bool short_scale,
                                                       const FormatConsts& fc, const TensorConsts& tc127) {
  constexpr int E = 16 / sizeof(T);
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  uint32_t u[E];  // fp32-position bits
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    if constexpr (sizeof(T) == 4) {
      u[k] = w[k];
    } else {
      u[2 * k] = lo_elem_bits<T>(w[k]);
      u[2 * k + 1] = hi_elem_bits<T>(w[k]);
    }
  }
  const float scale = as_f32(scale_bits);
  float g[E];  // rounded magnitudes, before the scale is put back
  if (f64) {
    double scale64 = (double)scale;
    asm volatile("" : "+v"(scale64));  // pins the fp64 divisions inside this branch (the compiler would run them ahead of it)
#pragma unroll
    for (int j = 0; j < E; ++j) {
      uint32_t te;
      (void)scaled_sum_f64(u[j], scale64, fc, tc127, te, g[j]);
    }
  } else {
    const ScaleOfBlock sb = scale_of_block(scale_bits);
    const float s_mant = __builtin_amdgcn_frexp_mantf(scale);
    const int s_exp = __builtin_amdgcn_frexp_expf(scale);
    ScaledSums ss[E];
#pragma unroll
    for (int j = 0; j < E; ++j) ss[j] = scaled_sums(u[j], sb, fc, tc127);
#pragma unroll
    for (int j = 0; j < E; ++j)  // voted per element slot: see encode_group_scaled
      if (__builtin_amdgcn_ballot_w64(ss[j].lo != ss[j].hi) != 0) {
        asm volatile("");  // a real branch: the compiler would otherwise settle every slot and select
        ss[j].lo = settle_scaled_sum(u[j], ss[j], s_mant, s_exp, fc);
      }
#pragma unroll
    for (int j = 0; j < E; ++j) g[j] = as_f32(ss[j].lo) - as_f32(ss[j].te) * fc.magic_scale;  // exact
  }
  float p[E];
#pragma unroll
  for (int j = 0; j < E; ++j) p[j] = g[j] * scale;
  if constexpr (sizeof(T) == 2) {
    if (__builtin_amdgcn_ballot_w64(scaled_products_suspect<T, E>(p, short_scale)) != 0) {
      asm volatile("");  // a real branch
      const float s_mant = __builtin_amdgcn_frexp_mantf(scale);
      const int s_exp = __builtin_amdgcn_frexp_expf(scale);
#pragma unroll
      for (int j = 0; j < E; ++j) p[j] = settle_scaled_product(p[j], g[j], s_mant, s_exp, scaled_product_low_bits_clear<T>(p[j]));
    }
  }
  uint32_t out[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    if constexpr (sizeof(T) == 4) {
      out[k] = (u[k] & 0x7FFFFFFFu) >= 0x7F800000u ? u[k] : bit_select(0x7FFFFFFFu, as_u32(p[k]), u[k]);
    } else if constexpr (kIsF16<T>) {
      const uint32_t lo = bit_select(0x7FFFFFFFu, as_u32(p[2 * k]), u[2 * k]);
      const uint32_t hi = bit_select(0x7FFFFFFFu, as_u32(p[2 * k + 1]), u[2 * k + 1]);
      out[k] = keep_nonfinite_halves(w[k], pack_elems<T, false>(lo, hi));
    } else {  // bf16: both products rounded by one conversion, signs and Inf / NaN put back afterwards
      const uint32_t pair = bit_select(0x7FFF7FFFu, round_pack_bf16(p[2 * k], p[2 * k + 1]), w[k]);
      out[k] = keep_nonfinite_bf16(w[k], pair);
    }
  }
  return make_uint4(out[0], out[1], out[2], out[3]);
}

// One element on its own (after the last whole vector): fp32-position bits of its emulated value.
template <typename T>
__device__ __forceinline__ uint32_t emulate_scaled_bits(uint32_t u, uint32_t scale_bits, bool f64, const FormatConsts& fc,
                                                        const TensorConsts& tc127) {
  float g;
  uint32_t te;
  if (f64) {
    double scale64 = (double)as_f32(scale_bits);
    asm volatile("" : "+v"(scale64));  // as in emulate_vector_scaled
    (void)scaled_sum_f64(u, scale64, fc, tc127, te, g);
  } else {
    const uint32_t sum = scaled_sum_settled(u, scale_bits, fc, tc127, te);
    g = as_f32(sum) - as_f32(te) * fc.magic_scale;
  }
  const uint32_t r = scaled_product_bits<T>(as_u32(g) | (u & 0x80000000u), as_f32(scale_bits));
  return (u & 0x7FFFFFFFu) >= 0x7F800000u ? u : r;
}

// wide_format: the format itself needs the fp64 path (Y > 21), whatever the metadata.
// kScaled: per-block fp32 scales instead of per-block metadata bytes.
template <typename T, int kBlock, int kUnroll, bool kNT, bool kScaled>
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
  const bool try_uniform = bi.size >= 4;  // at most 16 blocks per wavefront

  for (uint32_t tile = flat_tile(), once = 1; once && tile < tiles; once = 0) {
    const uint64_t v0 = (uint64_t)tile * TV;
    uint64_t blk0;
    uint32_t off;
    tile_first_block(v0, bi, blk0, off);
    const rsrc_t buf = make_rsrc(reinterpret_cast<uint4*>(data) + v0);
    const rsrc_t mt = kScaled ? make_rsrc(scale_address(args, blk0)) : make_rsrc(meta + blk0);
    const uint64_t left = V - v0;
    const uint32_t rem = left < TV ? (uint32_t)left : TV;
    uint4 v[kUnroll];
    uint32_t me[kUnroll];
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      if (r * kBlock + threadIdx.x < rem) {
        v[r] = load16<kNT>(buf, lane_off, r * kBlock * 16);
        me[r] = load_block_datum<kScaled>(mt, lane_block<TV>(off + r * kBlock + threadIdx.x, bi), args.scale_log2_bytes);
      }
    }
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      if (r * kBlock + threadIdx.x < rem) {
        if constexpr (kScaled)
          store16<kNT>(buf, lane_off, r * kBlock * 16,
                       emulate_vector_scaled<T>(v[r], me[r], args.scaled_f64 != 0, args.scale_log2_bytes == 1, fc, args.tc127));
        else
          store16<kNT>(buf, lane_off, r * kBlock * 16, emulate_vector_meta<T>(v[r], me[r], wide_format, fc, bc, try_uniform));
      }
    }
  }

  // Elements past the last whole 16-byte vector belong to the last block.
  if (flat_tile() == 0 && threadIdx.x < kPer) {
    const uint64_t i = V * kPer + threadIdx.x;
    if (i < n) {
      uint32_t u;
      if constexpr (sizeof(T) == 4)
        u = reinterpret_cast<uint32_t*>(data)[i];
      else
        u = elem_bits<T>(reinterpret_cast<uint16_t*>(data)[i]);
      uint32_t r;
      if constexpr (kScaled) {
        r = emulate_scaled_bits<T>(u, load_scale_bits(args, args.n_blocks - 1), args.scaled_f64 != 0, fc, args.tc127);
      } else {
        const uint32_t me = meta[args.n_blocks - 1];
        const TensorConsts tc = derive_tc(me, bc);
        const bool wide = __builtin_amdgcn_ballot_w64(wide_format || me > bc.wide_above) != 0;
        r = wide ? emulate_bits<true>(u, fc, tc) : emulate_bits<false>(u, fc, tc);
      }
      if ((u & 0x7FFFFFFFu) < 0x7F800000u) {  // Inf / NaN stay as they are
        if constexpr (sizeof(T) == 4)
          reinterpret_cast<uint32_t*>(data)[i] = r;
        else
          reinterpret_cast<uint16_t*>(data)[i] = to_elem<T>(r);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Maximum exponent of every block, "before rounding" or "after rounding"
// (Section 2 "Metadata"): the biased exponent of the block's largest finite
// magnitude, taken as it is or after that value is rounded to the mantissa width
// of the format's top binade, clamped into the valid range (see exp_key and
// meta_from_key).

template <typename T, typename V4>
__device__ __forceinline__ int32_t vector_exp_key(V4 v) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  if constexpr (std::is_same<T, uint16_t>::value)  // bf16: two elements per instruction
    return key_of_pair(max_pair_keys(max_pair_keys(pair_keys(w[0]), pair_keys(w[1])),
                                     max_pair_keys(pair_keys(w[2]), pair_keys(w[3]))));
  int32_t m = (int32_t)0x80000000;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    if constexpr (sizeof(T) == 4) {
      m = max(m, exp_key(w[k]));
    } else {
      m = max(m, exp_key(lo_elem_bits<T>(w[k])));
      m = max(m, exp_key(hi_elem_bits<T>(w[k])));
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
    u = elem_bits<T>(*reinterpret_cast<const uint16_t*>(p));
  return exp_key(u);
}

// Result of one block from the key of its largest finite magnitude.  kScale:
// the scale that maps that magnitude onto the largest value of the
// max_exp = 127 format (not below the smallest normal float), as fp32 or as the
// smallest bf16 not below it (capped at the largest finite bf16); else the
// metadatum.
template <bool kScale>
__device__ __forceinline__ void store_block_result(const BlockArgs& args, uint64_t block, int32_t key) {
  uint32_t a = key > 0 ? (uint32_t)key - 0x00800000u : 0u;  // bits of the largest finite magnitude (0 if none)
  if constexpr (kScale) {
    const uint32_t s = as_u32(fmaxf(as_f32(a) / args.vmax127, as_f32(0x00800000u)));
    char* p = scale_address(args, block);
    if (args.scale_log2_bytes == 2)
      *reinterpret_cast<uint32_t*>(p) = s;
    else
      *reinterpret_cast<uint16_t*>(p) = (uint16_t)min((s + 0xFFFFu) >> 16, 0x7F7Fu);
  } else {
    args.meta[block] = (uint8_t)meta_from_key(key, args.bc);
  }
}

// Blocks of 2^lg vectors, lg <= 6: flat tiles of kBlock * kUnroll vectors, one
// vector per lane and step; the lanes of a block combine with a butterfly.
template <typename T, int kBlock, int kUnroll, bool kScale>
__global__ __launch_bounds__(kBlock) void block_max_exp_small_kernel(const BlockArgs args) {
  constexpr int kPer = 16 / sizeof(T);
  constexpr uint32_t TV = kBlock * kUnroll;
  const T* __restrict__ src = static_cast<const T*>(args.src);
  const uint4* __restrict__ src4 = static_cast<const uint4*>(args.src);
  const uint64_t n = args.n;
  const uint32_t lg = args.bi.log2;  // of vectors per block
  const uint64_t V = n / kPer;                  // whole vectors
  const uint64_t Vall = (n + kPer - 1) / kPer;  // the last one may be partial
  const uint32_t tiles = (uint32_t)((Vall + TV - 1) / TV);
  for (uint32_t tile = flat_tile(), once = 1; once && tile < tiles; once = 0) {
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
      if (i < Vall && (threadIdx.x & ((1u << lg) - 1u)) == 0) store_block_result<kScale>(args, i >> lg, mm);
    }
  }
}

// Any other block size: a team of kTeam lanes per block, kTeam = 64 (a wavefront;
// blocks of up to about a thousand vectors) or kTeam = kBlock (the workgroup).
template <typename T, int kBlock, int kTeam, bool kScale>
__global__ __launch_bounds__(kBlock) void block_max_exp_team_kernel(const BlockArgs args) {
  static_assert(kTeam == 64 || kTeam == kBlock, "a team is a wavefront or the workgroup");
  constexpr int kPer = 16 / sizeof(T);
  constexpr uint32_t kTeams = kBlock / kTeam;
  __shared__ int32_t part[kBlock / 64];
  const T* __restrict__ src = static_cast<const T*>(args.src);
  const uint4* __restrict__ src4 = static_cast<const uint4*>(args.src);
  const uint64_t n = args.n;
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
      if (lane == 0 && row < args.n_blocks) store_block_result<kScale>(args, row, m);
    } else {
      if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
      __syncthreads();
      if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kBlock / 64; ++w) m = max(m, part[w]);
        store_block_result<kScale>(args, row, m);
      }
      __syncthreads();  // part is reused by the next block
    }
  }
}

}  // namespace emu
}  // namespace exmy
