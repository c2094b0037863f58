// Fused decode: power-of-2 planes -> eXmY codes (Section 2.2.2, Fig. 2 read right
// to left) -> bf16 / fp32 values (Section 2.2.1 "and vice versa").
//
// Mirror image of the encoder: one lane owns whole groups of 8 elements, reads
// the group's word from every plane, and writes the 8 values with 16-byte
// stores (one for bf16, two adjacent ones for fp32).  The code itself is never
// assembled: each plane field is extracted and added straight into the fp32
// bit pattern at the position it has there.
#include "exmy_common.hpp"
#include "exmy_launch.hpp"

namespace exmy {

namespace {

constexpr int kBlock = 256;

// The words of one group in every plane: plane p uses w[p][0 .. S/4) (one dword
// when S <= 4).
template <int W>
struct GroupWords {
  uint32_t w[Planes<W>::count][4];
};

template <int W, int P = 0>
__device__ __forceinline__ void load_group(const uint8_t* __restrict__ src, uint64_t G, uint64_t g, GroupWords<W>& gw) {
  if constexpr (P < Planes<W>::count) {
    constexpr int S = Planes<W>::seg(P);
    const uint8_t* plane = src + G * (uint64_t)Planes<W>::lo(P);
    if constexpr (S == 16) {
      const uint4 o = reinterpret_cast<const uint4*>(plane)[g];
      gw.w[P][0] = o.x; gw.w[P][1] = o.y; gw.w[P][2] = o.z; gw.w[P][3] = o.w;
    } else if constexpr (S == 8) {
      const uint2 o = reinterpret_cast<const uint2*>(plane)[g];
      gw.w[P][0] = o.x; gw.w[P][1] = o.y;
    } else if constexpr (S == 4) {
      gw.w[P][0] = reinterpret_cast<const uint32_t*>(plane)[g];
    } else if constexpr (S == 2) {
      gw.w[P][0] = reinterpret_cast<const uint16_t*>(plane)[g];
    } else {
      gw.w[P][0] = plane[g];
    }
    load_group<W, P + 1>(src, G, g, gw);
  }
}

// Add the magnitude bits that plane P holds for element j into g, at the place
// they have in the fp32 pattern.  The top plane's most significant bit is the
// sign and is left out here.
template <int W, int P>
__device__ __forceinline__ uint32_t add_fields(const GroupWords<W>& gw, int j, uint32_t g, const FormatConsts& fc) {
  if constexpr (P < Planes<W>::count) {
    constexpr int S = Planes<W>::seg(P);
    constexpr int LO = Planes<W>::lo(P);
    constexpr bool top = P == Planes<W>::count - 1;
    constexpr int width = top ? S - 1 : S;
    if constexpr (width > 0) {
      const int bit = S * j;
      const uint32_t field = __builtin_amdgcn_ubfe(gw.w[P][bit / 32], bit % 32, width);
      g = lshl_add(field, fc.exp_shift + LO, g);
    }
    return add_fields<W, P + 1>(gw, j, g, fc);
  } else {
    return g;
  }
}

// fp32 bit pattern of element j of the group.
template <int W, bool kX8>
__device__ __forceinline__ uint32_t element_bits(const GroupWords<W>& gw, int j, const FormatConsts& fc) {
  uint32_t g = add_fields<W, 0>(gw, j, fc.dec_bias, fc);
  if constexpr (kX8) g = min(g, fc.g_clamp);  // exponent code 255 is not a value: largest finite instead
  const uint32_t mag = finish_magnitude(g, fc);
  constexpr int PT = Planes<W>::count - 1;
  constexpr int ST = Planes<W>::seg(PT);
  const int bit = ST * j + ST - 1;  // the sign: top bit of the top plane's field
  const uint32_t s = gw.w[PT][bit / 32] << (31 - bit % 32);
  return (s & 0x80000000u) | mag;
}

template <typename T, int W, bool kX8>
__device__ __forceinline__ void decode_group(const GroupWords<W>& gw, const FormatConsts& fc, uint4* __restrict__ dst4,
                                             uint64_t g) {
  uint32_t b[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) b[j] = element_bits<W, kX8>(gw, j, fc);
  if constexpr (sizeof(T) == 4) {
    dst4[2 * g] = make_uint4(b[0], b[1], b[2], b[3]);
    dst4[2 * g + 1] = make_uint4(b[4], b[5], b[6], b[7]);
  } else {
    // every value is exact in bf16: keep the upper halves
    uint4 o;
    o.x = __builtin_amdgcn_perm(b[1], b[0], 0x07060302u);
    o.y = __builtin_amdgcn_perm(b[3], b[2], 0x07060302u);
    o.z = __builtin_amdgcn_perm(b[5], b[4], 0x07060302u);
    o.w = __builtin_amdgcn_perm(b[7], b[6], 0x07060302u);
    dst4[g] = o;
  }
}

template <typename T, int W, int kUnroll, bool kX8>
__global__ __launch_bounds__(kBlock) void decode_kernel(const uint8_t* __restrict__ src, T* __restrict__ dst,
                                                         uint64_t n, FormatConsts fc) {
  const uint64_t G = (n + 7) / 8;
  const uint64_t Gfull = n / 8;
  uint4* __restrict__ dst4 = reinterpret_cast<uint4*>(dst);

  const uint64_t tile_groups = (uint64_t)kBlock * kUnroll;
  const uint64_t tiles = (Gfull + tile_groups - 1) / tile_groups;
  for (uint64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const uint64_t g0 = tile * tile_groups + threadIdx.x;
    const bool whole = (tile + 1) * tile_groups <= Gfull;  // block-uniform
    GroupWords<W> gw[kUnroll];
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      const uint64_t g = g0 + (uint64_t)r * kBlock;
      if (whole || g < Gfull) load_group<W>(src, G, g, gw[r]);
    }
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      const uint64_t g = g0 + (uint64_t)r * kBlock;
      if (whole || g < Gfull) decode_group<T, W, kX8>(gw[r], fc, dst4, g);
    }
  }

  // Ragged last group: one lane writes the n % 8 values one by one.
  if (Gfull != G && blockIdx.x == 0 && threadIdx.x == 0) {
    GroupWords<W> gw;
    load_group<W>(src, G, Gfull, gw);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint64_t i = Gfull * 8 + j;
      if (i < n) {
        const uint32_t b = element_bits<W, kX8>(gw, j, fc);
        if constexpr (sizeof(T) == 4)
          reinterpret_cast<uint32_t*>(dst)[i] = b;
        else
          reinterpret_cast<uint16_t*>(dst)[i] = (uint16_t)(b >> 16);
      }
    }
  }
}

template <typename T, int W>
hipError_t launch_decode(bool x8, const void* src, void* dst, uint64_t n, const FormatConsts& fc,
                         hipStream_t stream) {
  constexpr int kUnroll = sizeof(T) == 4 ? 2 : 4;
  const uint64_t tile_groups = (uint64_t)kBlock * kUnroll;
  const uint64_t tiles = (n / 8 + tile_groups - 1) / tile_groups;
  const uint32_t grid = grid_for_tiles(tiles, 16);
  if constexpr (W >= 9) {  // X = 8 needs at least 9 bits
    if (x8) {
      hipLaunchKernelGGL((decode_kernel<T, W, kUnroll, true>), dim3(grid), dim3(kBlock), 0, stream,
                         static_cast<const uint8_t*>(src), static_cast<T*>(dst), n, fc);
      return hipGetLastError();
    }
  }
  hipLaunchKernelGGL((decode_kernel<T, W, kUnroll, false>), dim3(grid), dim3(kBlock), 0, stream,
                     static_cast<const uint8_t*>(src), static_cast<T*>(dst), n, fc);
  return hipGetLastError();
}

template <typename T>
hipError_t dispatch_w(int W, bool x8, const void* src, void* dst, uint64_t n, const FormatConsts& fc,
                      hipStream_t stream) {
  switch (W) {
#define EXMY_CASE(w) \
  case w:            \
    return launch_decode<T, w>(x8, src, dst, n, fc, stream);
    EXMY_CASE(1) EXMY_CASE(2) EXMY_CASE(3) EXMY_CASE(4) EXMY_CASE(5) EXMY_CASE(6) EXMY_CASE(7) EXMY_CASE(8)
    EXMY_CASE(9) EXMY_CASE(10) EXMY_CASE(11) EXMY_CASE(12) EXMY_CASE(13) EXMY_CASE(14) EXMY_CASE(15) EXMY_CASE(16)
#undef EXMY_CASE
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t decode_dispatch(exmy_dtype_t dt, int W, bool x8, const void* src, void* dst, uint64_t n,
                           const FormatConsts& fc, hipStream_t stream) {
  if (dt == EXMY_F32) return dispatch_w<float>(W, x8, src, dst, n, fc, stream);
  return dispatch_w<uint16_t>(W, x8, src, dst, n, fc, stream);
}

}  // namespace exmy
