// Fused encode: float -> eXmY code (Section 2.2.1) -> power-of-2 planes
// (Section 2.2.2, Fig. 2), optionally with the exponent histogram of Section 3.1
// taken from the same registers.
//
// Work decomposition: one lane owns whole groups of 8 consecutive elements, so
// every plane word it produces is complete and byte aligned.  A bf16 group is
// one 16-byte load, an fp32 group two adjacent ones; lane i of a block takes
// group (tile base + i), so a wavefront reads one contiguous span per load
// instruction.  kUnroll groups per lane are loaded before any is converted, to
// keep enough bytes in flight to cover HBM latency.
#include "exmy_common.hpp"
#include "exmy_launch.hpp"

namespace exmy {

namespace {

constexpr int kBlock = 256;

// Histogram bins are replicated kHistCopies times in LDS, copy chosen by lane,
// so that the few hot exponents of a real tensor do not serialise on one bank.
constexpr int kHistCopies = 8;

constexpr uint32_t kTilesPerFlush = 1u << 16;  // x 8192 elements per tile = 2^29 per block

// Fold the block's LDS histogram copies into the global 64-bit bins and clear them.
__device__ __forceinline__ void flush_bins(uint32_t* bins, unsigned long long* __restrict__ hist) {
  __syncthreads();
  for (int bin = threadIdx.x; bin < 256; bin += kBlock) {
    uint32_t c = 0;
#pragma unroll
    for (int r = 0; r < kHistCopies; ++r) {
      c += bins[bin * kHistCopies + r];
      bins[bin * kHistCopies + r] = 0;
    }
    if (c) atomicAdd(&hist[bin], (unsigned long long)c);
  }
  __syncthreads();
}

template <typename T>
struct Elem;
template <>
struct Elem<float> {
  static constexpr int kLoads = 2;  // 16-byte loads per group of 8
};
template <>
struct Elem<uint16_t> {
  static constexpr int kLoads = 1;
};

// fp32-position bit patterns of the 8 elements of a group.
template <typename T>
__device__ __forceinline__ void group_bits(const uint4* v, uint32_t u[8]) {
  if constexpr (sizeof(T) == 4) {
    u[0] = v[0].x; u[1] = v[0].y; u[2] = v[0].z; u[3] = v[0].w;
    u[4] = v[1].x; u[5] = v[1].y; u[6] = v[1].z; u[7] = v[1].w;
  } else {
    const uint32_t w[4] = {v[0].x, v[0].y, v[0].z, v[0].w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      u[2 * i] = w[i] << 16;
      u[2 * i + 1] = w[i] & 0xFFFF0000u;
    }
  }
}

// (hi : lo) >> shift, low 32 bits: with shift = 32 - S this appends the top S bits
// of lo under hi << S in one instruction.
__device__ __forceinline__ uint32_t append_top(uint32_t hi, uint32_t lo, int S) {
  return __builtin_amdgcn_alignbit(hi, lo, 32 - S);
}

// Write plane P of group g: the S-bit fields that sit at the TOP of t[0..7],
// element j at bits [S*j, S*j + S) of the little-endian plane word (Fig. 2).
template <int S>
__device__ __forceinline__ void store_plane_from_top(const uint32_t t[8], uint8_t* plane, uint64_t g) {
  if constexpr (S == 16) {
    uint4 o;
    o.x = append_top(t[1] >> 16, t[0], 16);
    o.y = append_top(t[3] >> 16, t[2], 16);
    o.z = append_top(t[5] >> 16, t[4], 16);
    o.w = append_top(t[7] >> 16, t[6], 16);
    reinterpret_cast<uint4*>(plane)[g] = o;
  } else if constexpr (S == 8) {
    uint2 o;
    o.x = append_top(append_top(append_top(t[3] >> 24, t[2], 8), t[1], 8), t[0], 8);
    o.y = append_top(append_top(append_top(t[7] >> 24, t[6], 8), t[5], 8), t[4], 8);
    reinterpret_cast<uint2*>(plane)[g] = o;
  } else {
    uint32_t word = t[7] >> (32 - S);
#pragma unroll
    for (int j = 6; j >= 0; --j) word = append_top(word, t[j], S);
    if constexpr (S == 4) reinterpret_cast<uint32_t*>(plane)[g] = word;
    if constexpr (S == 2) reinterpret_cast<uint16_t*>(plane)[g] = (uint16_t)word;
    if constexpr (S == 1) plane[g] = (uint8_t)word;
  }
}

// Peel the planes off the left-aligned codes from the most significant segment
// down.  With an odd W the top plane is 1 bit wide and is exactly the sign: it is
// taken from the source bits u, and f holds the magnitude alone.
template <int W, int P>
__device__ __forceinline__ void peel_planes(uint32_t f[8], const uint32_t u[8], uint8_t* dst, uint64_t G, uint64_t g) {
  constexpr int S = Planes<W>::seg(P);
  constexpr int LO = Planes<W>::lo(P);
  constexpr bool sign_plane = (W & 1) && P == Planes<W>::count - 1;
  uint8_t* plane = dst + G * (uint64_t)LO;  // planes before P hold LO bits per element = LO bytes per group
  if constexpr (sign_plane) {
    store_plane_from_top<S>(u, plane, g);
  } else {
    store_plane_from_top<S>(f, plane, g);
    if constexpr (P > 0) {
#pragma unroll
      for (int j = 0; j < 8; ++j) f[j] <<= S;
    }
  }
  if constexpr (P > 0) peel_planes<W, P - 1>(f, u, dst, G, g);
}

// Convert the 8 elements of group g (fp32-position bits u) and write its planes.
template <int W, bool kWide>
__device__ __forceinline__ void encode_group(const uint32_t u[8], const FormatConsts& fc, uint8_t* dst, uint64_t G,
                                             uint64_t g) {
  uint32_t f[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const uint32_t m = magnitude_code_left<kWide>(u[j], fc);
    f[j] = (W & 1) ? m : ((u[j] & 0x80000000u) | m);  // even W: the sign rides at bit 31
  }
  peel_planes<W, Planes<W>::count - 1>(f, u, dst, G, g);
}

template <typename T, int W, int kUnroll, bool kWide, bool kHist>
__global__ __launch_bounds__(kBlock) void encode_kernel(const T* __restrict__ src, uint8_t* __restrict__ dst,
                                                         uint64_t n, FormatConsts fc,
                                                         unsigned long long* __restrict__ hist) {
  constexpr int kLoads = Elem<T>::kLoads;
  const uint64_t G = (n + 7) / 8;      // groups, the last one possibly ragged
  const uint64_t Gfull = n / 8;        // groups with all 8 elements present
  const uint4* __restrict__ src4 = reinterpret_cast<const uint4*>(src);

  __shared__ uint32_t lds_hist[kHist ? 256 * kHistCopies : 1];
  if constexpr (kHist) {
    for (int i = threadIdx.x; i < 256 * kHistCopies; i += kBlock) lds_hist[i] = 0;
    __syncthreads();
  }
  const uint32_t hist_copy = threadIdx.x & (kHistCopies - 1);

  const uint64_t tile_groups = (uint64_t)kBlock * kUnroll;
  const uint64_t tiles = (Gfull + tile_groups - 1) / tile_groups;
  uint32_t since_flush = 0;
  for (uint64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    if constexpr (kHist) {
      // 32-bit LDS bins: fold them long before 2^32 elements have been counted
      if (++since_flush == kTilesPerFlush) {
        flush_bins(lds_hist, hist);
        since_flush = 0;
      }
    }
    const uint64_t g0 = tile * tile_groups + threadIdx.x;
    const bool whole = (tile + 1) * tile_groups <= Gfull;  // block-uniform
    uint4 v[kUnroll][kLoads];
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      const uint64_t g = g0 + (uint64_t)r * kBlock;
      if (whole || g < Gfull) {
#pragma unroll
        for (int l = 0; l < kLoads; ++l) v[r][l] = src4[g * kLoads + l];
      }
    }
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      const uint64_t g = g0 + (uint64_t)r * kBlock;
      if (whole || g < Gfull) {
        uint32_t u[8];
        group_bits<T>(v[r], u);
        if constexpr (kHist) {
#pragma unroll
          for (int j = 0; j < 8; ++j) atomicAdd(&lds_hist[((u[j] >> 23) & 0xFFu) * kHistCopies + hist_copy], 1u);
        }
        encode_group<W, kWide>(u, fc, dst, G, g);
      }
    }
  }

  // Ragged last group: one lane reads the n % 8 elements one by one and pads
  // with zero codes.
  if (Gfull != G && blockIdx.x == 0 && threadIdx.x == 0) {
    uint32_t u[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint64_t i = Gfull * 8 + j;
      u[j] = 0;  // +0 encodes to code 0
      if (i < n) {
        if constexpr (sizeof(T) == 4)
          u[j] = reinterpret_cast<const uint32_t*>(src)[i];
        else
          u[j] = (uint32_t) reinterpret_cast<const uint16_t*>(src)[i] << 16;
        if constexpr (kHist) atomicAdd(&lds_hist[((u[j] >> 23) & 0xFFu) * kHistCopies + hist_copy], 1u);
      }
    }
    encode_group<W, kWide>(u, fc, dst, G, Gfull);
  }

  if constexpr (kHist) flush_bins(lds_hist, hist);
}

template <typename T, int W, bool kWide, bool kHist>
hipError_t launch_encode(const void* src, void* dst, uint64_t n, const FormatConsts& fc, uint64_t* hist,
                         hipStream_t stream) {
  constexpr int kUnroll = sizeof(T) == 4 ? 2 : 4;
  const uint64_t tile_groups = (uint64_t)kBlock * kUnroll;
  const uint64_t tiles = (n / 8 + tile_groups - 1) / tile_groups;
  const uint32_t grid = grid_for_tiles(tiles, kHist ? 4 : 16);
  hipLaunchKernelGGL((encode_kernel<T, W, kUnroll, kWide, kHist>), dim3(grid), dim3(kBlock), 0, stream,
                     static_cast<const T*>(src), static_cast<uint8_t*>(dst), n, fc,
                     reinterpret_cast<unsigned long long*>(hist));
  return hipGetLastError();
}

template <typename T, bool kWide, bool kHist>
hipError_t dispatch_w(int W, const void* src, void* dst, uint64_t n, const FormatConsts& fc, uint64_t* hist,
                      hipStream_t stream) {
  switch (W) {
#define EXMY_CASE(w) \
  case w:            \
    return launch_encode<T, w, kWide, kHist>(src, dst, n, fc, hist, stream);
    EXMY_CASE(1) EXMY_CASE(2) EXMY_CASE(3) EXMY_CASE(4) EXMY_CASE(5) EXMY_CASE(6) EXMY_CASE(7) EXMY_CASE(8)
    EXMY_CASE(9) EXMY_CASE(10) EXMY_CASE(11) EXMY_CASE(12) EXMY_CASE(13) EXMY_CASE(14) EXMY_CASE(15) EXMY_CASE(16)
#undef EXMY_CASE
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t encode_dispatch(exmy_dtype_t dt, int W, bool wide, bool with_hist, const void* src, void* dst,
                           uint64_t n, const FormatConsts& fc, uint64_t* hist, hipStream_t stream) {
  if (dt == EXMY_F32) {
    if (with_hist) return wide ? dispatch_w<float, true, true>(W, src, dst, n, fc, hist, stream)
                               : dispatch_w<float, false, true>(W, src, dst, n, fc, hist, stream);
    return wide ? dispatch_w<float, true, false>(W, src, dst, n, fc, hist, stream)
                : dispatch_w<float, false, false>(W, src, dst, n, fc, hist, stream);
  }
  if (with_hist) return wide ? dispatch_w<uint16_t, true, true>(W, src, dst, n, fc, hist, stream)
                             : dispatch_w<uint16_t, false, true>(W, src, dst, n, fc, hist, stream);
  return wide ? dispatch_w<uint16_t, true, false>(W, src, dst, n, fc, hist, stream)
              : dispatch_w<uint16_t, false, false>(W, src, dst, n, fc, hist, stream);
}

}  // namespace exmy
