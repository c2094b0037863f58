// 256-bin histogram of the biased exponent field (Section 3.1, Fig. 3).
//
// Real tensors put most of their mass in about ten adjacent exponents, so a
// plain LDS histogram would serialise on a few addresses.  Each block keeps
// kCopies interleaved copies of the bins (copy = lane mod kCopies, address =
// bin * kCopies + copy): lanes of one LDS pass then hit different banks and,
// mostly, different addresses.  Blocks are resident and stride over the tiles,
// so the copies are folded into the caller's 64-bit global bins once per block.
#pragma once

#include "exmy_common.hpp"

namespace exmy {
namespace hist {

// 32-bit LDS bins are folded into the 64-bit global bins after this many tiles,
// long before 2^32 elements have been counted by one block.
constexpr uint32_t kTilesPerFlush = 1u << 15;

// Fold the block's LDS copies into the global 64-bit bins and clear them.
template <int kBlock, int kCopies>
__device__ __forceinline__ void flush_bins(uint32_t* bins, unsigned long long* __restrict__ hist) {
  __syncthreads();
  for (int bin = threadIdx.x; bin < 256; bin += kBlock) {
    uint32_t c = 0;
#pragma unroll
    for (int r = 0; r < kCopies; ++r) {
      // rotate the start so that the lanes of a pass read different banks
      const int rr = (r + threadIdx.x) & (kCopies - 1);
      c += bins[bin * kCopies + rr];
      bins[bin * kCopies + rr] = 0;
    }
    if (c) atomicAdd(&hist[bin], (unsigned long long)c);
  }
  __syncthreads();
}

// Count the exponents of the elements packed in one 16-byte vector.
template <typename T, int kCopies>
__device__ __forceinline__ void count_vector(uint4 v, uint32_t* bins, uint32_t copy) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    if constexpr (sizeof(T) == 4) {
      atomicAdd(&bins[__builtin_amdgcn_ubfe(w[k], 23, 8) * kCopies + copy], 1u);
    } else if constexpr (kIsF16<T>) {  // the exponent of the value as an fp32
      atomicAdd(&bins[__builtin_amdgcn_ubfe(lo_elem_bits<T>(w[k]), 23, 8) * kCopies + copy], 1u);
      atomicAdd(&bins[__builtin_amdgcn_ubfe(hi_elem_bits<T>(w[k]), 23, 8) * kCopies + copy], 1u);
    } else {
      atomicAdd(&bins[__builtin_amdgcn_ubfe(w[k], 7, 8) * kCopies + copy], 1u);
      atomicAdd(&bins[__builtin_amdgcn_ubfe(w[k], 23, 8) * kCopies + copy], 1u);
    }
  }
}

template <typename T, int kBlock, int kUnroll, int kCopies, bool kNT>
__global__ __launch_bounds__(kBlock) void histogram_kernel(const T* __restrict__ src, uint64_t n,
                                                            unsigned long long* __restrict__ hist) {
  constexpr int kPer = 16 / sizeof(T);
  constexpr uint32_t TV = kBlock * kUnroll;
  static_assert(TV * kPer >= 512, "tile counts must fit 32 bits for n <= 2^40");
  const uint64_t V = n / kPer;
  const uint32_t full_tiles = (uint32_t)(V / TV);
  const uint32_t rem = (uint32_t)(V - (uint64_t)full_tiles * TV);

  __shared__ uint32_t bins[256 * kCopies];
  for (int i = threadIdx.x; i < 256 * kCopies; i += kBlock) bins[i] = 0;
  __syncthreads();
  const uint32_t copy = threadIdx.x & (kCopies - 1);
  const uint32_t lane_off = threadIdx.x * 16;

  // Whole tiles: the loads of the block's next tile are in flight while it counts the current one.
  const uint4* __restrict__ src4 = reinterpret_cast<const uint4*>(src);
  uint32_t since_flush = 0;
  uint4 v[kUnroll], nxt[kUnroll];
  if (blockIdx.x < full_tiles) {
    const rsrc_t buf = make_rsrc(src4 + (uint64_t)blockIdx.x * TV);
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) nxt[r] = load16<kNT>(buf, lane_off, r * kBlock * 16);
  }
  for (uint32_t tile = blockIdx.x; tile < full_tiles; tile += gridDim.x) {
    if (++since_flush == kTilesPerFlush) {
      flush_bins<kBlock, kCopies>(bins, hist);
      since_flush = 0;
    }
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) v[r] = nxt[r];
    if (tile + gridDim.x < full_tiles) {
      const rsrc_t buf = make_rsrc(src4 + (uint64_t)(tile + gridDim.x) * TV);
#pragma unroll
      for (int r = 0; r < kUnroll; ++r) nxt[r] = load16<kNT>(buf, lane_off, r * kBlock * 16);
    }
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) count_vector<T, kCopies>(v[r], bins, copy);
  }
  // The partial last tile, taken by the block whose turn it would be.
  if (rem && blockIdx.x == full_tiles % gridDim.x) {
    const rsrc_t buf = make_rsrc(src4 + (uint64_t)full_tiles * TV);
#pragma unroll
    for (int r = 0; r < kUnroll; ++r)
      if (r * kBlock + threadIdx.x < rem) v[r] = load16<kNT>(buf, lane_off, r * kBlock * 16);
#pragma unroll
    for (int r = 0; r < kUnroll; ++r)
      if (r * kBlock + threadIdx.x < rem) count_vector<T, kCopies>(v[r], bins, copy);
  }

  // Elements past the last whole 16-byte vector.
  if (blockIdx.x == 0 && threadIdx.x < kPer) {
    const uint64_t i = V * kPer + threadIdx.x;
    if (i < n) {
      uint32_t e;
      if constexpr (sizeof(T) == 4)
        e = (reinterpret_cast<const uint32_t*>(src)[i] >> 23) & 0xFFu;
      else
        e = (elem_bits<T>(reinterpret_cast<const uint16_t*>(src)[i]) >> 23) & 0xFFu;
      atomicAdd(&bins[e * kCopies + copy], 1u);
    }
  }

  flush_bins<kBlock, kCopies>(bins, hist);
}

}  // namespace hist
}  // namespace exmy
