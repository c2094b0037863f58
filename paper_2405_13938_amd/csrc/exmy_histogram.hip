// 256-bin histogram of the biased exponent field (Section 3.1, Fig. 3).
//
// Real tensors put most of their mass in about ten adjacent exponents, so a
// plain LDS histogram would serialise on a few banks.  Each block keeps
// kCopies interleaved copies of the bins (copy = lane mod kCopies, address =
// bin * kCopies + copy, so neighbouring hot bins spread over all banks), and
// folds them into the caller's 64-bit global bins once at the end.
#include "exmy_common.hpp"
#include "exmy_launch.hpp"

namespace exmy {

namespace {

constexpr int kBlock = 256;
constexpr int kCopies = 8;
constexpr int kUnroll = 4;
constexpr uint32_t kTilesPerFlush = 1u << 16;  // x 8192 elements (bf16) per tile = 2^29 per block

// Fold the block's LDS copies into the global 64-bit bins and clear them.
__device__ __forceinline__ void flush_bins(uint32_t* bins, unsigned long long* __restrict__ hist) {
  __syncthreads();
  for (int bin = threadIdx.x; bin < 256; bin += kBlock) {
    uint32_t c = 0;
#pragma unroll
    for (int r = 0; r < kCopies; ++r) {
      c += bins[bin * kCopies + r];
      bins[bin * kCopies + r] = 0;
    }
    if (c) atomicAdd(&hist[bin], (unsigned long long)c);
  }
  __syncthreads();
}

template <typename T>
__global__ __launch_bounds__(kBlock) void histogram_kernel(const T* __restrict__ src, uint64_t n,
                                                            unsigned long long* __restrict__ hist) {
  constexpr int kPer = 16 / sizeof(T);
  const uint64_t V = n / kPer;
  const uint4* __restrict__ s4 = reinterpret_cast<const uint4*>(src);

  __shared__ uint32_t bins[256 * kCopies];
  for (int i = threadIdx.x; i < 256 * kCopies; i += kBlock) bins[i] = 0;
  __syncthreads();
  const uint32_t copy = threadIdx.x & (kCopies - 1);

  const uint64_t tile_vecs = (uint64_t)kBlock * kUnroll;
  const uint64_t tiles = (V + tile_vecs - 1) / tile_vecs;
  uint32_t since_flush = 0;
  for (uint64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    // 32-bit LDS bins: fold them long before 2^32 elements have been counted
    if (++since_flush == kTilesPerFlush) {
      flush_bins(bins, hist);
      since_flush = 0;
    }
    const uint64_t i0 = tile * tile_vecs + threadIdx.x;
    const bool whole = (tile + 1) * tile_vecs <= V;
    uint4 v[kUnroll];
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      const uint64_t i = i0 + (uint64_t)r * kBlock;
      if (whole || i < V) v[r] = s4[i];
    }
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      const uint64_t i = i0 + (uint64_t)r * kBlock;
      if (whole || i < V) {
        const uint32_t w[4] = {v[r].x, v[r].y, v[r].z, v[r].w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          if constexpr (sizeof(T) == 4) {
            atomicAdd(&bins[((w[k] >> 23) & 0xFFu) * kCopies + copy], 1u);
          } else {
            atomicAdd(&bins[((w[k] >> 7) & 0xFFu) * kCopies + copy], 1u);
            atomicAdd(&bins[((w[k] >> 23) & 0xFFu) * kCopies + copy], 1u);
          }
        }
      }
    }
  }

  if (blockIdx.x == 0 && threadIdx.x < kPer) {
    const uint64_t i = V * kPer + threadIdx.x;
    if (i < n) {
      uint32_t e;
      if constexpr (sizeof(T) == 4)
        e = (reinterpret_cast<const uint32_t*>(src)[i] >> 23) & 0xFFu;
      else
        e = (reinterpret_cast<const uint16_t*>(src)[i] >> 7) & 0xFFu;
      atomicAdd(&bins[e * kCopies + copy], 1u);
    }
  }

  flush_bins(bins, hist);
}

template <typename T>
hipError_t launch_histogram(const void* src, uint64_t n, uint64_t* hist, hipStream_t stream) {
  constexpr int kPer = 16 / sizeof(T);
  const uint64_t tile_vecs = (uint64_t)kBlock * kUnroll;
  const uint64_t tiles = (n / kPer + tile_vecs - 1) / tile_vecs;
  const uint32_t grid = grid_for_tiles(tiles, 8);
  hipLaunchKernelGGL((histogram_kernel<T>), dim3(grid), dim3(kBlock), 0, stream, static_cast<const T*>(src), n,
                     reinterpret_cast<unsigned long long*>(hist));
  return hipGetLastError();
}

}  // namespace

hipError_t histogram_dispatch(exmy_dtype_t dt, const void* src, uint64_t n, uint64_t* hist, hipStream_t stream) {
  if (dt == EXMY_F32) return launch_histogram<float>(src, n, hist, stream);
  return launch_histogram<uint16_t>(src, n, hist, stream);
}

}  // namespace exmy
