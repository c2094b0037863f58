// In-place emulation (Section 2.1): every element is replaced by the eXmY value
// nearest to it, kept in its own type; NaN and Inf are left untouched.
#include "exmy_common.hpp"
#include "exmy_launch.hpp"

namespace exmy {

namespace {

constexpr int kBlock = 256;

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

template <typename T, int kUnroll, bool kWide>
__global__ __launch_bounds__(kBlock) void emulate_kernel(T* __restrict__ data, uint64_t n, FormatConsts fc,
                                                          TensorConsts tc) {
  constexpr int kPer = 16 / sizeof(T);  // elements per 16-byte vector
  const uint64_t V = n / kPer;          // whole vectors
  uint4* __restrict__ d4 = reinterpret_cast<uint4*>(data);

  const uint64_t tile_vecs = (uint64_t)kBlock * kUnroll;
  const uint64_t tiles = (V + tile_vecs - 1) / tile_vecs;
  for (uint64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const uint64_t i0 = tile * tile_vecs + threadIdx.x;
    const bool whole = (tile + 1) * tile_vecs <= V;
    uint4 v[kUnroll];
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      const uint64_t i = i0 + (uint64_t)r * kBlock;
      if (whole || i < V) v[r] = d4[i];
    }
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      const uint64_t i = i0 + (uint64_t)r * kBlock;
      if (whole || i < V) {
        uint32_t w[4] = {v[r].x, v[r].y, v[r].z, v[r].w};
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
        d4[i] = make_uint4(w[0], w[1], w[2], w[3]);
      }
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

template <typename T, bool kWide>
hipError_t launch_emulate(void* data, uint64_t n, const FormatConsts& fc, const TensorConsts& tc,
                          hipStream_t stream) {
  constexpr int kUnroll = 4;
  constexpr int kPer = 16 / sizeof(T);
  const uint64_t tile_vecs = (uint64_t)kBlock * kUnroll;
  const uint64_t tiles = (n / kPer + tile_vecs - 1) / tile_vecs;
  const uint32_t grid = grid_for_tiles(tiles, 16);
  hipLaunchKernelGGL((emulate_kernel<T, kUnroll, kWide>), dim3(grid), dim3(kBlock), 0, stream,
                     static_cast<T*>(data), n, fc, tc);
  return hipGetLastError();
}

}  // namespace

hipError_t emulate_dispatch(exmy_dtype_t dt, bool wide, void* data, uint64_t n, const FormatConsts& fc,
                            const TensorConsts& tc, hipStream_t stream) {
  if (dt == EXMY_F32)
    return wide ? launch_emulate<float, true>(data, n, fc, tc, stream)
                : launch_emulate<float, false>(data, n, fc, tc, stream);
  return wide ? launch_emulate<uint16_t, true>(data, n, fc, tc, stream)
              : launch_emulate<uint16_t, false>(data, n, fc, tc, stream);
}

}  // namespace exmy
