// Fused encode: float -> eXmY code (Section 2.2.1) -> power-of-2 planes
// (Section 2.2.2, Fig. 2), optionally with the exponent histogram of Section 3.1
// taken from the same registers.
//
// Work decomposition: one lane owns whole groups of 8 consecutive elements, so
// every plane word it produces is complete and byte aligned.  A bf16 group is
// one 16-byte load and lane i of a block takes group (tile base + i), so a
// wavefront reads one contiguous span per load instruction; an fp32 group is two
// 16-byte pieces, which whole tiles read as contiguous spans as well and then
// exchange between neighbouring lanes (see row_slot).  A tile is kBlock * kUnroll groups; a block walks kChunk
// consecutive tiles and issues the loads of the next tile before converting the
// current one, so that bytes stay in flight while the ALUs work.  Blocks are
// launched one per chunk, in address order: the hardware dispatcher then keeps
// the set of active blocks on a compact, moving window of memory, which
// measured faster here than a grid-stride loop of resident blocks.
#pragma once

#include <type_traits>

#include "exmy_common.hpp"

namespace exmy {
namespace enc {

// Histogram bins are replicated kHistCopies times in LDS, copy chosen by lane,
// so that the few hot exponents of a real tensor do not serialise on one bank.
constexpr int kHistCopies = 32;

// 32-bit LDS bins are folded into the 64-bit global bins after this many tiles,
// long before 2^32 elements have been counted by one block.
constexpr uint32_t kTilesPerFlush = 1u << 15;

// Fold the block's LDS histogram copies into the global 64-bit bins and clear them.
template <int kBlock>
__device__ __forceinline__ void flush_bins(uint32_t* bins, unsigned long long* __restrict__ hist) {
  __syncthreads();
  for (int bin = threadIdx.x; bin < 256; bin += kBlock) {
    uint32_t c = 0;
#pragma unroll
    for (int r = 0; r < kHistCopies; ++r) {
      // rotate the start so that the lanes of a pass read different banks
      const int rr = (r + threadIdx.x) & (kHistCopies - 1);
      c += bins[bin * kHistCopies + rr];
      bins[bin * kHistCopies + rr] = 0;
    }
    if (c) atomicAdd(&hist[bin], (unsigned long long)c);
  }
  __syncthreads();
}

// The group of a tile row of kBlock groups that a lane converts when the row is whole.
// 16-bit elements: its own.  fp32: a row is read as two runs of 16 bytes per lane, so
// that each load covers whole lines (a lane reading its group's 32 bytes makes two loads
// that each skip every other 16 bytes: the same bytes, 5-8 % slower).  The lanes of a
// pair (2k, 2k+1) then hold both halves of groups k and kBlock / 2 + k; the even lane
// takes the first, the odd lane the second (see group_bits).
template <typename T, int kBlock>
__device__ __forceinline__ uint32_t row_slot() {
  if constexpr (sizeof(T) == 4)
    return (threadIdx.x >> 1) + (threadIdx.x & 1u) * (kBlock / 2);
  else
    return threadIdx.x;
}

// The other lane of the pair's value (all lanes of the wavefront must be active).
__device__ __forceinline__ uint32_t from_pair_lane(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0xB1 /* quad_perm 1,0,3,2 */, 0xF, 0xF, false);
}

// fp32-position bit patterns of the 8 elements of a group held in 16-byte vectors.
// kPaired (fp32 only): v[0], v[1] are the lane's two pieces of a whole row as
// load_tile reads it, and the lanes of a pair swap one piece each.
template <typename T, bool kPaired = false>
__device__ __forceinline__ void group_bits(const uint4* v, uint32_t u[8]) {
  if constexpr (sizeof(T) == 4 && kPaired) {
    const bool odd = threadIdx.x & 1u;
    const uint4 give = odd ? v[0] : v[1];  // the piece of the group the other lane takes
    const uint4 got = make_uint4(from_pair_lane(give.x), from_pair_lane(give.y), from_pair_lane(give.z), from_pair_lane(give.w));
    const uint4 lo = odd ? got : v[0], hi = odd ? v[1] : got;
    u[0] = lo.x; u[1] = lo.y; u[2] = lo.z; u[3] = lo.w;
    u[4] = hi.x; u[5] = hi.y; u[6] = hi.z; u[7] = hi.w;
  } else if constexpr (sizeof(T) == 4) {
    u[0] = v[0].x; u[1] = v[0].y; u[2] = v[0].z; u[3] = v[0].w;
    u[4] = v[1].x; u[5] = v[1].y; u[6] = v[1].z; u[7] = v[1].w;
  } else {
    const uint32_t w[4] = {v[0].x, v[0].y, v[0].z, v[0].w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      u[2 * i] = lo_elem_bits<T>(w[i]);
      u[2 * i + 1] = hi_elem_bits<T>(w[i]);
    }
  }
}

// (hi : lo) >> shift, low 32 bits: with shift = 32 - S this appends the top S bits
// of lo under hi << S in one instruction.
__device__ __forceinline__ uint32_t append_top(uint32_t hi, uint32_t lo, int S) {
  return __builtin_amdgcn_alignbit(hi, lo, 32 - S);
}

// The destination of one chunk: a descriptor per plane, based at the plane word
// of the chunk's first group.
template <int W>
struct PlaneDst {
  rsrc_t plane[Planes<W>::count];
};

template <int W, int P = 0>
__device__ __forceinline__ void make_plane_dst(uint8_t* dst, uint64_t G, uint64_t g0, PlaneDst<W>& pd) {
  if constexpr (P < Planes<W>::count) {
    constexpr uint64_t S = Planes<W>::seg(P);
    constexpr uint64_t LO = Planes<W>::lo(P);  // planes before P hold LO bits per element = LO bytes per group
    pd.plane[P] = make_rsrc(dst + (G * LO + g0 * S));
    make_plane_dst<W, P + 1>(dst, G, g0, pd);
  }
}

// The S * 8 bits of one plane word from the S-bit fields that sit at the TOP of
// t[0..7], element j at bits [S*j, S*j + S) of the little-endian plane word (Fig. 2):
// out[0 .. S/4) for S >= 4, else the low 2 or 1 bytes of out[0].
template <int S>
__device__ __forceinline__ void plane_word_from_top(const uint32_t t[8], uint32_t out[4]) {
  if constexpr (S == 16) {
    out[0] = append_top(t[1] >> 16, t[0], 16);
    out[1] = append_top(t[3] >> 16, t[2], 16);
    out[2] = append_top(t[5] >> 16, t[4], 16);
    out[3] = append_top(t[7] >> 16, t[6], 16);
  } else if constexpr (S == 8) {
    out[0] = append_top(append_top(append_top(t[3] >> 24, t[2], 8), t[1], 8), t[0], 8);
    out[1] = append_top(append_top(append_top(t[7] >> 24, t[6], 8), t[5], 8), t[4], 8);
  } else {
    uint32_t word = t[7] >> (32 - S);
#pragma unroll
    for (int j = 6; j >= 0; --j) word = append_top(word, t[j], S);
    out[0] = word;
  }
}

// Where a lane's plane words go.  PlaneDst: straight to memory, one store of S bytes
// per plane and group (the word goes to byte lane_group * S + tile_group * S of the
// plane descriptor).  PlaneStage: into an LDS image of one tile of kTileGroups groups
// (plane P at byte kTileGroups * lo(P), the word of the tile's group i at i * S
// inside it), which flush_stage then writes out in 16-byte pieces: stores of 4, 2 or
// 1 bytes per lane reach memory as partial lines and measured 10-17 % slower.
template <int W, int kTileGroups>
struct PlaneStage {
  uint8_t* lds;  // kTileGroups * W bytes, 16-byte aligned
};

template <int W, int P>
__device__ __forceinline__ void put_plane_word(const PlaneDst<W>& pd, uint32_t lane_group, uint32_t tile_group,
                                               const uint32_t w[4]) {
  constexpr int S = Planes<W>::seg(P);
  const rsrc_t plane = pd.plane[P];
  const uint32_t voff = lane_group * S, soff = tile_group * S;
  if constexpr (S == 16) store16<false>(plane, voff, soff, make_uint4(w[0], w[1], w[2], w[3]));
  if constexpr (S == 8) {
    const u32x2_t o = {w[0], w[1]};
    __builtin_amdgcn_raw_buffer_store_b64(o, plane, voff, soff, 0);
  }
  if constexpr (S == 4) __builtin_amdgcn_raw_buffer_store_b32(w[0], plane, voff, soff, 0);
  if constexpr (S == 2) __builtin_amdgcn_raw_buffer_store_b16((uint16_t)w[0], plane, voff, soff, 0);
  if constexpr (S == 1) __builtin_amdgcn_raw_buffer_store_b8((uint8_t)w[0], plane, voff, soff, 0);
}

template <int W, int P, int kTileGroups>
__device__ __forceinline__ void put_plane_word(const PlaneStage<W, kTileGroups>& st, uint32_t lane_group,
                                               uint32_t tile_group, const uint32_t w[4]) {
  constexpr int S = Planes<W>::seg(P);
  constexpr int LO = Planes<W>::lo(P);  // as a constant: the call itself would run its loop on the scalar unit
  uint8_t* p = st.lds + kTileGroups * LO + (lane_group + tile_group) * S;
  if constexpr (S == 16) *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
  if constexpr (S == 8) *reinterpret_cast<uint2*>(p) = make_uint2(w[0], w[1]);
  if constexpr (S == 4) *reinterpret_cast<uint32_t*>(p) = w[0];
  if constexpr (S == 2) *reinterpret_cast<uint16_t*>(p) = (uint16_t)w[0];
  if constexpr (S == 1) *p = (uint8_t)w[0];
}

// Write the image of the whole tile that starts at group g0 to the planes of dst: the
// copy alone (the caller places the barriers), and with a barrier on either side.
// Every lane of the workgroup calls them.
template <int W, int kTileGroups, int kBlock>
__device__ __forceinline__ void copy_stage(const PlaneStage<W, kTileGroups>& st, uint8_t* dst, uint64_t G, uint64_t g0) {
  constexpr uint32_t kPieces = kTileGroups * W / 16;
#pragma unroll
  for (uint32_t c0 = 0; c0 < kPieces; c0 += kBlock) {
    const uint32_t c = c0 + threadIdx.x;
    if (kPieces % kBlock == 0 || c < kPieces) {
      const uint4 v = *reinterpret_cast<const uint4*>(st.lds + c * 16);
      const u32x4_t w = {v.x, v.y, v.z, v.w};
      __builtin_nontemporal_store(w, reinterpret_cast<plane_piece_t*>(tile_piece_address<W, kTileGroups>(dst, G, g0, c * 16)));
    }
  }
}

template <int W, int kTileGroups, int kBlock>
__device__ __forceinline__ void flush_stage(const PlaneStage<W, kTileGroups>& st, uint8_t* dst, uint64_t G, uint64_t g0) {
  __syncthreads();  // every lane has put its words
  copy_stage<W, kTileGroups, kBlock>(st, dst, G, g0);
  __syncthreads();  // the image is free for the next tile
}

// The same for the first `count` groups of an image, through plane descriptors whose base lies `tile_group`
// groups before the image's first group: every plane's part in 16-byte pieces, and the up to 15 bytes that
// remain of it when count is not a multiple of 16 as single bytes.
template <int W, int kTileGroups, int kBlock, int P = 0>
__device__ __forceinline__ void copy_stage_groups(const PlaneStage<W, kTileGroups>& st, const PlaneDst<W>& pd,
                                                  uint32_t tile_group, uint32_t count) {
  if constexpr (P < Planes<W>::count) {
    constexpr uint32_t S = Planes<W>::seg(P);
    constexpr uint32_t LO = Planes<W>::lo(P);
    const uint32_t bytes = count * S;
    const uint32_t pieces = bytes / 16;
    for (uint32_t c = threadIdx.x; c < pieces; c += kBlock)
      store16<true>(pd.plane[P], c * 16, tile_group * S, *reinterpret_cast<const uint4*>(st.lds + kTileGroups * LO + c * 16));
    if constexpr (S < 16) {
      const uint32_t at = pieces * 16 + threadIdx.x;
      if (at < bytes) __builtin_amdgcn_raw_buffer_store_b8(st.lds[kTileGroups * LO + at], pd.plane[P], at, tile_group * S, 0);
    }
    copy_stage_groups<W, kTileGroups, kBlock, P + 1>(st, pd, tile_group, count);
  }
}

template <int W, int kTileGroups, int kBlock>
__device__ __forceinline__ void flush_stage_groups(const PlaneStage<W, kTileGroups>& st, const PlaneDst<W>& pd,
                                                   uint32_t tile_group, uint32_t count) {
  __syncthreads();
  copy_stage_groups<W, kTileGroups, kBlock>(st, pd, tile_group, count);
  __syncthreads();
}

// Peel the planes off the left-aligned codes from the most significant segment
// down.  With an odd W the top plane is 1 bit wide and is exactly the sign: it is
// taken from the source bits u, and f holds the magnitude alone.
// `lane_group` is the lane's group within the tile, `tile_group` the tile's first
// group relative to the destination's base (wave-uniform).
template <int W, int P, class Dst>
__device__ __forceinline__ void peel_planes(uint32_t f[8], const uint32_t u[8], const Dst& dst, uint32_t lane_group,
                                            uint32_t tile_group) {
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
  put_plane_word<W, P>(dst, lane_group, tile_group, word);
  if constexpr (P > 0) peel_planes<W, P - 1>(f, u, dst, lane_group, tile_group);
}

// Convert the 8 elements of one group (fp32-position bits u) and write its planes.
template <int W, bool kWide, class Dst>
__device__ __forceinline__ void encode_group(const uint32_t u[8], const FormatConsts& fc, const TensorConsts& tc,
                                             const Dst& pd, uint32_t lane_group, uint32_t tile_group) {
  uint32_t f[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const uint32_t m = magnitude_code_left<kWide>(u[j], fc, tc);
    f[j] = (W & 1) ? m : ((u[j] & 0x80000000u) | m);  // even W: the sign rides at bit 31
  }
  peel_planes<W, Planes<W>::count - 1>(f, u, pd, lane_group, tile_group);
}

template <typename T, int kUnroll>
struct TileRegs {
  static constexpr int kLoads = sizeof(T) == 4 ? 2 : 1;  // 16-byte loads per group of 8
  uint4 v[kUnroll][kLoads];
};

// Loads of one tile: `src` is the descriptor of the chunk, tile_group the tile's
// first group relative to it (wave-uniform).
// kGuard: only the first `rem` groups of the tile exist.  kPairs (whole tiles only):
// lane i ends up with groups r*kBlock + row_slot(), for fp32 through
// group_bits<T, true>; otherwise it loads groups r*kBlock + i.
template <typename T, int kBlock, int kUnroll, bool kNT, bool kGuard, bool kPairs = !kGuard>
__device__ __forceinline__ void load_tile(rsrc_t src, uint32_t tile_group, uint32_t rem, TileRegs<T, kUnroll>& regs) {
  static_assert(!(kGuard && kPairs), "lanes of a pair must both be active");
  constexpr int kLoads = TileRegs<T, kUnroll>::kLoads;
  constexpr uint32_t kGroupBytes = 16 * kLoads;
  constexpr bool kRuns = sizeof(T) == 4 && kPairs;  // pieces i and kBlock + i of the row instead of 2i and 2i + 1
  const uint32_t lane_off = threadIdx.x * (kRuns ? 16 : kGroupBytes);
#pragma unroll
  for (int r = 0; r < kUnroll; ++r) {
    if (!kGuard || r * kBlock + threadIdx.x < rem) {
#pragma unroll
      for (int l = 0; l < kLoads; ++l)
        regs.v[r][l] = load16<kNT>(src, lane_off, (tile_group + r * kBlock) * kGroupBytes + l * (kRuns ? 16 * kBlock : 16));
    }
  }
}

// Convert and store one tile.
template <typename T, int W, int kBlock, int kUnroll, bool kWide, bool kHist, bool kGuard, class Dst>
__device__ __forceinline__ void encode_tile(const TileRegs<T, kUnroll>& regs, const Dst& pd,
                                            uint32_t tile_group, uint32_t rem, const FormatConsts& fc,
                                            const TensorConsts& tc, uint32_t* lds_hist) {
#pragma unroll
  for (int r = 0; r < kUnroll; ++r) {
    if (!kGuard || r * kBlock + threadIdx.x < rem) {
      uint32_t u[8];
      group_bits<T, !kGuard>(regs.v[r], u);
      if constexpr (kHist) {
        const uint32_t copy = threadIdx.x & (kHistCopies - 1);
#pragma unroll
        for (int j = 0; j < 8; ++j) atomicAdd(&lds_hist[((u[j] >> 23) & 0xFFu) * kHistCopies + copy], 1u);
      }
      encode_group<W, kWide>(u, fc, tc, pd, kGuard ? threadIdx.x : row_slot<T, kBlock>(), tile_group + r * kBlock);
    }
  }
}

// The group's 8 elements in fp32 position: a 16-byte group from registers, or, for
// the ragged last group of the tensor, its elements one by one (zeros beyond n).
template <typename T>
__device__ __forceinline__ void ragged_group_bits(const void* src_v, uint64_t first, uint64_t n, uint32_t u[8]) {
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const uint64_t i = first + j;
    u[j] = 0;
    if (i < n) {
      if constexpr (sizeof(T) == 4)
        u[j] = static_cast<const uint32_t*>(src_v)[i];
      else
        u[j] = elem_bits<T>(static_cast<const uint16_t*>(src_v)[i]);
    }
  }
}

// Grid: x = one block per chunk of kChunk tiles of the largest tensor (any
// smaller x also works: blocks then stride over the chunks), y = tensor of the
// batch.  Blocks past the end of a smaller tensor find nothing to do.
//
// A chunk made of whole tiles takes the straight-line path: the loads of tile
// c + 1 are issued before tile c is converted, with no bounds checks and only
// wave-uniform address arithmetic.  The chunk that holds the end of the tensor
// takes a guarded loop.
template <typename T, int W, int kBlock, int kUnroll, int kChunk, bool kWide, bool kHist, bool kNT>
__global__ __launch_bounds__(kBlock) void encode_kernel(const BatchArgs batch) {
  constexpr uint32_t TG = kBlock * kUnroll;
  constexpr int kLoads = TileRegs<T, kUnroll>::kLoads;
  static_assert(TG >= 64, "tile counts must fit 32 bits for n <= 2^40");
  const TensorArgs& ta = batch.t[blockIdx.y];
  const uint4* __restrict__ src4 = static_cast<const uint4*>(ta.src);
  uint8_t* __restrict__ dst = static_cast<uint8_t*>(ta.dst);
  const uint64_t n = ta.n;
  const FormatConsts fc = batch.fc;
  const TensorConsts tc = ta.tc;
  unsigned long long* __restrict__ hist = batch.hist;
  const uint64_t G = (n + 7) / 8;  // groups, the last one possibly ragged
  const uint64_t Gfull = n / 8;    // groups with all 8 elements present
  const uint32_t full_tiles = (uint32_t)(Gfull / TG);
  const uint32_t rem_groups = (uint32_t)(Gfull - (uint64_t)full_tiles * TG);  // groups of the partial tile
  const uint32_t tiles = full_tiles + (rem_groups ? 1u : 0u);
  const uint32_t full_chunks = full_tiles / kChunk;
  const uint32_t chunks = (tiles + kChunk - 1) / kChunk;

  __shared__ uint32_t lds_hist[kHist ? 256 * kHistCopies : 1];
  __shared__ __align__(16) uint8_t lds_stage[TG * W];
  const PlaneStage<W, TG> stage{lds_stage};
  if constexpr (kHist) {
    for (int i = threadIdx.x; i < 256 * kHistCopies; i += kBlock) lds_hist[i] = 0;
    __syncthreads();
  }

  uint32_t since_flush = 0;
  for (uint32_t chunk = blockIdx.x; chunk < chunks; chunk += gridDim.x) {
    const uint64_t g0 = (uint64_t)chunk * (kChunk * TG);  // first group of the chunk
    const rsrc_t src = make_rsrc(src4 + g0 * kLoads);
    PlaneDst<W> pd;
    make_plane_dst<W>(dst, G, g0, pd);
    if (chunk < full_chunks) {
      TileRegs<T, kUnroll> regs[2];
      load_tile<T, kBlock, kUnroll, kNT, false>(src, 0, 0, regs[0]);
#pragma unroll
      for (int c = 0; c < kChunk; ++c) {
        if (c + 1 < kChunk) load_tile<T, kBlock, kUnroll, kNT, false>(src, (c + 1) * TG, 0, regs[(c + 1) & 1]);
        encode_tile<T, W, kBlock, kUnroll, kWide, kHist, false>(regs[c & 1], stage, 0, 0, fc, tc, lds_hist);
        flush_stage<W, TG, kBlock>(stage, dst, G, g0 + (uint64_t)c * TG);
      }
    } else {
      for (uint32_t tile = chunk * kChunk; tile < tiles; ++tile) {
        const uint32_t tile_group = (tile - chunk * kChunk) * TG;
        const uint32_t rem = tile < full_tiles ? TG : rem_groups;
        TileRegs<T, kUnroll> regs;
        load_tile<T, kBlock, kUnroll, kNT, true>(src, tile_group, rem, regs);
        encode_tile<T, W, kBlock, kUnroll, kWide, kHist, true>(regs, pd, tile_group, rem, fc, tc, lds_hist);
      }
    }
    if constexpr (kHist) {
      since_flush += kChunk;
      if (since_flush >= kTilesPerFlush) {
        flush_bins<kBlock>(lds_hist, hist);
        since_flush = 0;
      }
    }
  }

  // Ragged last group: one lane reads the n % 8 elements one by one and pads
  // with +0, which encodes to code 0.
  if (Gfull != G && blockIdx.x == 0 && threadIdx.x == 0) {
    const T* __restrict__ src = static_cast<const T*>(ta.src);
    uint32_t u[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint64_t i = Gfull * 8 + j;
      u[j] = 0;
      if (i < n) {
        if constexpr (sizeof(T) == 4)
          u[j] = reinterpret_cast<const uint32_t*>(src)[i];
        else
          u[j] = elem_bits<T>(reinterpret_cast<const uint16_t*>(src)[i]);
        if constexpr (kHist) atomicAdd(&lds_hist[((u[j] >> 23) & 0xFFu) * kHistCopies], 1u);
      }
    }
    PlaneDst<W> pd;
    make_plane_dst<W>(dst, G, Gfull, pd);
    encode_group<W, kWide>(u, fc, tc, pd, 0, 0);
  }

  if constexpr (kHist) flush_bins<kBlock>(lds_hist, hist);
}

// The same conversion with one tile per workgroup and no loop: grid x (and z, for tensors of more than
// gridDim.x tiles) = tile, y = tensor of the batch.  This is the form the plain encoder is launched in: a
// kernel whose chunk loop runs once still carries the loop's bookkeeping (register copies for the values
// the loop would carry, address set-up outside it), 10 % of this kernel's vector instructions, and the
// bf16 encoder at 7 bits is within reach of the vector ALU limit (+2-3 % throughput without them).
// Workgroups past a tensor's last tile find nothing to do; the workgroup of the tile after the last whole
// one takes the partial tile and the ragged last group.
template <typename T, int W, int kBlock, int kUnroll, bool kWide, bool kNT>
__global__ __launch_bounds__(kBlock) void encode_flat_kernel(const BatchArgs batch) {
  constexpr uint32_t TG = kBlock * kUnroll;
  constexpr int kLoads = TileRegs<T, kUnroll>::kLoads;
  static_assert(TG >= 64, "tile counts must fit 32 bits for n <= 2^40");
  const TensorArgs& ta = batch.t[blockIdx.y];
  const uint4* __restrict__ src4 = static_cast<const uint4*>(ta.src);
  uint8_t* __restrict__ dst = static_cast<uint8_t*>(ta.dst);
  const uint64_t n = ta.n;
  const FormatConsts fc = batch.fc;
  const TensorConsts tc = ta.tc;
  const uint64_t G = (n + 7) / 8;  // groups, the last one possibly ragged
  const uint64_t Gfull = n / 8;    // groups with all 8 elements present
  const uint32_t full_tiles = (uint32_t)(Gfull / TG);
  const uint32_t tile = blockIdx.z * gridDim.x + blockIdx.x;
  const uint64_t g0 = (uint64_t)tile * TG;
  const rsrc_t src = make_rsrc(src4 + g0 * kLoads);
  __shared__ __align__(16) uint8_t lds_stage[TG * W];
  const PlaneStage<W, TG> stage{lds_stage};

  if (tile < full_tiles) {
    TileRegs<T, kUnroll> regs;
    load_tile<T, kBlock, kUnroll, kNT, false>(src, 0, 0, regs);
    encode_tile<T, W, kBlock, kUnroll, kWide, false, false>(regs, stage, 0, 0, fc, tc, nullptr);
    __syncthreads();  // every lane has put its words
    copy_stage<W, TG, kBlock>(stage, dst, G, g0);
    return;
  }
  if (tile > full_tiles) return;

  const uint32_t rem_groups = (uint32_t)(Gfull - (uint64_t)full_tiles * TG);  // groups of the partial tile
  if (rem_groups) {
    PlaneDst<W> pd;
    make_plane_dst<W>(dst, G, g0, pd);
    TileRegs<T, kUnroll> regs;
    load_tile<T, kBlock, kUnroll, kNT, true>(src, 0, rem_groups, regs);
    encode_tile<T, W, kBlock, kUnroll, kWide, false, true>(regs, pd, 0, rem_groups, fc, tc, nullptr);
  }
  // Ragged last group: one lane reads the n % 8 elements one by one and pads with +0, which encodes to code 0.
  if (Gfull != G && threadIdx.x == 0) {
    uint32_t u[8];
    ragged_group_bits<T>(ta.src, Gfull * 8, n, u);
    PlaneDst<W> pd;
    make_plane_dst<W>(dst, G, Gfull, pd);
    encode_group<W, kWide>(u, fc, tc, pd, 0, 0);
  }
}

// ---------------------------------------------------------------------------
// Per-block metadata (Section 2 "Metadata", "Block Size"; Section 2.2.1).
//
// Tiles run flat over the tensor exactly as in the per-tensor kernel, whatever the
// block size: every lane looks up the metadatum of the block its own group lies
// in (see BlockIndex) and derives the block's constants in registers.

// One group with the rounding variant its block's metadatum needs.  The branch is
// taken for a whole wavefront at once (any lane that needs the fp64 path sends
// all of them there; both paths give the same result where both apply).
// try_uniform: look first for a metadatum common to the wavefront (see wave_uniform).
template <int W, class Dst>
__device__ __forceinline__ void encode_group_meta(const uint32_t u[8], uint32_t me, const FormatConsts& fc,
                                                  const BlockConsts& bc, const Dst& pd, uint32_t lane_group,
                                                  uint32_t tile_group, bool try_uniform = true) {
  uint32_t first;
  if (try_uniform && wave_uniform(me, first)) {
    const TensorConsts tc = derive_tc(first, bc);
    if (first > bc.wide_above)
      encode_group<W, true>(u, fc, tc, pd, lane_group, tile_group);
    else
      encode_group<W, false>(u, fc, tc, pd, lane_group, tile_group);
    return;
  }
  const TensorConsts tc = derive_tc(me, bc);
  if (__builtin_amdgcn_ballot_w64(me > bc.wide_above) != 0)
    encode_group<W, true>(u, fc, tc, pd, lane_group, tile_group);
  else
    encode_group<W, false>(u, fc, tc, pd, lane_group, tile_group);
}

// Float scaling: the group's elements take the codes, in the max_exp = 127 format, of their real
// quotients by the block's scale (see scaled_sums).  f64 and vote are wave-uniform; vote = false (a lane on
// its own) settles every element without asking the wavefront.
template <int W, class Dst>
__device__ __forceinline__ void encode_group_scaled(const uint32_t u[8], uint32_t scale_bits, bool f64,
                                                    const FormatConsts& fc, const TensorConsts& tc127, const Dst& pd,
                                                    uint32_t lane_group, uint32_t tile_group, bool vote = true) {
  uint32_t f[8];
  if (f64) {
    double scale64 = (double)as_f32(scale_bits);
    asm volatile("" : "+v"(scale64));  // pins the fp64 divisions inside this branch (the compiler would run them ahead of it)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      uint32_t te;
      float value;
      const uint32_t k = scaled_sum_f64(u[j], scale64, fc, tc127, te, value);
      f[j] = code_left_of_sum(k, te, fc, tc127);
    }
  } else {
    const ScaleOfBlock sb = scale_of_block(scale_bits);
    const float s_mant = __builtin_amdgcn_frexp_mantf(sb.scale);
    const int s_exp = __builtin_amdgcn_frexp_expf(sb.scale);
    ScaledSums ss[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) ss[j] = scaled_sums(u[j], sb, fc, tc127);
    // data of few significant bits (bf16 elements under a scale derived from one of them) puts a few elements
    // per thousand on or next to a boundary: the vote is taken per element slot, so that a wavefront settles
    // the slots that hold one (about one in four) and not all eight
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (!vote || __builtin_amdgcn_ballot_w64(ss[j].lo != ss[j].hi) != 0) {
        asm volatile("");  // a real branch: the compiler would otherwise settle every slot and select
        ss[j].lo = settle_scaled_sum(u[j], ss[j], s_mant, s_exp, fc);
      }
#pragma unroll
    for (int j = 0; j < 8; ++j) f[j] = code_left_of_sum(ss[j].lo, ss[j].te, fc, tc127);
  }
  if constexpr (!(W & 1)) {  // even W: the sign rides at bit 31
#pragma unroll
    for (int j = 0; j < 8; ++j) f[j] |= u[j] & 0x80000000u;
  }
  peel_planes<W, Planes<W>::count - 1>(f, u, pd, lane_group, tile_group);
}

// kScaled: per-block fp32 scales instead of per-block metadata bytes.
template <typename T, int W, int kBlock, int kUnroll, bool kNT, bool kScaled>
__global__ __launch_bounds__(kBlock) void encode_blocks_kernel(const BlockArgs args) {
  constexpr uint32_t TG = kBlock * kUnroll;
  constexpr int kLoads = TileRegs<T, kUnroll>::kLoads;
  const uint4* __restrict__ src4 = static_cast<const uint4*>(args.src);
  uint8_t* __restrict__ dst = static_cast<uint8_t*>(args.dst);
  const uint8_t* __restrict__ meta = args.meta;
  const uint64_t n = args.n;
  const FormatConsts fc = args.fc;
  const BlockConsts bc = args.bc;
  const BlockIndex bi = args.bi;  // in groups
  const uint64_t G = (n + 7) / 8;
  const uint64_t Gfull = n / 8;
  const uint32_t full_tiles = (uint32_t)(Gfull / TG);
  const uint32_t rem_groups = (uint32_t)(Gfull - (uint64_t)full_tiles * TG);
  const uint32_t tiles = full_tiles + (rem_groups ? 1u : 0u);
  __shared__ __align__(16) uint8_t lds_stage[TG * W];
  const PlaneStage<W, TG> stage{lds_stage};
  const bool try_uniform = bi.size >= 4;  // at most 16 blocks per wavefront

  for (uint32_t tile = flat_tile(), once = 1; once && tile < tiles; once = 0) {
    const uint64_t g0 = (uint64_t)tile * TG;
    uint64_t blk0;
    uint32_t off;
    tile_first_block(g0, bi, blk0, off);
    const rsrc_t src = make_rsrc(src4 + g0 * kLoads);
    const rsrc_t mt = kScaled ? make_rsrc(scale_address(args, blk0)) : make_rsrc(meta + blk0);
    PlaneDst<W> pd;
    make_plane_dst<W>(dst, G, g0, pd);
    TileRegs<T, kUnroll> regs;
    uint32_t me[kUnroll];  // the block's metadatum, or the bits of its scale
    if (tile < full_tiles) {
      load_tile<T, kBlock, kUnroll, kNT, false>(src, 0, 0, regs);
      const uint32_t slot = row_slot<T, kBlock>();
#pragma unroll
      for (int r = 0; r < kUnroll; ++r)
        me[r] = load_block_datum<kScaled>(mt, lane_block<TG>(off + r * kBlock + slot, bi), args.scale_log2_bytes);
#pragma unroll
      for (int r = 0; r < kUnroll; ++r) {
        uint32_t u[8];
        group_bits<T, true>(regs.v[r], u);
        if constexpr (kScaled)  // more arithmetic per element: the stage measured slower here
          encode_group_scaled<W>(u, me[r], args.scaled_f64 != 0, fc, args.tc127, pd, slot, r * kBlock);
        else
          encode_group_meta<W>(u, me[r], fc, bc, stage, slot, r * kBlock, try_uniform);
      }
      if constexpr (!kScaled) flush_stage<W, TG, kBlock>(stage, dst, G, g0);
    } else {
      load_tile<T, kBlock, kUnroll, kNT, true>(src, 0, rem_groups, regs);
#pragma unroll
      for (int r = 0; r < kUnroll; ++r)
        if (r * kBlock + threadIdx.x < rem_groups)
          me[r] = load_block_datum<kScaled>(mt, lane_block<TG>(off + r * kBlock + threadIdx.x, bi), args.scale_log2_bytes);
#pragma unroll
      for (int r = 0; r < kUnroll; ++r) {
        if (r * kBlock + threadIdx.x < rem_groups) {  // the rounding-variant vote is among the lanes that get here
          uint32_t u[8];
          group_bits<T>(regs.v[r], u);
          if constexpr (kScaled)
            encode_group_scaled<W>(u, me[r], args.scaled_f64 != 0, fc, args.tc127, pd, threadIdx.x, r * kBlock);
          else
            encode_group_meta<W>(u, me[r], fc, bc, pd, threadIdx.x, r * kBlock, try_uniform);
        }
      }
    }
  }

  // Ragged last group: it belongs to the last block.
  if (Gfull != G && flat_tile() == 0 && threadIdx.x == 0) {
    const T* __restrict__ src = static_cast<const T*>(args.src);
    uint32_t u[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint64_t i = Gfull * 8 + j;
      u[j] = 0;
      if (i < n) {
        if constexpr (sizeof(T) == 4)
          u[j] = reinterpret_cast<const uint32_t*>(src)[i];
        else
          u[j] = elem_bits<T>(reinterpret_cast<const uint16_t*>(src)[i]);
      }
    }
    PlaneDst<W> pd;
    make_plane_dst<W>(dst, G, Gfull, pd);
    if constexpr (kScaled)
      encode_group_scaled<W>(u, load_scale_bits(args, args.n_blocks - 1), args.scaled_f64 != 0, fc, args.tc127, pd, 0, 0, false);
    else
      encode_group_meta<W>(u, meta[args.n_blocks - 1], fc, bc, pd, 0, 0, false);
  }
}

// ---------------------------------------------------------------------------
// Metadata and codes in one pass over the source (Section 2.2.1: the encoded
// tensor is the codes plus the per-block maximum exponents): the elements stay in
// registers between the block maximum and the conversion.

__device__ __forceinline__ int32_t group_key(const uint32_t u[8]) {
  int32_t k = kNoKey;
#pragma unroll
  for (int j = 0; j < 8; ++j) k = max(k, exp_key(u[j]));
  return k;
}

// The same from the group as loaded (v) and unpacked (u): a bf16 group takes its key from the packed pairs.
template <typename T>
__device__ __forceinline__ int32_t group_key(const uint4* v, const uint32_t u[8]) {
  if constexpr (std::is_same<T, uint16_t>::value)
    return key_of_pair(max_pair_keys(max_pair_keys(pair_keys(v[0].x), pair_keys(v[0].y)),
                                     max_pair_keys(pair_keys(v[0].z), pair_keys(v[0].w))));
  return group_key(u);
}

// Blocks of 2^lg groups, lg <= 6: flat tiles; the lanes of a block combine their
// keys with a butterfly, one of them writes the metadatum, all of them encode.
template <typename T, int W, int kBlock, int kUnroll, bool kNT>
__global__ __launch_bounds__(kBlock) void encode_blocks_auto_small_kernel(const BlockArgs args) {
  constexpr uint32_t TG = kBlock * kUnroll;
  constexpr int kLoads = TileRegs<T, kUnroll>::kLoads;
  const uint4* __restrict__ src4 = static_cast<const uint4*>(args.src);
  uint8_t* __restrict__ dst = static_cast<uint8_t*>(args.dst);
  const uint64_t n = args.n;
  const FormatConsts fc = args.fc;
  const BlockConsts bc = args.bc;
  const uint32_t lg = args.bi.log2;
  const uint64_t G = (n + 7) / 8;
  const uint64_t Gfull = n / 8;
  const uint32_t tiles = (uint32_t)((G + TG - 1) / TG);
  const uint32_t full_tiles = (uint32_t)(Gfull / TG);
  const uint32_t rem_whole = (uint32_t)(Gfull - (uint64_t)full_tiles * TG);
  // a whole tile leaves through LDS: its plane words (see PlaneStage) and, behind them, its metadata bytes
  __shared__ __align__(16) uint8_t lds_stage[TG * W + TG];
  const PlaneStage<W, TG> stage{lds_stage};
  uint8_t* const lds_meta = lds_stage + TG * W;
  const bool meta_words = (reinterpret_cast<uintptr_t>(args.meta) & 3u) == 0 && (TG >> lg) >= 4;

  for (uint32_t tile = flat_tile(), once = 1; once && tile < tiles; once = 0) {
    const uint64_t g0 = (uint64_t)tile * TG;
    const rsrc_t src = make_rsrc(src4 + g0 * kLoads);
    const uint32_t whole = units_in_tile(tile, full_tiles, rem_whole, TG);  // groups of this tile with all 8 elements
    TileRegs<T, kUnroll> regs;
    if (tile < full_tiles) {
      load_tile<T, kBlock, kUnroll, kNT, false, false>(src, 0, 0, regs);  // neighbouring lanes share a block: no pairs
#pragma unroll
      for (int r = 0; r < kUnroll; ++r) {
        const uint32_t idx = r * kBlock + threadIdx.x;
        uint32_t u[8];
        group_bits<T>(regs.v[r], u);
        const uint32_t me = meta_from_key(max_over_lanes(group_key<T>(regs.v[r], u), lg), bc);
        if ((threadIdx.x & ((1u << lg) - 1u)) == 0) {
          if (meta_words)
            lds_meta[idx >> lg] = (uint8_t)me;
          else
            args.meta[(g0 + idx) >> lg] = (uint8_t)me;
        }
        encode_group_meta<W>(u, me, fc, bc, stage, threadIdx.x, r * kBlock, lg >= 2);
      }
      __syncthreads();
      copy_stage<W, TG, kBlock>(stage, dst, G, g0);
      if (meta_words && threadIdx.x < (TG >> lg) / 4)
        reinterpret_cast<uint32_t*>(args.meta + (g0 >> lg))[threadIdx.x] = reinterpret_cast<const uint32_t*>(lds_meta)[threadIdx.x];
      __syncthreads();  // the image is free for the next tile
      continue;
    }
    PlaneDst<W> pd;
    make_plane_dst<W>(dst, G, g0, pd);
    load_tile<T, kBlock, kUnroll, kNT, true>(src, 0, whole, regs);
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      const uint32_t idx = r * kBlock + threadIdx.x;
      const uint64_t g = g0 + idx;
      uint32_t u[8];
      int32_t key = kNoKey;
      if (idx < whole) {
        group_bits<T>(regs.v[r], u);
        key = group_key<T>(regs.v[r], u);
      } else if (g < G) {  // the ragged last group of the tensor
        ragged_group_bits<T>(args.src, g * 8, n, u);
        key = group_key(u);
      }
      key = max_over_lanes(key, lg);  // every lane takes part
      if (g < G) {
        const uint32_t me = meta_from_key(key, bc);
        if ((threadIdx.x & ((1u << lg) - 1u)) == 0) args.meta[g >> lg] = (uint8_t)me;
        encode_group_meta<W>(u, me, fc, bc, pd, threadIdx.x, r * kBlock, lg >= 2);
      }
    }
  }
}

// Longer blocks: one workgroup per block, every lane holding up to kUnroll of the
// block's groups (the block must not exceed kBlock * kUnroll groups).
template <typename T, int W, int kBlock, int kUnroll, bool kNT>
__global__ __launch_bounds__(kBlock) void encode_blocks_auto_team_kernel(const BlockArgs args) {
  constexpr uint32_t TG = kBlock * kUnroll;
  constexpr int kLoads = TileRegs<T, kUnroll>::kLoads;
  __shared__ int32_t part[kBlock / 64];
  __shared__ __align__(16) uint8_t lds_stage[TG * W];
  const PlaneStage<W, TG> stage{lds_stage};
  const uint4* __restrict__ src4 = static_cast<const uint4*>(args.src);
  uint8_t* __restrict__ dst = static_cast<uint8_t*>(args.dst);
  const uint64_t n = args.n;
  const FormatConsts fc = args.fc;
  const BlockConsts bc = args.bc;
  const uint64_t G = (n + 7) / 8;
  const uint64_t Gfull = n / 8;
  const uint32_t bg = args.block_groups;
  // only the last block can be short or end in a ragged group (see units_in_tile for why the bookkeeping
  // avoids 64-bit order compares)
  const uint64_t last_g0 = (args.n_blocks - 1) * bg;
  const uint32_t last_count = (uint32_t)(G - last_g0), last_whole = (uint32_t)(Gfull - last_g0);

  for (uint64_t b = (uint64_t)blockIdx.z * gridDim.x + blockIdx.x, once = 1; once && b < args.n_blocks; once = 0) {
    const uint64_t g0 = b * bg;
    const bool is_last = b + 1 == args.n_blocks;
    const uint32_t count = is_last ? last_count : bg;  // groups of this block, a ragged last one included
    const uint32_t whole = is_last ? last_whole : bg;  // of them, with all 8 elements
    const rsrc_t src = make_rsrc(src4 + g0 * kLoads);
    TileRegs<T, kUnroll> regs;
    load_tile<T, kBlock, kUnroll, kNT, true>(src, 0, whole, regs);
    uint32_t ragged[8];
    const bool has_ragged = whole < count && threadIdx.x == whole % kBlock;  // the lane that owns group `whole`
    if (has_ragged) ragged_group_bits<T>(args.src, (g0 + whole) * 8, n, ragged);
    int32_t key = kNoKey;
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      if (r * kBlock + threadIdx.x < whole) {
        uint32_t u[8];
        group_bits<T>(regs.v[r], u);
        key = max(key, group_key<T>(regs.v[r], u));
      }
    }
    if (has_ragged) key = max(key, group_key(ragged));
    key = max_over_lanes(key, 6);
    if constexpr (kBlock > 64) {
      if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = key;
      __syncthreads();
#pragma unroll
      for (int w = 0; w < kBlock / 64; ++w) key = max(key, part[w]);
      __syncthreads();  // part is reused by the next block
    }
    const uint32_t me = __builtin_amdgcn_readfirstlane(meta_from_key(key, bc));
    if (threadIdx.x == 0) args.meta[b] = (uint8_t)me;
    PlaneDst<W> pd;
    make_plane_dst<W>(dst, G, g0, pd);
    // every group leaves through the LDS image (the one lane with a ragged last group adds it to the image)
#pragma unroll
    for (int r = 0; r < kUnroll; ++r) {
      if (r * kBlock + threadIdx.x < whole) {
        uint32_t u[8];
        group_bits<T>(regs.v[r], u);
        encode_group_meta<W>(u, me, fc, bc, stage, threadIdx.x, r * kBlock, false);  // me is a scalar already
      }
    }
    if (has_ragged) encode_group_meta<W>(ragged, me, fc, bc, stage, whole, 0, false);
    flush_stage_groups<W, TG, kBlock>(stage, pd, 0, count);
  }
}

// Blocks too long for the registers of one workgroup: the workgroup first walks its
// block for the maximum, then walks it again to encode; the second walk finds the
// block (tens of KB) in the L2 cache, so HBM is still read once.
template <typename T, int W, int kBlock, int kUnroll, bool kNT>
__global__ __launch_bounds__(kBlock) void encode_blocks_auto_twopass_kernel(const BlockArgs args) {
  constexpr uint32_t TG = kBlock * kUnroll;
  constexpr int kLoads = TileRegs<T, kUnroll>::kLoads;
  __shared__ int32_t part[kBlock / 64];
  __shared__ __align__(16) uint8_t lds_stage[TG * W];
  const PlaneStage<W, TG> stage{lds_stage};
  const uint4* __restrict__ src4 = static_cast<const uint4*>(args.src);
  uint8_t* __restrict__ dst = static_cast<uint8_t*>(args.dst);
  const uint64_t n = args.n;
  const FormatConsts fc = args.fc;
  const BlockConsts bc = args.bc;
  const uint64_t G = (n + 7) / 8;
  const uint64_t Gfull = n / 8;
  const uint32_t bg = args.block_groups;
  // only the last block can be short or end in a ragged group (see units_in_tile for why the bookkeeping
  // avoids 64-bit order compares)
  const uint64_t last_g0 = (args.n_blocks - 1) * bg;
  const uint32_t last_count = (uint32_t)(G - last_g0), last_whole = (uint32_t)(Gfull - last_g0);

  for (uint64_t b = (uint64_t)blockIdx.z * gridDim.x + blockIdx.x, once = 1; once && b < args.n_blocks; once = 0) {
    const uint64_t g0 = b * bg;
    const bool is_last = b + 1 == args.n_blocks;
    const uint32_t count = is_last ? last_count : bg;  // groups of this block, a ragged last one included
    const uint32_t whole = is_last ? last_whole : bg;  // of them, with all 8 elements
    const rsrc_t src = make_rsrc(src4 + g0 * kLoads);
    const uint32_t tiles = (whole + TG - 1) / TG;

    // first walk (plain loads: the lines should stay cached for the second)
    int32_t key = kNoKey;
    for (uint32_t t = 0; t < tiles; ++t) {
      TileRegs<T, kUnroll> regs;
      load_tile<T, kBlock, kUnroll, false, true>(src, t * TG, whole - t * TG, regs);
#pragma unroll
      for (int r = 0; r < kUnroll; ++r) {
        if (r * kBlock + threadIdx.x < whole - t * TG) {
          uint32_t u[8];
          group_bits<T>(regs.v[r], u);
          key = max(key, group_key<T>(regs.v[r], u));
        }
      }
    }
    uint32_t ragged[8];
    const bool has_ragged = whole < count && threadIdx.x == 0;
    if (has_ragged) {
      ragged_group_bits<T>(args.src, (g0 + whole) * 8, n, ragged);
      key = max(key, group_key(ragged));
    }
    key = max_over_lanes(key, 6);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = key;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kBlock / 64; ++w) key = max(key, part[w]);
    __syncthreads();  // part is reused by the next block
    const uint32_t me = __builtin_amdgcn_readfirstlane(meta_from_key(key, bc));
    if (threadIdx.x == 0) args.meta[b] = (uint8_t)me;

    // second walk
    PlaneDst<W> pd;
    make_plane_dst<W>(dst, G, g0, pd);
    for (uint32_t t = 0; t < tiles; ++t) {
      TileRegs<T, kUnroll> regs;
      const uint32_t here = min(whole - t * TG, TG);  // groups of this tile
      load_tile<T, kBlock, kUnroll, kNT, true>(src, t * TG, here, regs);
#pragma unroll
      for (int r = 0; r < kUnroll; ++r) {
        if (r * kBlock + threadIdx.x < here) {
          uint32_t u[8];
          group_bits<T>(regs.v[r], u);
          encode_group_meta<W>(u, me, fc, bc, stage, threadIdx.x, r * kBlock, false);  // me is a scalar already
        }
      }
      flush_stage_groups<W, TG, kBlock>(stage, pd, t * TG, here);  // out through the LDS image
    }
    if (has_ragged) {
      PlaneDst<W> pr;
      make_plane_dst<W>(dst, G, g0 + whole, pr);
      encode_group_meta<W>(ragged, me, fc, bc, pr, 0, 0, false);  // me is a scalar already
    }
  }
}

}  // namespace enc
}  // namespace exmy
