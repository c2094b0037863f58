// Shared declarations of the gfx950 eXmY codec kernels: wave-uniform format
// constants, the per-element conversion routines and the plane gather / scatter
// helpers.  Notation follows arxiv 2405.13938: X exponent bits, Y mantissa bits,
// W = 1 + X + Y, max_exp = the metadatum of Section 2 "Metadata".
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/exmy.h"

namespace exmy {

// Wave-uniform constants of a call, derived on the host and passed by value in
// the kernel arguments (they land in SGPRs).  FormatConsts depends on (X, Y)
// only and is shared by every tensor of a batch; TensorConsts also depends on
// the tensor's max_exp.
//
// emin8 = max_exp - 2^X + 2 is the biased exponent of the binade with exponent
// code 1; values under 2^(emin8-127) are rounded on the subnormal grid whose
// quantum is 2^(emin8-127-Y) (Section 2 "Subnormals").
struct FormatConsts {
  float magic_scale;    // 2^(23-Y): exponent-only float * this = the magic addend of the rounding step
  int32_t wide_exp;     // wide path: 1023 - 127 + 52 - Y, the fp64 exponent offset of the magic addend
  // The encoder builds the code left-aligned in a 32-bit register (sign, if it is
  // part of the register, at bit 31) so that plane fields can be peeled off the top.
  uint32_t left_shift;  // L: position of code bit 0 in that register
  uint32_t exp_lshift;  // L - (23 - Y): moves (clamped exponent << 23) to (exponent << (Y + L))
  uint32_t exp_shift;   // 23 - Y
  uint32_t g_clamp;     // X = 8 only: bits of the largest finite value, the cap for exponent code 255
};

struct TensorConsts {
  // ---- encode / emulate
  uint32_t sat_bits;   // fp32 bits of the largest normal; larger magnitudes (and Inf / NaN) clamp to it
  uint32_t emin_bits;  // emin8 << 23
  uint32_t bias_left;  // -(emin8 << (Y + L)) mod 2^32
  // ---- decode
  uint32_t dec_bias;   // (emin8 - 1) << 23
  float fix_mul;       // subnormal fix r = min(g, g * fix_mul + fix_add): (2, -2^(emin8-127)), or (1, 0) if emin8 = 1
  float fix_add;
};

// One tensor of a batched launch.  For encode src holds n elements and dst the
// packed planes; for decode the other way round; emulate uses src == dst.
struct TensorArgs {
  const void* src;
  void* dst;
  uint64_t n;
  TensorConsts tc;
};

// A launch covers up to kMaxBatch tensors (32: launches of 64 tensors of the checkpoint workload measured
// 2-3 % slower per byte than two launches of 32): blockIdx.y selects the tensor,
// blockIdx.x the chunk of tiles inside it.
constexpr int kMaxBatch = 32;
struct BatchArgs {
  FormatConsts fc;
  uint32_t count;
  unsigned long long* hist;  // encode with histogram only (single tensor), else null
  TensorArgs t[kMaxBatch];
};

// Per-block metadata (Section 2 "Metadata", "Block Size"): the tensor is cut into
// consecutive blocks of `block` elements, each with its own 8-bit max_exp held
// in device memory, so TensorConsts are derived on the device.  BlockConsts is
// what that derivation needs beyond the metadatum; it depends on (X, Y) only.
struct BlockConsts {
  uint32_t meta_lo;     // metadata is clamped into [meta_lo, meta_hi]: [2^X, 254], or [1, 253] for X = 0
  uint32_t meta_hi;
  uint32_t emin_off;    // emin8 = max_exp - emin_off (= 2^X - 2)
  uint32_t sat_mant;    // mantissa field of the largest value
  uint32_t sat_mask;    // all ones; 0 for e0m0, whose only magnitude is 0
  uint32_t bias_shift;  // Y + L, taken modulo 32 ...
  uint32_t bias_mask;   // ... with the result masked to 0 when Y + L = 32
  uint32_t wide_above;  // metadata above this needs the fp64 rounding path (231 + Y)
  // "maximum exponent after rounding": the block maximum's fp32 bits a become
  // a + round_half + ((a >> round_shift) & round_odd) before the exponent is read
  // (round to nearest even at the mantissa width of the top binade); all zero for
  // "before rounding".
  uint32_t round_half;
  uint32_t round_shift;
  uint32_t round_odd;
};

// Constants of the formats with reserved NaN / Inf code points (see exmy_specials_kernel.hpp).
struct SpecialConsts {
  uint32_t nan_left;    // the all-ones magnitude code, left-aligned as magnitude_code_left returns codes
  uint32_t inf_left;    // the Inf code likewise; NaN only: the largest finite code (Inf saturates)
  // decode side, on g = (code << (23 - Y)) + dec_bias, which grows with the code:
  uint32_t g_last;      // g of the largest finite code
  uint32_t g_inf;       // g of the Inf code; NaN only: 0xFFFFFFFF, which no code reaches
};

// Constants of the two's complement reading of e0mY (Section 2 "Format"): the
// code is a (1 + Y)-bit two's complement integer k, the value k quanta.
struct IntConsts {
  uint32_t sat_pos_bits;     // fp32 bits of (2^Y - 1) quanta, the largest positive value
  uint32_t neg_extra;        // fp32 bits of 2^Y quanta (the most negative magnitude) minus sat_pos_bits
  uint32_t left_shift;       // 31 - Y: moves the low 1 + Y bits of a register to its top
  float magic;               // 2^(emin8 - 127 + 23 - Y): adding it leaves round(|x| / quantum) in the low bits
  float quantum;             // 2^(emin8 - 127 - Y), emin8 = max_exp + 1
};

// How a kernel finds the metadata block of a piece of work.  Work is counted in
// the kernel's own units (groups of 8 elements, or 16-byte vectors); a block is
// `size` of them.  Tiles run flat over the tensor and may straddle blocks: the
// tile's first block and its offset inside it are wave-uniform (a shift for
// power-of-two sizes, else a multiplication by recip64 = ceil(2^64 / size), exact
// for every offset below 2^37); a lane then adds the blocks that start between
// the tile's first unit and its own.
struct BlockIndex {
  uint32_t size;     // units per block
  uint32_t log2;     // log2(size) if a power of two, else kNotPow2
  uint64_t recip64;  // ceil(2^64 / size); unused for powers of two
  uint32_t recip32;  // floor(2^32 / size) + 1: (j * recip32) >> 32 = j / size for j * size < 2^32
};
constexpr uint32_t kNotPow2 = 0xFFFFFFFFu;

// Kernel arguments of the per-block-metadata kernels (one tensor per launch).
struct BlockArgs {
  FormatConsts fc;
  BlockConsts bc;
  BlockIndex bi;        // in the launched kernel's units (set by its dispatcher)
  const void* src;      // encode / emulate: elements; decode: packed planes
  void* dst;            // encode: packed planes; decode: elements; emulate: unused
  uint8_t* meta;        // one byte per block (read; written by the max-exponent kernel)
  // Float scaling (Section 2 "Metadata": an extra bf16 or fp32 scaling factor per
  // block; Section 2.1: the third scheme of the emulation example): one scale per
  // block instead of the metadata byte, with the constants of max_exp = 127.  A
  // bf16 scale is used widened to fp32.
  void* scale;
  uint32_t scale_log2_bytes;  // 2: fp32 scales, 1: bf16 scales
  uint32_t scaled_f64;        // quotients are formed and rounded in fp64 (X = 7 or Y > 17: see scaled_sum_f64)
  TensorConsts tc127;
  float vmax127;        // largest value of the format with max_exp = 127
  uint64_t n;           // elements
  uint64_t n_blocks;    // ceil(n / block)
  uint32_t block_groups;  // block / 8
};

// Blocks that are columns or 2-D tiles of a row-major matrix (Section 2 "Block
// Size").  Lengths are in the launched kernel's units (a unit is a run of
// consecutive elements of one matrix row: a group of 8, or a 16-byte vector).
// Workgroup tiles run flat over the matrix; the row, tile row and tile column of a
// workgroup tile's first unit are wave-uniform divisions, and a lane adds the few
// rows and tiles that start between that unit and its own (see tile_meta_offset).
struct TileIndex {
  BlockIndex row;        // units per matrix row
  BlockIndex trow;       // matrix rows per tile
  BlockIndex tcol;       // units per tile along a row (columns: unused)
  uint32_t meta_stride;  // metadata bytes per tile row: tiles along a matrix row (columns: cols)
  uint32_t unit_elems;   // columns: metadata bytes per unit = elements per unit
};

// Kernel arguments of the kernels for blocks that are columns or 2-D tiles.
struct TileArgs {
  FormatConsts fc;
  BlockConsts bc;
  TileIndex ti;          // in the launched kernel's units (set by its dispatcher)
  const void* src;       // encode / emulate / maximum: the matrix; decode: packed planes
  void* dst;             // encode: packed planes; decode: the matrix
  uint8_t* meta;         // row-major (tile rows, tile columns) bytes
  uint64_t rows, cols;   // of the matrix; cols is a multiple of 8
  uint64_t tile_rows, tile_cols;  // clamped to the matrix; tile_cols is 1 or a multiple of 8
  uint64_t tiles_along_row;       // ceil(cols / tile_cols)
};

// Kernel arguments of the kernels that pack along rows (Section 2.2.2: groups are
// the 8 rows of a row block at one column of a row-major matrix).
struct RowsArgs {
  FormatConsts fc;
  TensorConsts tc;      // per-tensor metadata (meta == null)
  BlockConsts bc;       // per-row metadata: derivation constants
  BlockIndex tiles;     // tiles per row block, for the tile -> (row block, column tile) split
  const void* src;      // encode: matrix; decode: packed planes
  void* dst;            // encode: packed planes; decode: matrix
  const uint8_t* meta;  // one byte per row, or null
  uint64_t rows;
  uint32_t cols;        // a multiple of 8
  uint64_t xcd_chunk;   // 0: workgroup w takes tile w; else tile (w % 8) * xcd_chunk + w / 8 (see die_ranged_tile)
};

inline BlockIndex make_block_index(uint64_t size) {
  BlockIndex bi;
  bi.size = (uint32_t)size;
  bi.log2 = kNotPow2;
  bi.recip64 = 0;
  bi.recip32 = 0;
  if ((size & (size - 1)) == 0) {
    bi.log2 = 0;
    while ((1ull << bi.log2) < size) ++bi.log2;
  } else {
    bi.recip64 = ~0ull / size + 1;  // size is not a power of two: this is ceil(2^64 / size)
    bi.recip32 = (uint32_t)(0xFFFFFFFFull / size + 1);
  }
  return bi;
}

constexpr int kFlatWidth = 32;   // segments of 16, 8, 4, 2 and 1 bits; 32 is e8m23, the array of codes itself
constexpr int kBlockWidth = 16;
constexpr int kAnyWidth = 64;

// Host: validate (dtype, X, Y, max_exp) and fill the constants (either may be
// null).  max_width: largest W the caller's kernels handle (kFlatWidth for the
// per-tensor packed form, kBlockWidth for the per-block, scaled and row-packed
// forms, kAnyWidth for emulation, which has no packed form).
exmy_status_t make_format(exmy_dtype_t dt, int X, int Y, int max_exp, int max_width, FormatConsts* fc,
                          TensorConsts* tc, bool* needs_wide);

// Host: validate (dtype, Y, max_exp) for the two's complement reading and fill ic.
exmy_status_t make_int_format(exmy_dtype_t dt, int Y, int max_exp, bool packed, IntConsts* ic);

// Host: validate (dtype, X, Y) for per-block metadata and fill fc / bc.
// after_rounding selects the scheme of the maximum-exponent kernel; y_known is false for the "before
// rounding" maximum, whose entry point has no Y (matters for the fp16 container's metadata range only).
exmy_status_t make_block_format(exmy_dtype_t dt, int X, int Y, int max_width, bool after_rounding, bool y_known,
                                FormatConsts* fc, BlockConsts* bc);

#if defined(__HIPCC__)

__device__ __forceinline__ float as_f32(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __float_as_uint(f); }

// Global memory is reached through buffer instructions: a wave-uniform
// descriptor (base pointer in SGPRs) plus a 32-bit per-lane byte offset and a
// wave-uniform byte offset.  All 64-bit address arithmetic then stays on the
// scalar unit; a lane only ever computes lane * element_size once per block.
// Descriptors are rebuilt per chunk of tiles, so 32-bit offsets always suffice.
// kNT adds the non-temporal hint: the data is streamed once, and keeping it out
// of the caches' way leaves them to the other stream.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
// A 16-byte piece of a plane in memory.  Plane p of a tensor of G groups starts G * lo(p) bytes into the
// packed form; lo(p) is a sum of wider segments and therefore even, so a piece is known to be 2-byte
// aligned and no more (global memory takes 16-byte accesses at any alignment).
typedef u32x4_t plane_piece_t __attribute__((aligned(2)));
typedef __amdgpu_buffer_rsrc_t rsrc_t;

__device__ __forceinline__ rsrc_t make_rsrc(const void* base) {
  // raw buffer, 32-bit data format, whole 4 GiB window: callers never form an offset outside their tensor
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0xFFFFFFFFu, 0x00020000);
}

constexpr int kAuxNT = 2;  // cache-policy bit of the non-temporal hint

template <bool kNT>
__device__ __forceinline__ uint4 load16(rsrc_t r, uint32_t voffset, uint32_t soffset) {
  const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, voffset, soffset, kNT ? kAuxNT : 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}
// The wave-uniform part of the offset is added into the per-lane offset here,
// not passed in the instruction's scalar-offset field: a 16-byte buffer store
// that takes its offset from an SGPR was seen, on gfx950, to pick up a VALU
// write to its data registers issued in the very next cycle (wrong third dword
// in memory).  The compiler only spaces such a pair when the scalar-offset field
// is not a register, so the field is kept at zero.  Stores of 8 bytes or less
// read their data in one pass and are not affected.
template <bool kNT>
__device__ __forceinline__ void store16(rsrc_t r, uint32_t voffset, uint32_t soffset, uint4 v) {
  const u32x4_t w = {v.x, v.y, v.z, v.w};
  __builtin_amdgcn_raw_buffer_store_b128(w, r, voffset + soffset, 0, kNT ? kAuxNT : 0);
}

// (a << shift) + c in one VALU instruction.  The compiler would otherwise
// re-associate chains of these into separate shifts and a three-way add.
__device__ __forceinline__ uint32_t lshl_add(uint32_t a, uint32_t shift, uint32_t c) {
  uint32_t d;
  asm("v_lshl_add_u32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "s"(shift), "v"(c));
  return d;
}

// Magnitude code of one value given its fp32 bit pattern u (sign ignored),
// returned left-aligned: code << fc.left_shift (mod 2^32).
//
// Rounding (Section 2 "Rounding", Section 2.1 outcomes a-d) is done by the
// floating point adder: with ec = max(exponent of |x|, emin8), adding
// 2^(ec-127+23-Y) to |x| leaves the sum with an ulp of 2^(ec-127-Y), so the
// hardware's round-to-nearest-even produces k = round(|x| / quantum) in the low
// bits of the sum: the significand with its leading one in the normal range,
// the subnormal mantissa (possibly 0 = flushed, or 2^Y = rounded up to the
// smallest normal) below it.  A carry into the next binade needs no special
// case: the code is (ec - emin8) * 2^Y + k.  Saturation is applied on the way
// in: magnitudes above the largest normal, Inf and NaN patterns compare larger
// as unsigned integers and clamp to it.
//
// The three terms are summed already shifted left by L; everything in the sum
// above bit Y+1 belongs to the addend's exponent field and is shifted out, so
// no mask is needed: code << L = (sum << L) + (ec << (Y + L)) - (emin8 << (Y + L)).
//
// kWide = false needs max(max_exp, emin8) + 23 - Y <= 254 so that the addend is
// a finite fp32; kWide = true does the same sum in fp64 and has no such limit.
template <bool kWide>
__device__ __forceinline__ uint32_t magnitude_code_left(uint32_t u, const FormatConsts& fc, const TensorConsts& tc) {
  uint32_t a = u & 0x7FFFFFFFu;
  a = min(a, tc.sat_bits);
  const uint32_t te = max(a, tc.emin_bits) & 0x7F800000u;  // ec << 23
  uint32_t k;
  if constexpr (!kWide) {
    k = as_u32(__builtin_fmaf(as_f32(te), fc.magic_scale, as_f32(a)));
  } else {
    const uint32_t hi = ((te >> 23) + (uint32_t)fc.wide_exp) << 20;
    const double m = __hiloint2double((int)hi, 0);
    const double s = (double)as_f32(a) + m;
    k = (uint32_t)__double2loint(s);
  }
  const uint32_t q = lshl_add(te, fc.exp_lshift, tc.bias_left);
  return lshl_add(k, fc.left_shift, q);
}

// Value of a magnitude code from g = (code << (23 - Y)) + ((emin8 - 1) << 23),
// as fp32 bits with the sign clear.
//
// For exponent codes >= 1, g is already the bit pattern of the value (an affine
// map of the code).  For exponent code 0, g reads as (2^Y + M) * quantum / 2
// while the value is M * quantum = 2g - 2^(emin8-127); for every other code
// 2g - that constant is >= g, so one fused multiply-add and a minimum pick the
// right one without a branch.  When emin8 = 1, g is an fp32 denormal and already
// the value: the constants (1, 0) then make the second operand equal g.
// g is never a NaN pattern here (X = 8 callers clamp it first), so the minimum
// is taken with the bare instruction, without a canonicalising pre-pass.
__device__ __forceinline__ uint32_t finish_magnitude(uint32_t g_bits, const TensorConsts& tc) {
  const float g = as_f32(g_bits);
  const float t = __builtin_fmaf(g, tc.fix_mul, tc.fix_add);
  float r;
  asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(g), "v"(t));
  return as_u32(r);
}

// TensorConsts of a block from its metadata byte (see make_format on the host for
// the same derivation from a host-side max_exp).
__device__ __forceinline__ TensorConsts derive_tc(uint32_t max_exp, const BlockConsts& bc) {
  const uint32_t me = min(max(max_exp, bc.meta_lo), bc.meta_hi);
  const uint32_t emin8 = me - bc.emin_off;
  TensorConsts tc;
  tc.sat_bits = ((me << 23) | bc.sat_mant) & bc.sat_mask;
  tc.emin_bits = emin8 << 23;
  tc.bias_left = ((0u - emin8) << bc.bias_shift) & bc.bias_mask;
  tc.dec_bias = (emin8 - 1u) << 23;  // emin8 >= 2 in block mode: never an fp32-denormal pattern
  tc.fix_mul = 2.0f;
  tc.fix_add = as_f32(0x80000000u | (emin8 << 23));  // -2^(emin8-127)
  return tc;
}

// Whether every active lane of the wavefront holds the same value (then also in `first`, as a scalar).  With one
// metadatum for the whole wavefront (blocks of 512 elements or more, or neighbouring blocks that agree) the
// block kernels derive the constants once, on the scalar unit, instead of per lane: 8 VALU operations per group
// or vector less, which is +11 % for the bf16 emulation.
__device__ __forceinline__ bool wave_uniform(uint32_t v, uint32_t& first) {
  first = __builtin_amdgcn_readfirstlane(v);
  return __builtin_amdgcn_ballot_w64(v != first) == 0;
}

// Key of an element for the block maximum: its magnitude bits plus one in the
// exponent field, as a signed integer.  Inf / NaN patterns come out negative, so
// a signed maximum over keys skips them; no finite element gives a key <= 0.
__device__ __forceinline__ int32_t exp_key(uint32_t u) { return (int32_t)((u & 0x7FFFFFFFu) + 0x00800000u); }
constexpr int32_t kNoKey = (int32_t)0x80000000;

// The same keys for the two bf16 halves of a dword at once, as two signed 16-bit integers (the upper 16
// bits of exp_key of each element): no carry crosses the halves, and a packed 16-bit maximum then handles
// two elements per instruction.  key_of_pair is the larger of the two as an exp_key.
typedef short i16x2_t __attribute__((ext_vector_type(2)));
constexpr uint32_t kNoPairKeys = 0x80008000u;
__device__ __forceinline__ uint32_t pair_keys(uint32_t w) { return (w & 0x7FFF7FFFu) + 0x00800080u; }
__device__ __forceinline__ uint32_t max_pair_keys(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(i16x2_t, a), __builtin_bit_cast(i16x2_t, b)));
}
__device__ __forceinline__ int32_t key_of_pair(uint32_t p) { return max((int32_t)(p & 0xFFFF0000u), (int32_t)(p << 16)); }

// Metadatum of a block from the largest key of its elements: the biased exponent
// of the largest finite magnitude, "before rounding" or, with the round_* fields
// set, after that magnitude is rounded to the mantissa width of the top binade
// (Section 2 "Metadata"), clamped into the valid range.
__device__ __forceinline__ uint32_t meta_from_key(int32_t key, const BlockConsts& bc) {
  uint32_t a = key > 0 ? (uint32_t)key - 0x00800000u : 0u;  // bits of the largest finite magnitude (0 if none)
  a += bc.round_half + ((a >> bc.round_shift) & bc.round_odd);  // may carry up to exponent 255
  return min(max(a >> 23, bc.meta_lo), bc.meta_hi);
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

// The tile of a workgroup in the kernels that take one tile per workgroup: x, continued in z for tensors of
// more than gridDim.x tiles (y, where used, selects the tensor of a batch).  Such kernels are written as
//   for (uint32_t tile = flat_tile(), once = 1; once && tile < tiles; once = 0) { ... }
// a loop that the compiler can see runs at most once, so that `continue` still means "done with this
// tile" while none of a real loop's bookkeeping (copies of loop-carried registers, set-up hoisted out of
// it: 10 % of the 7-bit encoder's vector instructions) is generated.
__device__ __forceinline__ uint32_t flat_tile() { return blockIdx.z * gridDim.x + blockIdx.x; }

// Units of workgroup tile `tile` when `full_tiles` whole tiles of kTile units are followed by one of `rem`
// units.  Kept in 32-bit scalar compares on purpose: the same bookkeeping written as a 64-bit
// "left < kTile ? left : kTile" followed by a branch on the result was seen to be compiled into a select on
// a stale condition code by this toolchain (the partial tile then ran as a whole one).
__device__ __forceinline__ uint32_t units_in_tile(uint32_t tile, uint32_t full_tiles, uint32_t rem, uint32_t kTile) {
  return tile < full_tiles ? kTile : (tile == full_tiles ? rem : 0u);
}

// Tile of this workgroup when every accelerator die takes a contiguous range of `chunk` tiles.  Workgroups are
// handed to the 8 dies (each with an L2 cache of its own) in turn, so with tile = workgroup, the cache lines
// that neighbouring tiles share when matrix rows do not end on line boundaries are held, partly written, in
// two L2 caches and reach memory as two partial writes (or are fetched once per die).  With die k working on
// tiles [k * chunk, (k + 1) * chunk) such a line stays within one L2 (+10-20 % for the row-packing kernels on
// such matrices; on aligned data, and for lines of metadata bytes written one byte per workgroup, the plain
// order measured 2-5 % faster).  chunk = 0: tile = workgroup.  The grid must hold 8 * chunk workgroups; tiles
// past the last one are the caller's to skip.
__device__ __forceinline__ uint64_t die_ranged_tile(uint64_t chunk) {
  const uint64_t w = flat_tile();
  return chunk ? (w & 7u) * chunk + (w >> 3) : w;
}

// First block touched by the tile whose first unit is w0, and w0's offset inside it.
__device__ __forceinline__ void tile_first_block(uint64_t w0, const BlockIndex& bi, uint64_t& blk0, uint32_t& off) {
  if (bi.log2 != kNotPow2) {
    blk0 = w0 >> bi.log2;
    off = (uint32_t)w0 & (bi.size - 1u);
  } else {
    blk0 = __umul64hi(w0, bi.recip64);
    off = (uint32_t)(w0 - blk0 * bi.size);
  }
}

// Block of the unit j = off + (the lane's unit inside the tile), relative to the
// tile's first block.  kTile = units per tile.
template <uint32_t kTile>
__device__ __forceinline__ uint32_t lane_block(uint32_t j, const BlockIndex& bi) {
  if (bi.log2 != kNotPow2) return j >> bi.log2;
  if (bi.size >= kTile) return j >= bi.size ? 1u : 0u;  // a tile straddles at most one boundary
  return __umulhi(j, bi.recip32);                       // j < 2 * kTile
}

// Uniform position of a workgroup tile whose first unit is w0: its matrix row's
// tile row (through `meta_row`, the metadata offset of that tile row), the row's
// place inside that tile row, the unit's place in its matrix row, and that
// place's tile column and remainder.
struct TileStart {
  uint64_t meta_row;  // tile row * meta_stride
  uint32_t rr0;       // matrix row - tile row * rows per tile
  uint32_t cu0;       // unit inside the matrix row
  uint32_t ct0, cr0;  // cu0 / tile width, cu0 % tile width (tiles only)
  bool one_row;       // the workgroup tile ends inside the matrix row it starts in
};

template <uint32_t kTile, bool kColumns>
__device__ __forceinline__ TileStart tile_start(uint64_t w0, const TileIndex& ti) {
  TileStart ts;
  uint64_t row0, tb0;
  tile_first_block(w0, ti.row, row0, ts.cu0);
  ts.one_row = ts.cu0 + kTile <= ti.row.size;
  tile_first_block(row0, ti.trow, tb0, ts.rr0);
  ts.meta_row = tb0 * ti.meta_stride;
  ts.ct0 = ts.cr0 = 0;
  if constexpr (!kColumns) {
    uint64_t q;
    tile_first_block(ts.cu0, ti.tcol, q, ts.cr0);
    ts.ct0 = (uint32_t)q;
  }
  return ts;
}

// Metadata byte offset, from the start of the workgroup tile's tile row, of unit
// jl < kTile of the workgroup tile.  All quotients have small numerators (see
// lane_block): a lane is at most kTile units past the uniform start.  kColumns:
// one metadatum per element and column; the offset is that of the unit's first
// element.
template <uint32_t kTile, bool kColumns>
__device__ __forceinline__ uint32_t tile_meta_offset(uint32_t jl, const TileIndex& ti, const TileStart& ts) {
  if (ts.one_row) {  // wave-uniform: same matrix row and tile row as the start
    if constexpr (kColumns) return (ts.cu0 + jl) * ti.unit_elems;
    return ts.ct0 + lane_block<kTile>(ts.cr0 + jl, ti.tcol);
  }
  const uint32_t j = ts.cu0 + jl;
  const uint32_t dr = lane_block<kTile>(j, ti.row);                 // matrix rows that start in between
  const uint32_t dt = lane_block<kTile>(ts.rr0 + dr, ti.trow);      // tile rows that start in between
  const uint32_t cu = j - dr * ti.row.size;                         // unit inside its own matrix row
  if constexpr (kColumns) return dt * ti.meta_stride + cu * ti.unit_elems;
  // same matrix row as the start: continue from its tile column; a later row restarts at column 0 (then cu <= jl)
  const uint32_t ct = (dr ? 0u : ts.ct0) + lane_block<kTile>(dr ? cu : ts.cr0 + jl, ti.tcol);
  return dt * ti.meta_stride + ct;
}

// The datum of block number `block` of the array behind `r`: a metadata byte, or
// the fp32 bits of a scale stored as fp32 or bf16 (`scale_log2_bytes`, uniform).
template <bool kScaled>
__device__ __forceinline__ uint32_t load_block_datum(rsrc_t r, uint32_t block, uint32_t scale_log2_bytes) {
  if constexpr (kScaled) {
    if (scale_log2_bytes == 2) return __builtin_amdgcn_raw_buffer_load_b32(r, block * 4u, 0, 0);
    return (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(r, block * 2u, 0, 0) << 16;
  }
  return __builtin_amdgcn_raw_buffer_load_b8(r, block, 0, 0);
}

// Address of the scale of block `block`, and its fp32 bits.
__device__ __forceinline__ char* scale_address(const BlockArgs& args, uint64_t block) {
  return static_cast<char*>(args.scale) + (block << args.scale_log2_bytes);
}
__device__ __forceinline__ uint32_t load_scale_bits(const BlockArgs& args, uint64_t block) {
  const char* p = scale_address(args, block);
  if (args.scale_log2_bytes == 2) return *reinterpret_cast<const uint32_t*>(p);
  return (uint32_t)*reinterpret_cast<const uint16_t*>(p) << 16;
}

// Element types: float (fp32), uint16_t (bf16: the upper half of an fp32) and
// f16_t (IEEE half: converted exactly to fp32 on the way in; the formats admitted
// for it decode to fp16 values only, so the way out is exact too).  Elements of
// the 16-bit types travel in pairs inside dwords.
struct f16_t {
  uint16_t bits;
};
template <typename T>
inline constexpr bool kIsF16 = false;
template <>
inline constexpr bool kIsF16<f16_t> = true;

// fp32-position bits of a 16-bit element.
template <typename T>
__device__ __forceinline__ uint32_t elem_bits(uint16_t raw) {
  if constexpr (kIsF16<T>) return as_u32((float)__builtin_bit_cast(_Float16, raw));
  return (uint32_t)raw << 16;
}
template <typename T>
__device__ __forceinline__ uint32_t lo_elem_bits(uint32_t w) {
  if constexpr (kIsF16<T>) return elem_bits<T>((uint16_t)w);
  return w << 16;
}
template <typename T>
__device__ __forceinline__ uint32_t hi_elem_bits(uint32_t w) {
  if constexpr (kIsF16<T>) return elem_bits<T>((uint16_t)(w >> 16));
  return w & 0xFFFF0000u;
}
// The 16-bit element with exactly the value of these fp32 bits, and a pair of them in a dword.
template <typename T>
__device__ __forceinline__ uint16_t to_elem(uint32_t bits) {
  if constexpr (kIsF16<T>) return __builtin_bit_cast(uint16_t, (_Float16)as_f32(bits));
  return (uint16_t)(bits >> 16);
}
// kExact: the values are known to be values of T (any rounding mode converts them exactly); otherwise an
// fp16 pair is rounded to nearest even here, and a bf16 pair must have been rounded by the caller.
template <typename T, bool kExact = true>
__device__ __forceinline__ uint32_t pack_elems(uint32_t lo_bits, uint32_t hi_bits) {
  if constexpr (kIsF16<T>) {
    if constexpr (kExact) return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(as_f32(lo_bits), as_f32(hi_bits)));
    return (uint32_t)to_elem<T>(lo_bits) | ((uint32_t)to_elem<T>(hi_bits) << 16);
  }
  return __builtin_amdgcn_perm(hi_bits, lo_bits, 0x07060302u);
}

// Of a pair of halves w, the original 16 bits where the half is Inf / NaN (a half's NaN payload would
// not survive the round trip through fp32 unchanged); elsewhere the pair `emulated`.
__device__ __forceinline__ uint32_t keep_nonfinite_halves(uint32_t w, uint32_t emulated);

// (mask & a) | (~mask & b) in one instruction.
__device__ __forceinline__ uint32_t bit_select(uint32_t mask, uint32_t a, uint32_t b) {
  uint32_t d;
  asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(d) : "v"(mask), "v"(a), "v"(b));
  return d;
}

// ---------------------------------------------------------------- float scaling
//
// Section 2 "Metadata" / Section 2.1 (an extra fp32 or bf16 scale per block, codes of the max_exp = 127
// format).  The code of x is that of the real quotient |x| / s: nearest grid point, ties to even.  The
// kernels multiply by inv = fl(1 / s) instead of dividing, so their quotient q = fl(|x| * inv) carries a
// relative error of up to 2^-23 (2^-21.7 when s > 2^126 makes inv an fp32 denormal); that matters only
// for the few elements whose quotient lies that close to a rounding boundary of the grid.  They are
// found by rounding twice, q * (1 - eps) and q * (1 + eps) (each inside one fused multiply-add with the
// rounding addend, so the perturbation itself is not rounded): where both give the same sum the real
// quotient, which lies in between, gives it too.  Where they differ (by one grid step) the boundary m
// between the two candidates is a short float, and the sign of the exact residual |x| - m * s, again one
// fused multiply-add, says on which side of it the real quotient lies (zero: an exact tie, the even
// candidate).  That second step runs only in wavefronts where a ballot finds such an element.
//
// Valid for X <= 6 and Y <= 21: every rounding boundary of the format is then far above the fp32
// denormals, so a quotient small enough to lose bits rounds to zero whatever its error.  e7mY (whose
// subnormal grid lies among the fp32 denormals) and Y > 21 take scaled_sum_f64 below.
struct ScaleOfBlock {
  float scale;   // s, finite and >= FLT_MIN
  float inv;     // fl(1 / s)
  float one_lo;  // 1 - eps
  float one_hi;  // 1 + eps
};

__device__ __forceinline__ ScaleOfBlock scale_of_block(uint32_t scale_bits) {
  ScaleOfBlock sb;
  sb.scale = as_f32(scale_bits);
  sb.inv = 1.0f / sb.scale;
  const bool tiny_inv = scale_bits > 0x7E800000u;  // s > 2^126: inv is a denormal with 22 or 21 significant bits
  sb.one_lo = tiny_inv ? 1.0f - 0x1p-20f : 1.0f - 0x1p-22f;
  sb.one_hi = tiny_inv ? 1.0f + 0x1p-20f : 1.0f + 0x1p-22f;
  return sb;
}

// The two rounded sums of the element with fp32-position bits u (see magnitude_code_left for what a sum
// is: rounding addend + |value|, whose low bits are round(|value| / quantum)); te = clamped exponent << 23.
struct ScaledSums {
  uint32_t te, lo, hi;
};
__device__ __forceinline__ ScaledSums scaled_sums(uint32_t u, const ScaleOfBlock& sb, const FormatConsts& fc,
                                                  const TensorConsts& tc127) {
  uint32_t q = as_u32(__builtin_fabsf(as_f32(u)) * sb.inv);  // Inf, NaN and overflow: patterns above sat_bits
  q = min(q, tc127.sat_bits);
  ScaledSums r;
  r.te = max(q, tc127.emin_bits) & 0x7F800000u;
  const float addend = as_f32(r.te) * fc.magic_scale;  // a power of two: exact
  r.lo = as_u32(__builtin_fmaf(as_f32(q), sb.one_lo, addend));
  r.hi = as_u32(__builtin_fmaf(as_f32(q), sb.one_hi, addend));
  return r;
}

// The sum of the real quotient for an element whose two sums differ (for one whose sums agree: that sum).
// s_mant, s_exp: the scale as s_mant * 2^s_exp with s_mant in [0.5, 1).  All operands of the residual are
// brought near 1 first, so that it cannot underflow: m * s_mant has at most 42 significant bits above
// 2^-105, and |x| * 2^-s_exp is exact because it is about as large as that product.  A residual of zero is an
// exact tie and goes to the even sum: a term far below any non-zero residual, positive when the lower sum
// is odd, turns that into the same sign test.
__device__ __forceinline__ uint32_t settle_scaled_sum(uint32_t u, const ScaledSums& ss, float s_mant, int s_exp,
                                                      const FormatConsts& fc) {
  const float addend = as_f32(ss.te) * fc.magic_scale;
  // lower candidate (the sum minus the addend) + half a quantum (the addend * 2^-24): the boundary, exact
  const float m = __builtin_fmaf(addend, 0x1p-24f - 1.0f, as_f32(ss.lo));
  const float a = __builtin_ldexpf(__builtin_fabsf(as_f32(u)), -s_exp);
  const float resid = __builtin_fmaf(-m, s_mant, a);                // sign of |x| - m * s, exact
  const float tie = as_f32((ss.lo << 31) + 0x83800000u);           // -2^-120, or +2^-120 when the lower sum is odd
  return resid + tie > 0.0f ? ss.hi : ss.lo;
}

// Left-aligned magnitude code (as magnitude_code_left returns it) from a sum and its te.
__device__ __forceinline__ uint32_t code_left_of_sum(uint32_t sum, uint32_t te, const FormatConsts& fc,
                                                     const TensorConsts& tc) {
  return lshl_add(sum, fc.left_shift, lshl_add(te, fc.exp_lshift, tc.bias_left));
}

// The same rounding in fp64, for the formats the scheme above does not cover: the quotient is the IEEE
// fp64 division |x| / s, within 2^-53 of the real one and exact where the real one is a double.  A real
// quotient that is exactly a rounding boundary is one (boundaries have at most 26 significant bits); any
// other stays more than 2^-51 of its size away from every boundary (a 24-bit number against the product
// of a boundary and a 24-bit scale), further than the division's error.  Returns the low word of the fp64
// sum (k) and te; `value` receives the rounded magnitude.
__device__ __forceinline__ uint32_t scaled_sum_f64(uint32_t u, double scale64, const FormatConsts& fc,
                                                   const TensorConsts& tc127, uint32_t& te, float& value) {
  double t = __builtin_fabs((double)as_f32(u)) / scale64;
  const double vmax = (double)as_f32(tc127.sat_bits);
  t = t < vmax ? t : vmax;  // anything above the largest value, Inf and NaN (for which the compare is false)
  const uint32_t e11 = (uint32_t)__double2hiint(t) >> 20;
  const uint32_t ec = max(e11, (tc127.emin_bits >> 23) + 896u);  // as an fp64 exponent field (1023 = 127 + 896)
  const double addend = __hiloint2double((int)((ec - 896u + (uint32_t)fc.wide_exp) << 20), 0);
  const double sum = t + addend;
  te = (ec - 896u) << 23;
  value = (float)(sum - addend);
  return (uint32_t)__double2loint(sum);
}

// Float scaling, decode side: the real product v * s rounded once, to nearest even, into the container.
// fp32: the multiplication itself.  bf16 / fp16: the fp32 product p is rounded again by the conversion,
// which goes wrong exactly when p is inexact and lies half-way between two values of the narrower type.
// All such p have their low 15 (bf16) / 12 (fp16, whose denormals shift the half-way bit upwards) bits
// clear; scaled_product_suspect says whether p is one of those, and settle_scaled_product then moves an
// inexact p one ulp towards the real product, which takes it off the half-way point on the right side
// (and does no harm to a p that is a value of the narrower type).
template <typename T>
__device__ __forceinline__ bool scaled_product_low_bits_clear(float p) {
  return (as_u32(p) & (kIsF16<T> ? 0x00000FFFu : 0x00007FFFu)) == 0;
}

// Whether one of a lane's E products may be such a half-way case (then every lane of the wavefront settles
// its products).  short_scale (wave-uniform): the scales are bf16 values, so a product has at most 19
// significant bits and is exact unless it falls among the fp32 denormals.
template <typename T, int E>
__device__ __forceinline__ bool scaled_products_suspect(const float (&p)[E], bool short_scale) {
  if (short_scale) {
    uint32_t lowest = 0xFFFFFFFFu;
#pragma unroll
    for (int j = 0; j < E; ++j) lowest = min(lowest, (as_u32(p[j]) << 1) - 2u);  // sign dropped; zero wraps to the top
    return lowest < 0x00FFFFFEu;
  }
  if constexpr (kIsF16<T>) {
    uint32_t lowest = 0xFFFFFFFFu;
#pragma unroll
    for (int j = 0; j < E; ++j) lowest = min(lowest, as_u32(p[j]) << 20);
    return lowest == 0;
  } else {
    // bf16: the half-way pattern is a lower half of 0x8000, the smallest signed 16-bit number, so a packed
    // signed minimum over the products' bits finds it (the upper halves ride along unused)
    uint32_t lowest = 0x7FFF7FFFu;
#pragma unroll
    for (int j = 0; j < E; ++j)
      lowest = __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(i16x2_t, lowest),
                                                                      __builtin_bit_cast(i16x2_t, as_u32(p[j]))));
    return (lowest & 0xFFFFu) == 0x8000u;
  }
}

// p = fl(v * s) moved one ulp towards the real product where it is inexact and `suspect` (its low bits
// are clear); s = s_mant * 2^s_exp with s_mant in [0.5, 1).  Signs ride along untouched.
__device__ __forceinline__ float settle_scaled_product(float p, float v, float s_mant, int s_exp, bool suspect) {
  // v * s - p on magnitudes, exactly signed: operands brought near 1 so that the residual cannot underflow
  const float av = __builtin_fabsf(v), ap = __builtin_fabsf(p);
  const float v_mant = __builtin_amdgcn_frexp_mantf(av);
  const int v_exp = __builtin_amdgcn_frexp_expf(av);
  const float resid = __builtin_fmaf(v_mant, s_mant, -__builtin_ldexpf(ap, -(v_exp + s_exp)));  // > 0: p is too small
  uint32_t b = as_u32(p);
  const bool finite_nonzero = (as_u32(ap) - 1u) < 0x7F7FFFFFu;
  if (suspect && finite_nonzero && resid != 0.0f) b += resid > 0.0f ? 1u : 0xFFFFFFFFu;  // the magnitude, +-1 ulp
  return as_f32(b);
}

// One product on its own (the few elements after the last whole vector): fp32-position bits of v * s
// rounded once to T (bf16: in the upper half), under the sign of v.
template <typename T>
__device__ __forceinline__ uint32_t scaled_product_bits(uint32_t v_bits, float scale) {
  float p = as_f32(v_bits) * scale;
  if constexpr (sizeof(T) == 2) {
    p = settle_scaled_product(p, as_f32(v_bits), __builtin_amdgcn_frexp_mantf(scale), __builtin_amdgcn_frexp_expf(scale),
                              scaled_product_low_bits_clear<T>(p));
    if constexpr (!kIsF16<T>) {
      uint32_t m = as_u32(p) & 0x7FFFFFFFu;
      m += 0x7FFFu + ((m >> 16) & 1u);  // to nearest even at bit 16; a carry may run up to the Inf pattern
      return (m & 0xFFFF0000u) | (v_bits & 0x80000000u);
    }
  }
  return as_u32(p);
}

// One element's code sum on its own, always settled (no vote): the sum and its te.
__device__ __forceinline__ uint32_t scaled_sum_settled(uint32_t u, uint32_t scale_bits, const FormatConsts& fc,
                                                       const TensorConsts& tc127, uint32_t& te) {
  const ScaleOfBlock sb = scale_of_block(scale_bits);
  const ScaledSums ss = scaled_sums(u, sb, fc, tc127);
  te = ss.te;
  return settle_scaled_sum(u, ss, __builtin_amdgcn_frexp_mantf(sb.scale), __builtin_amdgcn_frexp_expf(sb.scale), fc);
}

__device__ __forceinline__ uint32_t keep_nonfinite_halves(uint32_t w, uint32_t emulated) {
  const uint32_t lo = (w & 0x00007C00u) == 0x00007C00u ? 0x0000FFFFu : 0u;
  const uint32_t hi = (w & 0x7C000000u) == 0x7C000000u ? 0xFFFF0000u : 0u;
  return bit_select(lo | hi, w, emulated);
}

// The same for a pair of bf16.
__device__ __forceinline__ uint32_t keep_nonfinite_bf16(uint32_t w, uint32_t emulated) {
  const uint32_t lo = (w & 0x00007F80u) == 0x00007F80u ? 0x0000FFFFu : 0u;
  const uint32_t hi = (w & 0x7F800000u) == 0x7F800000u ? 0xFFFF0000u : 0u;
  return bit_select(lo | hi, w, emulated);
}

// Two fp32 values rounded to nearest even into a bf16 pair: the conversion instruction of
// gfx950 (an overflow gives Inf, as in the library conversion).
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t round_pack_bf16(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// ---------------------------------------------------------------- planes

// Number of planes and their segment widths, widest first (7 -> 4, 2, 1).
template <int W>
struct Planes {
  static constexpr int count = __builtin_popcount(W);
  __host__ __device__ static constexpr int seg(int p) {
    int s = 16, i = 0;
    while (true) {
      if (W & s) {
        if (i == p) return s;
        ++i;
      }
      s >>= 1;
    }
  }
  __host__ __device__ static constexpr int lo(int p) {  // lowest code bit of plane p
    int l = 0;
    for (int i = 0; i < p; ++i) l += seg(i);
    return l;
  }
};


// The LDS image of a tile of kTileGroups groups holds the tile's part of plane P at byte
// kTileGroups * lo(P), the word of the tile's group i at i * seg(P) inside it.  Memory
// address of the 16-byte piece at byte `off` of that image; g0 is the tile's first group,
// G the tensor's group count.  A piece lies inside one plane because kTileGroups is a
// multiple of 16.
template <int W, int kTileGroups, int P = 0>
__device__ __forceinline__ uint8_t* tile_piece_address(uint8_t* packed, uint64_t G, uint64_t g0, uint32_t off) {
  static_assert(kTileGroups % 16 == 0, "plane images must be whole 16-byte pieces");
  constexpr uint32_t S = Planes<W>::seg(P);
  constexpr uint32_t LO = Planes<W>::lo(P);
  if constexpr (P + 1 < Planes<W>::count) {
    if (off >= kTileGroups * (LO + S)) return tile_piece_address<W, kTileGroups, P + 1>(packed, G, g0, off);
  }
  return packed + (G * LO + g0 * S + (off - kTileGroups * LO));
}

#endif  // __HIPCC__

}  // namespace exmy
