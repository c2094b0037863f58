// C ABI of the eXmY codec: host-side validation, derivation of the wave-uniform
// format constants, and dispatch to the gfx950 kernels.  Declared and documented
// in include/exmy.h.
#include <math.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <vector>

#include "exmy_common.hpp"
#include "exmy_launch.hpp"

namespace exmy {

namespace {

uint32_t float_bits(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  return u;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

int compute_units() {
  constexpr int kMaxDevices = 64;
  static std::atomic<int> cached[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
  int cu = cached[dev].load(std::memory_order_relaxed);
  if (cu == 0) {
    if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu <= 0) cu = 256;
    cached[dev].store(cu, std::memory_order_relaxed);
  }
  return cu;
}

exmy_status_t make_format(exmy_dtype_t dt, int X, int Y, int max_exp, int max_width, FormatConsts* fc,
                          TensorConsts* tc, bool* needs_wide) {
  if (dt != EXMY_F32 && dt != EXMY_BF16 && dt != EXMY_F16) return EXMY_ERR_FORMAT;
  if (X < 0 || X > 8 || Y < 0) return EXMY_ERR_FORMAT;
  if (dt == EXMY_F16 && X > 5) return EXMY_ERR_FORMAT;
  // Section 2.1: bf16 holds Y <= 7, fp16 Y <= 10 (and X <= 5), fp32 Y <= 23; a sign-magnitude
  // format (X = 0) has no leading one, so its Y bits need only Y significant bits of the container.
  const int P = dt == EXMY_F32 ? 23 : (dt == EXMY_F16 ? 10 : 7);
  if (Y > (X >= 1 ? P : P + 1)) return EXMY_ERR_FORMAT;
  if (1 + X + Y > max_width) return EXMY_ERR_FORMAT;
  if (max_width != kAnyWidth && Y > 23) return EXMY_ERR_FORMAT;  // e0m24 packs as e1m23, which it equals bit for bit
  if (X == 8) {
    if (max_exp != 255) return EXMY_ERR_MAX_EXP;
  } else if (X == 0) {
    if (max_exp < 0 || max_exp > 253) return EXMY_ERR_MAX_EXP;
    if (Y == P + 1 && max_exp < 1) return EXMY_ERR_MAX_EXP;  // quantum below the container's
  } else {
    if (max_exp < (1 << X) - 1 || max_exp > 254) return EXMY_ERR_MAX_EXP;
  }

  const int emin8 = max_exp - (1 << X) + 2;
  // fp16 holds binades 2^-14 .. 2^15 and multiples of 2^-24 below them: the format's top binade and its
  // quantum must lie inside, so that every decoded value is an fp16 value
  if (dt == EXMY_F16 && (max_exp > 142 || emin8 - 127 - Y < -24)) return EXMY_ERR_MAX_EXP;
  const uint32_t ones_y = (uint32_t)((1ull << Y) - 1ull);
  // Odd widths end in a 1-bit plane that holds exactly the sign: the encoder takes
  // it from the source bits and left-aligns the magnitude alone.
  const int W = 1 + X + Y;
  const int L = ((W & 1) ? 32 : 31) - (X + Y);
  // Largest value: (2 - 2^-Y) * 2^(max_exp-127) with X >= 1 (X = 8: exponent 254, the
  // largest finite float); (2^Y - 1) quanta with X = 0.
  uint32_t sat_bits;
  if (X == 0) {
    sat_bits = float_bits(ldexpf((float)ones_y, emin8 - 127 - Y));
  } else {
    const uint32_t top = X == 8 ? 254u : (uint32_t)max_exp;
    sat_bits = (top << 23) | (ones_y << (23 - Y));
  }

  if (fc) {
    memset(fc, 0, sizeof(*fc));
    fc->magic_scale = ldexpf(1.0f, 23 - Y);
    fc->wide_exp = 1023 - 127 + 52 - Y;
    fc->left_shift = (uint32_t)(L & 31);  // L = 32 only for W = 1, where no magnitude bits exist
    fc->exp_lshift = (uint32_t)((L - (23 - Y)) & 31);
    fc->exp_shift = (uint32_t)((23 - Y) & 31);  // Y = 24 (X = 0, fp32) is reachable by emulate only, which does not use it
    fc->g_clamp = sat_bits;
  }
  if (tc) {
    memset(tc, 0, sizeof(*tc));
    tc->sat_bits = sat_bits;
    tc->emin_bits = (uint32_t)emin8 << 23;
    tc->bias_left = (uint32_t)(0ull - ((uint64_t)emin8 << (Y + L)));
    tc->dec_bias = (uint32_t)(emin8 - 1) << 23;
    if (emin8 == 1) {
      tc->fix_mul = 1.0f;
      tc->fix_add = 0.0f;
    } else {
      tc->fix_mul = 2.0f;
      tc->fix_add = -ldexpf(1.0f, emin8 - 127);
    }
  }
  // The fp32 magic addend 2^(ec-127+23-Y) must be finite for the largest clamped
  // exponent ec, and the sum must stay in the addend's binade (Y <= 21).
  const int ec_max = X == 0 ? emin8 : (X == 8 ? 254 : max_exp);
  // Codes of more than 23 bits (24 with the sign riding along) would also pick up exponent
  // bits of the fp32 sum when it is shifted left; the fp64 sum has zeros there.
  const int kept = X + Y + ((W & 1) ? 0 : 1);
  if (needs_wide) *needs_wide = (ec_max + 23 - Y > 254) || (Y > 21) || (kept > 23);
  return EXMY_OK;
}

exmy_status_t make_block_format(exmy_dtype_t dt, int X, int Y, int max_width, bool after_rounding, bool y_known,
                                FormatConsts* fc, BlockConsts* bc) {
  if (X == 8) return EXMY_ERR_FORMAT;  // identity exponent map: nothing for a block to choose
  // valid metadata: [2^X, 254] ([1, 253] for X = 0); inside fp16 also the container's limits on the top binade
  // (at most 2^15) and, where the caller knows Y, on the quantum (at least 2^-24)
  int lo = X == 0 ? 1 : (1 << X);
  int hi = X == 0 ? 253 : 254;
  if (dt == EXMY_F16) {
    hi = 142;
    if (y_known) lo = std::max(lo, X == 0 ? 102 + Y : 101 + Y + (1 << X));
    if (X <= 5 && lo > hi) return EXMY_ERR_FORMAT;  // no metadatum keeps this format inside fp16
  }
  if (exmy_status_t st = make_format(dt, X, Y, hi, max_width, fc, nullptr, nullptr)) return st;
  if (bc) {
    const int W = 1 + X + Y;
    const int L = ((W & 1) ? 32 : 31) - (X + Y);
    bc->meta_lo = (uint32_t)lo;
    bc->meta_hi = (uint32_t)hi;
    bc->emin_off = (1u << X) - 2u;  // X = 0: 2^0 - 2 = -1, i.e. emin8 = max_exp + 1 (wraps as intended)
    // largest value: exponent field max_exp; mantissa all ones with X >= 1; with X = 0 it is
    // (2^Y - 1) quanta = 1.1...1b (Y - 1 ones) * 2^(max_exp - 127)
    if (X >= 1)
      bc->sat_mant = (uint32_t)(((1ull << Y) - 1ull) << (23 - Y));
    else
      bc->sat_mant = Y >= 1 ? (uint32_t)(((1ull << (Y - 1)) - 1ull) << (24 - Y)) : 0u;
    bc->sat_mask = (X == 0 && Y == 0) ? 0u : 0xFFFFFFFFu;
    bc->bias_shift = (uint32_t)((Y + L) & 31);
    bc->bias_mask = (Y + L) >= 32 ? 0u : 0xFFFFFFFFu;
    bc->wide_above = (uint32_t)(231 + Y - (X == 0 ? 1 : 0));  // largest clamped exponent is max_exp (+1 for X = 0)
    // mantissa bits of the top binade: Y, or Y - 1 for X = 0 (see sat_mant)
    const int top_bits = X >= 1 ? Y : (Y >= 1 ? Y - 1 : 0);
    bc->round_half = bc->round_shift = bc->round_odd = 0;
    if (after_rounding && top_bits == 0) {
      bc->round_half = 1u << 22;  // the kept significand is the leading one, always odd: a tie goes up
    } else if (after_rounding && top_bits < 23) {
      bc->round_half = (1u << (22 - top_bits)) - 1u;
      bc->round_shift = (uint32_t)(23 - top_bits);
      bc->round_odd = 1u;
    }
  }
  return EXMY_OK;
}

exmy_status_t make_int_format(exmy_dtype_t dt, int Y, int max_exp, bool packed, IntConsts* ic) {
  if (dt != EXMY_F32 && dt != EXMY_BF16 && dt != EXMY_F16) return EXMY_ERR_FORMAT;
  const int P = dt == EXMY_F32 ? 23 : (dt == EXMY_F16 ? 10 : 7);
  // at least one magnitude bit; the container's significand holds Y + 1 bits (as for e0mY); the packed
  // form stops at 16 bits; the single fp32 rounding addend needs Y <= 21
  if (Y < 1 || Y > P + 1 || Y > 21 || (packed && 1 + Y > kBlockWidth)) return EXMY_ERR_FORMAT;
  if (max_exp < 0 || max_exp > 253) return EXMY_ERR_MAX_EXP;
  if (Y == P + 1 && max_exp < 1) return EXMY_ERR_MAX_EXP;  // the quantum must be a value of the container
  const int emin8 = max_exp + 1;
  if (emin8 + 23 - Y > 254) return EXMY_ERR_MAX_EXP;  // the rounding addend must be a finite float
  // inside fp16 the quantum must be at least 2^-24 and -2^Y quanta = -2^(max_exp - 126) at most 2^15 in magnitude
  if (dt == EXMY_F16 && (max_exp > 141 || emin8 - 127 - Y < -24)) return EXMY_ERR_MAX_EXP;
  if (ic) {
    ic->sat_pos_bits = float_bits(ldexpf((float)((1u << Y) - 1u), emin8 - 127 - Y));
    ic->neg_extra = float_bits(ldexpf(1.0f, emin8 - 127)) - ic->sat_pos_bits;
    ic->left_shift = (uint32_t)(31 - Y);
    ic->magic = ldexpf(1.0f, emin8 - 127 + 23 - Y);
    ic->quantum = ldexpf(1.0f, emin8 - 127 - Y);
  }
  return EXMY_OK;
}

}  // namespace exmy

using namespace exmy;

namespace {

enum class Op { kEncode, kDecode };

// Validate every tensor of a batch, then launch it in pieces of at most kMaxBatch
// tensors whose chunk counts are alike (a launch's grid is as wide as its largest
// tensor, so very different sizes do not share one).  Nothing is launched if any
// tensor fails validation.
exmy_status_t run_batch(Op op, const exmy_tensor_t* tensors, size_t count, exmy_dtype_t dt, int X, int Y,
                        uint64_t* hist, bool with_hist, void* stream) {
  if (count == 0) return exmy_check_format(dt, X, Y, X == 8 ? 255 : (X == 0 ? 1 : 254), 1);
  if (!tensors) return EXMY_ERR_NULL;
  FormatConsts fc;
  bool any_wide = false;
  for (size_t i = 0; i < count; ++i) {
    const exmy_tensor_t& t = tensors[i];
    bool wide = false;
    if (exmy_status_t st = make_format(dt, X, Y, t.max_exp, kFlatWidth, &fc, nullptr, &wide)) return st;
    any_wide = any_wide || wide;
    if (t.n > EXMY_MAX_ELEMENTS) return EXMY_ERR_COUNT;
    if (t.n == 0) continue;
    if (!t.src || !t.dst) return EXMY_ERR_NULL;
    if (!aligned16(t.src) || !aligned16(t.dst)) return EXMY_ERR_ALIGN;
  }
  if (with_hist) {
    if (!hist) return EXMY_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(hist) & 7u) return EXMY_ERR_ALIGN;
  }

  const int W = 1 + X + Y;
  BatchArgs args;
  args.fc = fc;
  args.hist = reinterpret_cast<unsigned long long*>(hist);
  args.count = 0;
  uint64_t hi = 0;  // largest element count in the pending launch
  auto flush = [&]() -> hipError_t {
    if (args.count == 0) return hipSuccess;
    const hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e;
    if (W == 32) {  // e8m23: no planes to form; a histogram asked for alongside takes its own pass
      e = codes32_dispatch(op == Op::kDecode, args, hi, s);
      for (int k = 0; with_hist && e == hipSuccess && k < args.count; ++k)
        e = histogram_dispatch(dt, args.t[k].src, args.t[k].n, hist, s);
    } else {
      e = op == Op::kEncode ? encode_dispatch(dt, W, any_wide, with_hist, args, hi, s)
                            : decode_dispatch(dt, W, X == 8, args, hi, s);
    }
    args.count = 0;
    return e;
  };
  // Tensors are independent, so they may be launched in any order: walk them by size
  // (stable, so equal sizes keep their memory order) and cut a launch when it is full
  // or when more than a quarter of its blocks would fall off the end of a tensor.
  std::vector<uint32_t> order;
  order.reserve(count);
  for (size_t i = 0; i < count; ++i)
    if (tensors[i].n) order.push_back((uint32_t)i);
  std::stable_sort(order.begin(), order.end(),
                   [&](uint32_t a, uint32_t b) { return tensors[a].n > tensors[b].n; });
  for (uint32_t i : order) {
    const exmy_tensor_t& t = tensors[i];
    if (args.count == kMaxBatch || (args.count && t.n < hi - hi / 4)) {
      if (flush() != hipSuccess) return EXMY_ERR_DEVICE;
    }
    if (args.count == 0) hi = t.n;  // sizes only shrink from here
    TensorArgs& ta = args.t[args.count++];
    ta.src = t.src;
    ta.dst = t.dst;
    ta.n = t.n;
    make_format(dt, X, Y, t.max_exp, kFlatWidth, nullptr, &ta.tc, nullptr);
  }
  return flush() == hipSuccess ? EXMY_OK : EXMY_ERR_DEVICE;
}

// kMaxExpOfFormat: the "before rounding" maximum brought into the range valid for (X, Y), not only for X
enum class BlockOp { kMaxExp, kMaxExpOfFormat, kMaxExpRounded, kScale, kEncode, kDecode, kEmulate, kAutoEncode, kAutoEncodeRounded };

// Shared validation and launch of the per-block entry points.  `elems` is the
// bf16 / fp32 side, `packed` the plane side (encode and decode only); `side` is
// the per-block array: metadata bytes, or scales of type `scale_dt` when `scaled` is set.
exmy_status_t run_blocks(BlockOp op, bool scaled, const void* elems, const void* packed, exmy_dtype_t dt, uint64_t n,
                         uint64_t block, int X, int Y, const void* side, void* stream,
                         exmy_dtype_t scale_dt = EXMY_F32) {
  BlockArgs args;
  if (scaled && scale_dt != EXMY_F32 && scale_dt != EXMY_BF16) return EXMY_ERR_FORMAT;
  const bool is_auto = op == BlockOp::kAutoEncode || op == BlockOp::kAutoEncodeRounded;
  const bool is_packed = op == BlockOp::kEncode || op == BlockOp::kDecode || is_auto;
  const bool rounded = op == BlockOp::kMaxExpRounded || op == BlockOp::kAutoEncodeRounded;
  if (exmy_status_t st = make_block_format(dt, X, Y, is_packed ? kBlockWidth : kAnyWidth, rounded,
                                           op != BlockOp::kMaxExp, &args.fc, &args.bc))
    return st;
  bool wide_format = Y > 21;
  args.vmax127 = 0.0f;
  if (scaled) {
    // codes of the max_exp = 127 format; a format whose only magnitude is 0 has nothing to scale
    if (X == 0 && Y == 0) return EXMY_ERR_FORMAT;
    if (exmy_status_t st = make_format(dt, X, Y, 127, is_packed ? kBlockWidth : kAnyWidth, nullptr, &args.tc127,
                                       &wide_format)) return st;
    uint32_t sat = args.tc127.sat_bits;
    memcpy(&args.vmax127, &sat, 4);
  }
  // the fp32 form of the scaled rounding needs every rounding boundary above the fp32 denormals (X <= 6)
  // and a quantum wider than the uncertainty of the fp32 quotient (Y <= 17)
  args.scaled_f64 = (scaled && (X == 7 || Y > 17 || wide_format)) ? 1u : 0u;
  if (block < 8 || block % 8 || block > EXMY_MAX_BLOCK) return EXMY_ERR_BLOCK;
  if (n > EXMY_MAX_ELEMENTS) return EXMY_ERR_COUNT;
  if (n == 0) return EXMY_OK;
  if (!elems || !side || (is_packed && !packed)) return EXMY_ERR_NULL;
  if (!aligned16(elems) || (is_packed && !aligned16(packed))) return EXMY_ERR_ALIGN;
  if (scaled && (reinterpret_cast<uintptr_t>(side) & (scale_dt == EXMY_F32 ? 3u : 1u))) return EXMY_ERR_ALIGN;

  args.n = n;
  args.n_blocks = (n + block - 1) / block;
  args.block_groups = (uint32_t)(block / 8);
  args.bi = make_block_index(args.block_groups);  // dispatchers rescale it to their kernel's units
  args.meta = scaled ? nullptr : static_cast<uint8_t*>(const_cast<void*>(side));
  args.scale = scaled ? const_cast<void*>(side) : nullptr;
  args.scale_log2_bytes = scale_dt == EXMY_F32 ? 2u : 1u;
  const hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = hipSuccess;
  switch (op) {
    case BlockOp::kMaxExp:
    case BlockOp::kMaxExpOfFormat:
    case BlockOp::kMaxExpRounded:
    case BlockOp::kScale:
      args.src = elems;
      args.dst = nullptr;
      e = block_max_exp_dispatch(dt, args, scaled, s);
      break;
    case BlockOp::kEncode:
      args.src = elems;
      args.dst = const_cast<void*>(packed);
      e = encode_blocks_dispatch(dt, 1 + X + Y, args, scaled, s);
      break;
    case BlockOp::kAutoEncode:
    case BlockOp::kAutoEncodeRounded:
      args.src = elems;
      args.dst = const_cast<void*>(packed);
      e = encode_blocks_auto_dispatch(dt, 1 + X + Y, args, s);
      break;
    case BlockOp::kDecode:
      args.src = packed;
      args.dst = const_cast<void*>(elems);
      e = decode_blocks_dispatch(dt, 1 + X + Y, args, scaled, s);
      break;
    case BlockOp::kEmulate:
      args.src = elems;
      args.dst = nullptr;
      e = emulate_blocks_dispatch(dt, args, wide_format, scaled, s);
      break;
  }
  return e == hipSuccess ? EXMY_OK : EXMY_ERR_DEVICE;
}

// Shared validation and launch of the entry points for blocks that are columns or
// 2-D tiles.  `matrix` is the bf16 / fp16 / fp32 side, `packed` the plane side.
exmy_status_t run_tiles(BlockOp op, const void* matrix, const void* packed, exmy_dtype_t dt, uint64_t rows,
                        uint64_t cols, uint64_t tile_rows, uint64_t tile_cols, int X, int Y, const uint8_t* meta,
                        void* stream) {
  TileArgs args;
  const bool is_packed = op == BlockOp::kEncode || op == BlockOp::kDecode;
  if (exmy_status_t st = make_block_format(dt, X, Y, is_packed ? kBlockWidth : kAnyWidth, op == BlockOp::kMaxExpRounded,
                                           op != BlockOp::kMaxExp, &args.fc, &args.bc))
    return st;
  if (cols % 8 || cols > EXMY_MAX_COLS || rows > EXMY_MAX_ROWS) return EXMY_ERR_SHAPE;
  if (tile_rows == 0 || tile_cols == 0 || (tile_cols != 1 && tile_cols % 8 && tile_cols < cols)) return EXMY_ERR_BLOCK;
  if (rows * cols > EXMY_MAX_ELEMENTS) return EXMY_ERR_COUNT;
  if (rows == 0 || cols == 0) return EXMY_OK;
  if (!matrix || !meta || (is_packed && !packed)) return EXMY_ERR_NULL;
  tile_rows = tile_rows < rows ? tile_rows : rows;
  tile_cols = tile_cols < cols ? tile_cols : cols;
  // Tiles that are runs of consecutive elements (whole rows, or parts that divide a row) are the blocks of
  // the flat entry points.
  const uint64_t run = tile_cols == cols ? tile_rows * cols : (tile_rows == 1 && cols % tile_cols == 0 ? tile_cols : 0);
  if (run >= 8 && run % 8 == 0 && run <= EXMY_MAX_BLOCK)
    return run_blocks(op, false, matrix, packed, dt, rows * cols, run, X, Y, meta, stream);
  if (!aligned16(matrix) || !aligned16(meta) || (is_packed && !aligned16(packed))) return EXMY_ERR_ALIGN;

  args.rows = rows;
  args.cols = cols;
  args.tile_rows = tile_rows;
  args.tile_cols = tile_cols;
  args.tiles_along_row = (cols + tile_cols - 1) / tile_cols;
  args.meta = const_cast<uint8_t*>(meta);
  const hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = hipSuccess;
  switch (op) {
    case BlockOp::kMaxExp:
    case BlockOp::kMaxExpRounded:
      args.src = matrix;
      args.dst = nullptr;
      e = tile_max_exp_dispatch(dt, args, s);
      break;
    case BlockOp::kEncode:
      args.src = matrix;
      args.dst = const_cast<void*>(packed);
      e = encode_tiles_dispatch(dt, 1 + X + Y, args, s);
      break;
    case BlockOp::kDecode:
      args.src = packed;
      args.dst = const_cast<void*>(matrix);
      e = decode_tiles_dispatch(dt, 1 + X + Y, args, s);
      break;
    case BlockOp::kEmulate:
      args.src = matrix;
      args.dst = nullptr;
      e = emulate_tiles_dispatch(dt, args, Y > 21, s);
      break;
    default:
      return EXMY_ERR_FORMAT;
  }
  return e == hipSuccess ? EXMY_OK : EXMY_ERR_DEVICE;
}

enum class RowsOp { kEncode, kDecode };

// Shared validation and launch of the entry points that pack along rows.
exmy_status_t run_rows(RowsOp op, const void* matrix, const void* packed, exmy_dtype_t dt, uint64_t rows, uint64_t cols,
                       int X, int Y, int max_exp, const uint8_t* max_exp_rows, void* stream) {
  RowsArgs args;
  bool wide = false;
  if (max_exp_rows) {
    if (exmy_status_t st = make_block_format(dt, X, Y, kBlockWidth, false, true, &args.fc, &args.bc)) return st;
    memset(&args.tc, 0, sizeof(args.tc));
  } else {
    if (exmy_status_t st = make_format(dt, X, Y, max_exp, kBlockWidth, &args.fc, &args.tc, &wide)) return st;
    memset(&args.bc, 0, sizeof(args.bc));
  }
  if (cols % 8 || cols > EXMY_MAX_COLS) return EXMY_ERR_SHAPE;
  if (cols && rows > EXMY_MAX_ELEMENTS / cols) return EXMY_ERR_COUNT;
  if (rows == 0 || cols == 0) return EXMY_OK;
  if (!matrix || !packed) return EXMY_ERR_NULL;
  if (!aligned16(matrix) || !aligned16(packed)) return EXMY_ERR_ALIGN;
  args.meta = max_exp_rows;
  args.rows = rows;
  args.cols = (uint32_t)cols;
  args.tiles = make_block_index(1);
  const hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  if (op == RowsOp::kEncode) {
    args.src = matrix;
    args.dst = const_cast<void*>(packed);
    e = encode_rows_dispatch(dt, 1 + X + Y, args, max_exp_rows != nullptr, wide, s);
  } else {
    args.src = packed;
    args.dst = const_cast<void*>(matrix);
    e = decode_rows_dispatch(dt, 1 + X + Y, args, max_exp_rows != nullptr, X == 8, s);
  }
  return e == hipSuccess ? EXMY_OK : EXMY_ERR_DEVICE;
}

}  // namespace

extern "C" {

size_t exmy_packed_bytes(uint64_t n, int X, int Y) { return (size_t)(((n + 7) / 8) * (uint64_t)(1 + X + Y)); }

exmy_status_t exmy_check_format(exmy_dtype_t dt, int X, int Y, int max_exp, int packed) {
  return make_format(dt, X, Y, max_exp, packed ? kFlatWidth : kAnyWidth, nullptr, nullptr, nullptr);
}

exmy_status_t exmy_encode(const void* src, exmy_dtype_t dt, uint64_t n, int X, int Y, int max_exp,
                          void* dst_packed, void* stream) {
  const exmy_tensor_t t = {src, dst_packed, n, max_exp};
  return run_batch(Op::kEncode, &t, 1, dt, X, Y, nullptr, false, stream);
}

exmy_status_t exmy_encode_with_histogram(const void* src, exmy_dtype_t dt, uint64_t n, int X, int Y, int max_exp,
                                         void* dst_packed, uint64_t* hist256_dev, void* stream) {
  const exmy_tensor_t t = {src, dst_packed, n, max_exp};
  return run_batch(Op::kEncode, &t, 1, dt, X, Y, hist256_dev, true, stream);
}

exmy_status_t exmy_decode(const void* src_packed, exmy_dtype_t dt_out, uint64_t n, int X, int Y, int max_exp,
                          void* dst, void* stream) {
  const exmy_tensor_t t = {src_packed, dst, n, max_exp};
  return run_batch(Op::kDecode, &t, 1, dt_out, X, Y, nullptr, false, stream);
}

exmy_status_t exmy_encode_batch(const exmy_tensor_t* tensors, size_t count, exmy_dtype_t dt, int X, int Y,
                                void* stream) {
  return run_batch(Op::kEncode, tensors, count, dt, X, Y, nullptr, false, stream);
}

exmy_status_t exmy_decode_batch(const exmy_tensor_t* tensors, size_t count, exmy_dtype_t dt_out, int X, int Y,
                                void* stream) {
  return run_batch(Op::kDecode, tensors, count, dt_out, X, Y, nullptr, false, stream);
}

exmy_status_t exmy_emulate(void* data_inout, exmy_dtype_t dt, uint64_t n, int X, int Y, int max_exp, void* stream) {
  FormatConsts fc;
  TensorConsts tc;
  bool wide = false;
  if (exmy_status_t st = make_format(dt, X, Y, max_exp, kAnyWidth, &fc, &tc, &wide)) return st;
  if (n > EXMY_MAX_ELEMENTS) return EXMY_ERR_COUNT;
  if (n == 0) return EXMY_OK;
  if (!data_inout) return EXMY_ERR_NULL;
  if (!aligned16(data_inout)) return EXMY_ERR_ALIGN;
  const hipError_t e = emulate_dispatch(dt, wide, data_inout, n, fc, tc, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? EXMY_OK : EXMY_ERR_DEVICE;
}

exmy_status_t exmy_exponent_histogram(const void* src, exmy_dtype_t dt, uint64_t n, uint64_t* hist256_dev,
                                      void* stream) {
  if (dt != EXMY_F32 && dt != EXMY_BF16 && dt != EXMY_F16) return EXMY_ERR_FORMAT;
  if (n > EXMY_MAX_ELEMENTS) return EXMY_ERR_COUNT;
  if (!hist256_dev) return EXMY_ERR_NULL;
  if (n == 0) return EXMY_OK;
  if (!src) return EXMY_ERR_NULL;
  if (!aligned16(src) || (reinterpret_cast<uintptr_t>(hist256_dev) & 7u)) return EXMY_ERR_ALIGN;
  const hipError_t e = histogram_dispatch(dt, src, n, hist256_dev, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? EXMY_OK : EXMY_ERR_DEVICE;
}

namespace {
exmy_status_t run_records(bool decode, const void* src, void* dst, exmy_dtype_t dt, uint64_t n, int X, int Y,
                          int max_exp, void* stream) {
  FormatConsts fc;
  TensorConsts tc;
  bool wide = false;
  if (exmy_status_t st = make_format(dt, X, Y, max_exp, kBlockWidth, &fc, &tc, &wide)) return st;
  if (n > EXMY_MAX_ELEMENTS) return EXMY_ERR_COUNT;
  if (n == 0) return EXMY_OK;
  if (!src || !dst) return EXMY_ERR_NULL;
  if (!aligned16(src) || !aligned16(dst)) return EXMY_ERR_ALIGN;
  const int W = 1 + X + Y;
  if (W == 8 || W == 16)  // one plane: the records are the planar form
    return decode ? exmy_decode(src, dt, n, X, Y, max_exp, dst, stream) : exmy_encode(src, dt, n, X, Y, max_exp, dst, stream);
  const hipError_t e = records_dispatch(dt, W, decode, decode ? X == 8 : wide, src, dst, n, fc, tc,
                                        static_cast<hipStream_t>(stream));
  return e == hipSuccess ? EXMY_OK : EXMY_ERR_DEVICE;
}
}  // namespace

exmy_status_t exmy_encode_records(const void* src, exmy_dtype_t dt, uint64_t n, int X, int Y, int max_exp,
                                  void* dst_records, void* stream) {
  return run_records(false, src, dst_records, dt, n, X, Y, max_exp, stream);
}

exmy_status_t exmy_decode_records(const void* src_records, exmy_dtype_t dt_out, uint64_t n, int X, int Y, int max_exp,
                                  void* dst, void* stream) {
  return run_records(true, src_records, dst, dt_out, n, X, Y, max_exp, stream);
}

namespace {
// op: 0 = encode, 1 = decode, 2 = emulate in place (src == dst)
exmy_status_t run_specials(int op, const void* src, void* dst, exmy_dtype_t dt, uint64_t n, int X, int Y, int max_exp,
                           exmy_specials_t specials, void* stream) {
  if (specials != EXMY_SPECIALS_IEEE && specials != EXMY_SPECIALS_NAN_ONLY) return EXMY_ERR_FORMAT;
  FormatConsts fc;
  TensorConsts tc;
  bool wide = false;
  if (exmy_status_t st = make_format(dt, X, Y, max_exp, op == 2 ? kAnyWidth : kBlockWidth, &fc, &tc, &wide)) return st;
  if (specials == EXMY_SPECIALS_IEEE ? X < 1 : (X == 8 || X + Y < 1)) return EXMY_ERR_FORMAT;
  if (n > EXMY_MAX_ELEMENTS) return EXMY_ERR_COUNT;
  if (n == 0) return EXMY_OK;
  if (!src || !dst) return EXMY_ERR_NULL;
  if (!aligned16(src) || !aligned16(dst)) return EXMY_ERR_ALIGN;

  // the largest finite magnitude code and its value, which becomes the saturation bound
  const uint64_t top = (1ull << X) - 1ull, ones = (1ull << Y) - 1ull, all_ones = (1ull << (X + Y)) - 1ull;
  const uint64_t last = specials == EXMY_SPECIALS_IEEE ? (top << Y) - 1ull : all_ones - 1ull;
  const int emin8 = max_exp - (1 << X) + 2;
  const uint64_t E = last >> Y, M = last & ones;
  tc.sat_bits = E == 0 ? float_bits(ldexpf((float)M, emin8 - 127 - Y))
                       : (uint32_t)(((E - 1 + (uint64_t)emin8) << 23) | (M << (23 - Y)));
  const hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  if (op == 2) {
    e = emulate_dispatch(dt, wide, dst, n, fc, tc, s);  // Inf / NaN pass through; only the bound differs
  } else {
    const uint64_t inf = specials == EXMY_SPECIALS_IEEE ? top << Y : last;
    SpecialConsts sc;
    sc.nan_left = (uint32_t)(all_ones << fc.left_shift);
    sc.inf_left = (uint32_t)(inf << fc.left_shift);
    sc.g_last = (uint32_t)(last << (23 - Y)) + tc.dec_bias;
    sc.g_inf = specials == EXMY_SPECIALS_IEEE ? (uint32_t)(inf << (23 - Y)) + tc.dec_bias : 0xFFFFFFFFu;
    e = specials_dispatch(dt, 1 + X + Y, op == 1, wide, src, dst, n, fc, tc, sc, s);
  }
  return e == hipSuccess ? EXMY_OK : EXMY_ERR_DEVICE;
}
}  // namespace

exmy_status_t exmy_encode_specials(const void* src, exmy_dtype_t dt, uint64_t n, int X, int Y, int max_exp,
                                   exmy_specials_t specials, void* dst_packed, void* stream) {
  return run_specials(0, src, dst_packed, dt, n, X, Y, max_exp, specials, stream);
}

exmy_status_t exmy_decode_specials(const void* src_packed, exmy_dtype_t dt_out, uint64_t n, int X, int Y, int max_exp,
                                   exmy_specials_t specials, void* dst, void* stream) {
  return run_specials(1, src_packed, dst, dt_out, n, X, Y, max_exp, specials, stream);
}

exmy_status_t exmy_emulate_specials(void* data_inout, exmy_dtype_t dt, uint64_t n, int X, int Y, int max_exp,
                                    exmy_specials_t specials, void* stream) {
  return run_specials(2, data_inout, data_inout, dt, n, X, Y, max_exp, specials, stream);
}

size_t exmy_block_count(uint64_t n, uint64_t block) { return block ? (size_t)((n + block - 1) / block) : 0; }

size_t exmy_tile_count(uint64_t rows, uint64_t cols, uint64_t tile_rows, uint64_t tile_cols) {
  if (!tile_rows || !tile_cols) return 0;
  return (size_t)(((rows + tile_rows - 1) / tile_rows) * ((cols + tile_cols - 1) / tile_cols));
}

exmy_status_t exmy_tile_max_exp(const void* src, exmy_dtype_t dt, uint64_t rows, uint64_t cols, uint64_t tile_rows,
                                uint64_t tile_cols, int X, int Y, exmy_scheme_t scheme, uint8_t* max_exp_dev,
                                void* stream) {
  if (scheme != EXMY_MAX_EXP_BEFORE_ROUNDING && scheme != EXMY_MAX_EXP_AFTER_ROUNDING) return EXMY_ERR_FORMAT;
  const bool rounded = scheme == EXMY_MAX_EXP_AFTER_ROUNDING;
  return run_tiles(rounded ? BlockOp::kMaxExpRounded : BlockOp::kMaxExp, src, nullptr, dt, rows, cols, tile_rows,
                   tile_cols, X, rounded ? Y : 0, max_exp_dev, stream);
}

exmy_status_t exmy_encode_tiles(const void* src, exmy_dtype_t dt, uint64_t rows, uint64_t cols, uint64_t tile_rows,
                                uint64_t tile_cols, int X, int Y, const uint8_t* max_exp_dev, void* dst_packed,
                                void* stream) {
  return run_tiles(BlockOp::kEncode, src, dst_packed, dt, rows, cols, tile_rows, tile_cols, X, Y, max_exp_dev, stream);
}

exmy_status_t exmy_decode_tiles(const void* src_packed, exmy_dtype_t dt_out, uint64_t rows, uint64_t cols,
                                uint64_t tile_rows, uint64_t tile_cols, int X, int Y, const uint8_t* max_exp_dev,
                                void* dst, void* stream) {
  return run_tiles(BlockOp::kDecode, dst, src_packed, dt_out, rows, cols, tile_rows, tile_cols, X, Y, max_exp_dev, stream);
}

exmy_status_t exmy_emulate_tiles(void* data_inout, exmy_dtype_t dt, uint64_t rows, uint64_t cols, uint64_t tile_rows,
                                 uint64_t tile_cols, int X, int Y, const uint8_t* max_exp_dev, void* stream) {
  return run_tiles(BlockOp::kEmulate, data_inout, nullptr, dt, rows, cols, tile_rows, tile_cols, X, Y, max_exp_dev, stream);
}

exmy_status_t exmy_block_max_exp(const void* src, exmy_dtype_t dt, uint64_t n, uint64_t block, int X,
                                 uint8_t* max_exp_dev, void* stream) {
  return run_blocks(BlockOp::kMaxExp, false, src, nullptr, dt, n, block, X, 0, max_exp_dev, stream);
}

exmy_status_t exmy_block_max_exp_after_rounding(const void* src, exmy_dtype_t dt, uint64_t n, uint64_t block, int X,
                                                int Y, uint8_t* max_exp_dev, void* stream) {
  return run_blocks(BlockOp::kMaxExpRounded, false, src, nullptr, dt, n, block, X, Y, max_exp_dev, stream);
}

exmy_status_t exmy_encode_blocks_auto(const void* src, exmy_dtype_t dt, uint64_t n, uint64_t block, int X, int Y,
                                      exmy_scheme_t scheme, uint8_t* max_exp_dev, void* dst_packed, void* stream) {
  if (scheme != EXMY_MAX_EXP_BEFORE_ROUNDING && scheme != EXMY_MAX_EXP_AFTER_ROUNDING) return EXMY_ERR_FORMAT;
  // validate the second launch before the first, so that an error leaves both outputs untouched
  if (exmy_status_t st = make_block_format(dt, X, Y, kBlockWidth, false, true, nullptr, nullptr)) return st;
  if (n && !dst_packed) return EXMY_ERR_NULL;
  if (n && !aligned16(dst_packed)) return EXMY_ERR_ALIGN;
  const bool rounded = scheme == EXMY_MAX_EXP_AFTER_ROUNDING;
  if (block >= 8 && block % 8 == 0 && block <= EXMY_MAX_BLOCK && encode_blocks_auto_fits(dt, (uint32_t)(block / 8)))
    return run_blocks(rounded ? BlockOp::kAutoEncodeRounded : BlockOp::kAutoEncode, false, src, dst_packed, dt, n, block, X,
                      Y, max_exp_dev, stream);  // one pass: the block stays in registers
  const BlockOp op = rounded ? BlockOp::kMaxExpRounded : BlockOp::kMaxExpOfFormat;
  if (exmy_status_t st = run_blocks(op, false, src, nullptr, dt, n, block, X, Y, max_exp_dev, stream)) return st;
  return run_blocks(BlockOp::kEncode, false, src, dst_packed, dt, n, block, X, Y, max_exp_dev, stream);
}

exmy_status_t exmy_encode_blocks(const void* src, exmy_dtype_t dt, uint64_t n, uint64_t block, int X, int Y,
                                 const uint8_t* max_exp_dev, void* dst_packed, void* stream) {
  return run_blocks(BlockOp::kEncode, false, src, dst_packed, dt, n, block, X, Y, max_exp_dev, stream);
}

exmy_status_t exmy_decode_blocks(const void* src_packed, exmy_dtype_t dt_out, uint64_t n, uint64_t block, int X, int Y,
                                 const uint8_t* max_exp_dev, void* dst, void* stream) {
  return run_blocks(BlockOp::kDecode, false, dst, src_packed, dt_out, n, block, X, Y, max_exp_dev, stream);
}

exmy_status_t exmy_emulate_blocks(void* data_inout, exmy_dtype_t dt, uint64_t n, uint64_t block, int X, int Y,
                                  const uint8_t* max_exp_dev, void* stream) {
  return run_blocks(BlockOp::kEmulate, false, data_inout, nullptr, dt, n, block, X, Y, max_exp_dev, stream);
}

exmy_status_t exmy_block_scale(const void* src, exmy_dtype_t dt, uint64_t n, uint64_t block, int X, int Y,
                               void* scale_dev, exmy_dtype_t scale_dt, void* stream) {
  return run_blocks(BlockOp::kScale, true, src, nullptr, dt, n, block, X, Y, scale_dev, stream, scale_dt);
}

exmy_status_t exmy_encode_scaled(const void* src, exmy_dtype_t dt, uint64_t n, uint64_t block, int X, int Y,
                                 const void* scale_dev, exmy_dtype_t scale_dt, void* dst_packed, void* stream) {
  return run_blocks(BlockOp::kEncode, true, src, dst_packed, dt, n, block, X, Y, scale_dev, stream, scale_dt);
}

exmy_status_t exmy_decode_scaled(const void* src_packed, exmy_dtype_t dt_out, uint64_t n, uint64_t block, int X, int Y,
                                 const void* scale_dev, exmy_dtype_t scale_dt, void* dst, void* stream) {
  return run_blocks(BlockOp::kDecode, true, dst, src_packed, dt_out, n, block, X, Y, scale_dev, stream, scale_dt);
}

exmy_status_t exmy_emulate_scaled(void* data_inout, exmy_dtype_t dt, uint64_t n, uint64_t block, int X, int Y,
                                  const void* scale_dev, exmy_dtype_t scale_dt, void* stream) {
  return run_blocks(BlockOp::kEmulate, true, data_inout, nullptr, dt, n, block, X, Y, scale_dev, stream, scale_dt);
}

size_t exmy_packed_bytes_rows(uint64_t rows, uint64_t cols, int X, int Y) {
  return (size_t)(((rows + 7) / 8) * cols * (uint64_t)(1 + X + Y));
}

exmy_status_t exmy_encode_rows(const void* src, exmy_dtype_t dt, uint64_t rows, uint64_t cols, int X, int Y,
                               int max_exp, const uint8_t* max_exp_rows_dev, void* dst_packed, void* stream) {
  return run_rows(RowsOp::kEncode, src, dst_packed, dt, rows, cols, X, Y, max_exp, max_exp_rows_dev, stream);
}

exmy_status_t exmy_decode_rows(const void* src_packed, exmy_dtype_t dt_out, uint64_t rows, uint64_t cols, int X, int Y,
                               int max_exp, const uint8_t* max_exp_rows_dev, void* dst, void* stream) {
  return run_rows(RowsOp::kDecode, dst, src_packed, dt_out, rows, cols, X, Y, max_exp, max_exp_rows_dev, stream);
}

exmy_status_t exmy_encode_int(const void* src, exmy_dtype_t dt, uint64_t n, int Y, int max_exp, void* dst_packed,
                              void* stream) {
  IntConsts ic;
  if (exmy_status_t st = make_int_format(dt, Y, max_exp, true, &ic)) return st;
  if (n > EXMY_MAX_ELEMENTS) return EXMY_ERR_COUNT;
  if (n == 0) return EXMY_OK;
  if (!src || !dst_packed) return EXMY_ERR_NULL;
  if (!aligned16(src) || !aligned16(dst_packed)) return EXMY_ERR_ALIGN;
  const hipError_t e = encode_int_dispatch(dt, 1 + Y, src, dst_packed, n, ic, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? EXMY_OK : EXMY_ERR_DEVICE;
}

exmy_status_t exmy_decode_int(const void* src_packed, exmy_dtype_t dt_out, uint64_t n, int Y, int max_exp, void* dst,
                              void* stream) {
  IntConsts ic;
  if (exmy_status_t st = make_int_format(dt_out, Y, max_exp, true, &ic)) return st;
  if (n > EXMY_MAX_ELEMENTS) return EXMY_ERR_COUNT;
  if (n == 0) return EXMY_OK;
  if (!src_packed || !dst) return EXMY_ERR_NULL;
  if (!aligned16(src_packed) || !aligned16(dst)) return EXMY_ERR_ALIGN;
  const hipError_t e = decode_int_dispatch(dt_out, 1 + Y, src_packed, dst, n, ic, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? EXMY_OK : EXMY_ERR_DEVICE;
}

exmy_status_t exmy_emulate_int(void* data_inout, exmy_dtype_t dt, uint64_t n, int Y, int max_exp, void* stream) {
  IntConsts ic;
  if (exmy_status_t st = make_int_format(dt, Y, max_exp, false, &ic)) return st;
  if (n > EXMY_MAX_ELEMENTS) return EXMY_ERR_COUNT;
  if (n == 0) return EXMY_OK;
  if (!data_inout) return EXMY_ERR_NULL;
  if (!aligned16(data_inout)) return EXMY_ERR_ALIGN;
  const hipError_t e = emulate_int_dispatch(dt, data_inout, n, ic, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? EXMY_OK : EXMY_ERR_DEVICE;
}

int exmy_max_exp_from_histogram(const uint64_t* hist256_host, double coverage) {
  if (!hist256_host) return -1;
  uint64_t finite = 0;
  for (int e = 0; e <= 254; ++e) finite += hist256_host[e];
  if (finite == 0) return -1;
  const double need = coverage * (double)finite;
  uint64_t seen = 0;
  for (int e = 0; e <= 254; ++e) {
    seen += hist256_host[e];
    if ((double)seen >= need) return e;
  }
  return 254;
}

const char* exmy_status_string(exmy_status_t status) {
  switch (status) {
    case EXMY_OK: return "ok";
    case EXMY_ERR_NULL: return "null pointer";
    case EXMY_ERR_FORMAT: return "format (X, Y, width or dtype) not supported";
    case EXMY_ERR_MAX_EXP: return "max_exp out of range for this X";
    case EXMY_ERR_COUNT: return "element count too large";
    case EXMY_ERR_ALIGN: return "pointer not 16-byte aligned";
    case EXMY_ERR_DEVICE: return "HIP launch error";
    case EXMY_ERR_SHAPE: return "column count not a multiple of 8, or above 2^26";
    case EXMY_ERR_BLOCK: return "block size not a multiple of 8 in [8, 2^31]";
  }
  return "unknown status";
}

}  // extern "C"
