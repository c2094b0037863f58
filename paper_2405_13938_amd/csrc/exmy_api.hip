// C ABI of the eXmY codec: host-side validation, derivation of the wave-uniform
// format constants, and dispatch to the gfx950 kernels.  Declared and documented
// in include/exmy.h.
#include <math.h>
#include <string.h>

#include <atomic>

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

exmy_status_t make_format(exmy_dtype_t dt, int X, int Y, int max_exp, bool packed, FormatConsts* fc,
                          bool* needs_wide) {
  if (dt != EXMY_F32 && dt != EXMY_BF16) return EXMY_ERR_FORMAT;
  if (X < 0 || X > 8 || Y < 0) return EXMY_ERR_FORMAT;
  // Section 2.1: bf16 holds Y <= 7, fp32 Y <= 23; a sign-magnitude format (X = 0) has
  // no leading one, so its Y bits need only Y significant bits of the container.
  const int P = dt == EXMY_F32 ? 23 : 7;
  if (Y > (X >= 1 ? P : P + 1)) return EXMY_ERR_FORMAT;
  if (packed && 1 + X + Y > 16) return EXMY_ERR_FORMAT;
  if (X == 8) {
    if (max_exp != 255) return EXMY_ERR_MAX_EXP;
  } else if (X == 0) {
    if (max_exp < 0 || max_exp > 253) return EXMY_ERR_MAX_EXP;
    if (Y == P + 1 && max_exp < 1) return EXMY_ERR_MAX_EXP;  // quantum below the container's
  } else {
    if (max_exp < (1 << X) - 1 || max_exp > 254) return EXMY_ERR_MAX_EXP;
  }
  if (!fc) return EXMY_OK;

  const int emin8 = max_exp - (1 << X) + 2;
  const uint32_t ones_y = (1u << Y) - 1u;
  memset(fc, 0, sizeof(*fc));
  fc->xy = (uint32_t)(X + Y);
  fc->y = (uint32_t)Y;
  fc->mag_mask = (uint32_t)((1ull << (X + Y)) - 1ull);
  fc->exp_shift = (uint32_t)(23 - Y);  // Y = 24 cannot occur with X >= 1; X = 0, Y = 24 handled below
  fc->emin_bits = (uint32_t)emin8 << 23;
  // Odd widths end in a 1-bit plane that holds exactly the sign: the encoder takes
  // it from the source bits and left-aligns the magnitude alone.
  const int W = 1 + X + Y;
  const int L = ((W & 1) ? 32 : 31) - (X + Y);
  fc->left_shift = (uint32_t)(L & 31);  // L = 32 only for W = 1, where no magnitude bits exist
  fc->exp_lshift = (uint32_t)((L - (23 - Y)) & 31);
  fc->bias_left = (uint32_t)(0ull - ((uint64_t)emin8 << (Y + L)));
  fc->magic_scale = ldexpf(1.0f, 23 - Y);
  fc->wide_exp = 1023 - 127 + 52 - Y;

  // Largest value: (2 - 2^-Y) * 2^(max_exp-127) with X >= 1 (X = 8: exponent 254, the
  // largest finite float); (2^Y - 1) quanta with X = 0.
  if (X == 0) {
    fc->sat_bits = float_bits(ldexpf((float)ones_y, emin8 - 127 - Y));
  } else {
    const uint32_t top = X == 8 ? 254u : (uint32_t)max_exp;
    fc->sat_bits = (top << 23) | (Y <= 23 ? (ones_y << (23 - Y)) : 0u);
  }
  fc->g_clamp = fc->sat_bits;

  fc->dec_bias = (uint32_t)(emin8 - 1) << 23;
  if (emin8 == 1) {
    fc->fix_mul = 1.0f;
    fc->fix_add = 0.0f;
  } else {
    fc->fix_mul = 2.0f;
    fc->fix_add = -ldexpf(1.0f, emin8 - 127);
  }

  // The fp32 magic addend 2^(ec-127+23-Y) must be finite for the largest clamped
  // exponent ec, and the sum must stay in the addend's binade (Y <= 21).
  const int ec_max = X == 0 ? emin8 : (X == 8 ? 254 : max_exp);
  if (needs_wide) *needs_wide = (ec_max + 23 - Y > 254) || (Y > 21);
  return EXMY_OK;
}

}  // namespace exmy

using namespace exmy;

extern "C" {

size_t exmy_packed_bytes(uint64_t n, int X, int Y) { return (size_t)(((n + 7) / 8) * (uint64_t)(1 + X + Y)); }

exmy_status_t exmy_check_format(exmy_dtype_t dt, int X, int Y, int max_exp, int packed) {
  return make_format(dt, X, Y, max_exp, packed != 0, nullptr, nullptr);
}

static exmy_status_t encode_common(const void* src, exmy_dtype_t dt, uint64_t n, int X, int Y, int max_exp,
                                   void* dst_packed, uint64_t* hist, bool with_hist, void* stream) {
  FormatConsts fc;
  bool wide = false;
  if (exmy_status_t st = make_format(dt, X, Y, max_exp, true, &fc, &wide)) return st;
  if (n > EXMY_MAX_ELEMENTS) return EXMY_ERR_COUNT;
  if (with_hist && !hist) return EXMY_ERR_NULL;
  if (n == 0) return EXMY_OK;
  if (!src || !dst_packed) return EXMY_ERR_NULL;
  if (!aligned16(src) || !aligned16(dst_packed)) return EXMY_ERR_ALIGN;
  if (with_hist && (reinterpret_cast<uintptr_t>(hist) & 7u)) return EXMY_ERR_ALIGN;
  const hipError_t e = encode_dispatch(dt, 1 + X + Y, wide, with_hist, src, dst_packed, n, fc, hist,
                                       static_cast<hipStream_t>(stream));
  return e == hipSuccess ? EXMY_OK : EXMY_ERR_DEVICE;
}

exmy_status_t exmy_encode(const void* src, exmy_dtype_t dt, uint64_t n, int X, int Y, int max_exp,
                          void* dst_packed, void* stream) {
  return encode_common(src, dt, n, X, Y, max_exp, dst_packed, nullptr, false, stream);
}

exmy_status_t exmy_encode_with_histogram(const void* src, exmy_dtype_t dt, uint64_t n, int X, int Y, int max_exp,
                                         void* dst_packed, uint64_t* hist256_dev, void* stream) {
  return encode_common(src, dt, n, X, Y, max_exp, dst_packed, hist256_dev, true, stream);
}

exmy_status_t exmy_decode(const void* src_packed, exmy_dtype_t dt_out, uint64_t n, int X, int Y, int max_exp,
                          void* dst, void* stream) {
  FormatConsts fc;
  if (exmy_status_t st = make_format(dt_out, X, Y, max_exp, true, &fc, nullptr)) return st;
  if (n > EXMY_MAX_ELEMENTS) return EXMY_ERR_COUNT;
  if (n == 0) return EXMY_OK;
  if (!src_packed || !dst) return EXMY_ERR_NULL;
  if (!aligned16(src_packed) || !aligned16(dst)) return EXMY_ERR_ALIGN;
  const hipError_t e = decode_dispatch(dt_out, 1 + X + Y, X == 8, src_packed, dst, n, fc, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? EXMY_OK : EXMY_ERR_DEVICE;
}

exmy_status_t exmy_emulate(void* data_inout, exmy_dtype_t dt, uint64_t n, int X, int Y, int max_exp, void* stream) {
  FormatConsts fc;
  bool wide = false;
  if (exmy_status_t st = make_format(dt, X, Y, max_exp, false, &fc, &wide)) return st;
  if (n > EXMY_MAX_ELEMENTS) return EXMY_ERR_COUNT;
  if (n == 0) return EXMY_OK;
  if (!data_inout) return EXMY_ERR_NULL;
  if (!aligned16(data_inout)) return EXMY_ERR_ALIGN;
  const hipError_t e = emulate_dispatch(dt, wide, data_inout, n, fc, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? EXMY_OK : EXMY_ERR_DEVICE;
}

exmy_status_t exmy_exponent_histogram(const void* src, exmy_dtype_t dt, uint64_t n, uint64_t* hist256_dev,
                                      void* stream) {
  if (dt != EXMY_F32 && dt != EXMY_BF16) return EXMY_ERR_FORMAT;
  if (n > EXMY_MAX_ELEMENTS) return EXMY_ERR_COUNT;
  if (!hist256_dev) return EXMY_ERR_NULL;
  if (n == 0) return EXMY_OK;
  if (!src) return EXMY_ERR_NULL;
  if (!aligned16(src) || (reinterpret_cast<uintptr_t>(hist256_dev) & 7u)) return EXMY_ERR_ALIGN;
  const hipError_t e = histogram_dispatch(dt, src, n, hist256_dev, static_cast<hipStream_t>(stream));
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
  }
  return "unknown status";
}

}  // extern "C"
