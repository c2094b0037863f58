// eXmY CPU oracle: TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, scalar implementation of what the eXmY tensor codec computes,
// written from the paper's definitions in real-number terms (double precision,
// frexp / ldexp / nearbyint), with plain loops for the bit packing.  It shares
// no code, header, table or constant with the HIP library and must never be
// called from the product path: only tests, the smoke check and the
// cpu_baseline leg of the benchmark may use it.
//
// Paper passages followed (arxiv 2405.13938):
//   * Section 2 "Format", "Subnormals": 1 sign bit, X exponent bits, Y mantissa
//     bits; exponent field 0 with non-zero mantissa is a subnormal; every code
//     is a finite value (Section 5).
//   * Section 2 "Exponent Bias", "Metadata": the bias is software defined; the
//     metadatum is the maximum biased (fp32/bf16, bias 127) exponent, max_exp,
//     which is the exponent the top eXmY exponent code stands for.
//   * Section 2 "Rounding": round-to-nearest-even to Y mantissa bits.
//   * Section 2.1 "Emulation": outcomes saturate / round / subnormal / flush;
//     NaN and Inf are preserved.
//   * Section 2.2.1 "Type Conversion" and 2.2.2 "Bit Packing & Unpacking:
//     Power-of-2 Decomposition", Fig. 2.
//   * Section 3.1 "Exponent Distribution": 256-bin histogram of the biased
//     exponent; keeping the top 2^X-1 exponents plus zero.
//
// Readings where the paper is silent (documented in the repository's design
// notes):
//   - code bit order is sign | exponent | mantissa (IEEE order);
//   - the binary expansion of W = 1+X+Y is walked from its largest power of two
//     s downwards while the code is walked from bit 0 upwards, so the widest
//     plane holds the least significant bits (Fig. 2 drawn MSB-left);
//   - a group is 8 consecutive elements; element j of a group sits at bits
//     [s*j, s*j+s) of a little-endian 8s-bit word; planes are laid back to
//     back, widest first; a ragged last group is padded with zero codes;
//   - a rounding tie goes to the even multiple of the quantum of x's binade
//     (round-half-even on the significand, what nearbyint gives below): the
//     even code whenever Y >= 1; with Y = 0 a tie 1.5 * 2^e goes up to 2^(e+1);
//   - encode maps +-Inf and NaN to sign + largest magnitude code (parity
//     unpinned by the paper: a convention of this repository);
//   - X = 8 forces max_exp = 255 (identity exponent map); exponent code 255 is
//     not produced and decodes to the largest finite value (parity unpinned);
//   - ragged n (n % 8 != 0) handling is likewise parity unpinned;
//   - per-block metadata: blocks are runs of `block` consecutive elements
//     (a multiple of 8), the metadatum is the maximum biased exponent of the
//     block's finite values ("before rounding"), clamped into [2^X, 254]
//     ([1, 253] for X = 0);
//   - "maximum exponent after rounding": the exponent of the block's largest
//     finite magnitude once that value is rounded (ties to even) to as many
//     mantissa bits as the format's top binade has (Y, or Y - 1 when X = 0), so
//     that the block maximum is rounded and never cut off by saturation.
//
//   - fp16 container (Section 2.1: fp16 emulates X <= 5, Y <= 10): every half is
//     converted exactly to fp32 first; a format is valid with a max_exp only if its
//     top binade and its quantum are fp16 values (max_exp <= 142 and
//     max_exp - 2^X + 2 - 127 - Y >= -24), so that every decoded value is exact;
//     the histogram bins by the exponent of the value as an fp32 (an fp16
//     denormal therefore does not fall in bin 0);
//   - packing along rows (Section 2.2.2: (8R, C) -> arrays of shape (R, C)): the
//     group of output position (r, c) is elements (8r + j, c), j = 0..7, of the
//     row-major matrix; rows beyond the last are zero codes; each plane is a
//     row-major (R, C) array of words, planes back to back, widest first;
//   - two's complement reading of X = 0 (Section 2 "Format": e0m3 used as int4
//     represents [-8, 7]): the W = 1 + Y bits are a two's complement integer k in
//     [-2^Y, 2^Y - 1] and the value is k quanta; k = round-half-even(x / quantum),
//     clamped; Inf / NaN go to the end of the range on the side of their sign bit;
//     -0 and negative values that round to 0 give k = 0, which decodes to +0;
//   - float scaling at maximum exponent 127 (Section 2 "Metadata", Section
//     2.1): the paper gives no formulas.  Reading: the block's scale is
//     s = max|x| / vmax rounded once to fp32 (vmax = largest value of the format
//     with max_exp = 127; s is raised to FLT_MIN if smaller); the code of x is
//     that of the real quotient |x| / s in the max_exp = 127 format (nearest grid
//     point, ties to even, saturating), under the sign of x; the decoded value is
//     the real product value * s rounded once, to nearest even, into the
//     container (fp32, bf16 or fp16).  Both are evaluated in double: the
//     product of a value of at most 24 bits and a 24-bit scale is exact there,
//     and the quotient of two fp32 numbers is either exactly a rounding
//     boundary of the grid (boundaries have at most Y + 2 <= 26 significant
//     bits, hence are doubles, and the double division then returns it exactly)
//     or further from every boundary than 2^-51 of its size (a 24-bit number
//     minus a product of at most 50 bits), which the 2^-53 error of the double
//     division cannot bridge.  Parity unpinned by the paper beyond the
//     property that the block maximum is reproduced almost exactly.  The bf16
//     form of the scaling factor named in the same passage: the smallest bf16
//     value not below that fp32 scale (never below, so that the block maximum
//     divided by it still lies within the format's range), at most the largest
//     finite bf16; it enters encode and decode widened exactly to fp32.
//
// Pinned by tests/test_oracle_pins.py, tests/test_oracle_pack.py and
// tests/test_oracle_blocks.py against the
// paper's worked examples, library float8 / bfloat16 / float16 conversions and a
// brute-force nearest-value search.

#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <thread>
#include <vector>
#include <algorithm>

extern "C" {

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F16 = 2 };
enum {
  ORACLE_OK = 0,
  ORACLE_ERR_NULL = 1,
  ORACLE_ERR_FORMAT = 2,
  ORACLE_ERR_MAX_EXP = 3,
};

}  // extern "C"

namespace {

struct Format {
  int X, Y, max_exp;
  int emin8;       // biased (127) exponent of the binade with exponent code 1
  int64_t cmax;    // largest magnitude code that encode may produce
  int W;
};

// Mantissa bits the float container itself stores.
int container_mantissa(int dt) { return dt == ORACLE_F32 ? 23 : (dt == ORACLE_F16 ? 10 : 7); }

// Section 2.1: a format can be emulated in (and therefore converted from / to)
// a float container when its exponent and mantissa fit.  With X = 0 a code has
// only Y significant bits, one fewer than a normal with Y mantissa bits, so one
// more is allowed.
int check_format(int dt, int X, int Y, int max_exp, bool packed, Format* f) {
  if (dt != ORACLE_F32 && dt != ORACLE_BF16 && dt != ORACLE_F16) return ORACLE_ERR_FORMAT;
  if (X < 0 || X > 8 || Y < 0) return ORACLE_ERR_FORMAT;
  if (dt == ORACLE_F16 && X > 5) return ORACLE_ERR_FORMAT;  // Section 2.1: fp16 emulates X <= 5, Y <= 10
  const int P = container_mantissa(dt);
  if (X >= 1 ? (Y > P) : (Y > P + 1)) return ORACLE_ERR_FORMAT;
  if (packed && 1 + X + Y > 32) return ORACLE_ERR_FORMAT;  // segments of 32, 16, 8, 4, 2 and 1 bits; 32 is e8m23 alone
  if (packed && Y > 23) return ORACLE_ERR_FORMAT;          // e0m24 packs as e1m23, which it equals bit for bit
  if (X == 8) {
    if (max_exp != 255) return ORACLE_ERR_MAX_EXP;
  } else if (X == 0) {
    if (max_exp < 0 || max_exp > 253) return ORACLE_ERR_MAX_EXP;
    // the quantum 2^(max_exp + 1 - 127 - Y) must be a value of the container
    if (Y == P + 1 && max_exp < 1) return ORACLE_ERR_MAX_EXP;
  } else {
    if (max_exp < (1 << X) - 1 || max_exp > 254) return ORACLE_ERR_MAX_EXP;
  }
  if (dt == ORACLE_F16) {
    // fp16 holds binades 2^-14 .. 2^15 and multiples of 2^-24 below: the top binade of the format and
    // its quantum must lie inside
    if (max_exp > 142) return ORACLE_ERR_MAX_EXP;
    if (max_exp - (1 << X) + 2 - 127 - Y < -24) return ORACLE_ERR_MAX_EXP;
  }
  f->X = X;
  f->Y = Y;
  f->max_exp = max_exp;
  f->W = 1 + X + Y;
  f->emin8 = max_exp - (1 << X) + 2;
  f->cmax = ((int64_t)1 << (X + Y)) - 1;
  if (X == 8) f->cmax = ((int64_t)254 << Y) | (((int64_t)1 << Y) - 1);
  return ORACLE_OK;
}

// The value a magnitude code stands for (Section 2 "Format", "Subnormals",
// "Exponent Bias").
double code_magnitude(const Format& f, int64_t c) {
  if (f.X == 8 && c > f.cmax) c = f.cmax;
  const int64_t E = c >> f.Y;
  const int64_t M = c & (((int64_t)1 << f.Y) - 1);
  if (E == 0) return std::ldexp((double)M, f.emin8 - 127 - f.Y);
  return std::ldexp((double)(((int64_t)1 << f.Y) + M), (int)(E - 1) + f.emin8 - 127 - f.Y);
}

// Magnitude code of a finite, non-negative real a (Section 2 "Rounding",
// Section 2.1 outcomes).
int64_t magnitude_code(const Format& f, double a) {
  const double smallest_normal = std::ldexp(1.0, f.emin8 - 127);
  int64_t c;
  if (a < smallest_normal) {
    // subnormal range: fixed quantum; may round to 0 (flush) or up to the
    // smallest normal, whose code is 2^Y.
    c = (int64_t)std::nearbyint(std::ldexp(a, -(f.emin8 - 127 - f.Y)));
  } else {
    int ee;
    (void)std::frexp(a, &ee);  // a = m * 2^ee, m in [0.5, 1)
    int e = ee - 1;            // floor(log2 a)
    int64_t k = (int64_t)std::nearbyint(std::ldexp(a, -(e - f.Y)));  // in [2^Y, 2^(Y+1)]
    if (k == ((int64_t)1 << (f.Y + 1))) {
      e += 1;
      k = (int64_t)1 << f.Y;
    }
    const int64_t E = (int64_t)e + 127 - f.emin8 + 1;
    c = (E << f.Y) + (k - ((int64_t)1 << f.Y));
  }
  return std::min(c, f.cmax);  // saturate to the largest normal
}

inline float bits_to_float(uint32_t b);
inline uint32_t float_to_bits(float f);

// fp32 bits of an IEEE half: 1 sign, 5 exponent (bias 15), 10 mantissa bits; every half is an fp32 value.
inline uint32_t half_to_float_bits(uint16_t h) {
  const uint32_t sign = (uint32_t)(h >> 15) << 31;
  const int e = (h >> 10) & 0x1F;
  const int m = h & 0x3FF;
  if (e == 31) return sign | 0x7F800000u | ((uint32_t)m << 13);      // Inf, or NaN with its payload
  const float v = e == 0 ? std::ldexp((float)m, -24) : std::ldexp((float)(1024 + m), e - 25);
  return sign | float_to_bits(v);
}

// The half with exactly the value of these fp32 bits; aborts if there is none (the callers only store
// values that the format's validation has shown to be fp16 values).
inline uint16_t float_bits_to_half_exact(uint32_t bits) {
  const uint16_t sign = (uint16_t)((bits >> 31) << 15);
  const float a = std::fabs(bits_to_float(bits));
  if (a == 0.0f) return sign;
  if (std::isinf(a)) return (uint16_t)(sign | 0x7C00);
  int e;
  const float frac = std::frexp(a, &e);  // a = frac * 2^e, frac in [0.5, 1)
  if (e - 1 >= -14) {                    // normal half: 11 significant bits
    const float k = std::ldexp(frac, 11);
    if (e - 1 > 15 || k != std::floor(k)) std::abort();
    return (uint16_t)(sign | ((e - 1 + 15) << 10) | ((int)k - 1024));
  }
  const float k = std::ldexp(a, 24);     // subnormal half: a multiple of 2^-24
  if (k != std::floor(k) || k >= 1024.0f) std::abort();
  return (uint16_t)(sign | (int)k);
}

inline uint32_t load_bits(const void* src, int dt, uint64_t i) {
  if (dt == ORACLE_F32) return ((const uint32_t*)src)[i];
  if (dt == ORACLE_F16) return half_to_float_bits(((const uint16_t*)src)[i]);
  return (uint32_t)((const uint16_t*)src)[i] << 16;  // bf16 = upper half of fp32
}

inline void store_bits(void* dst, int dt, uint64_t i, uint32_t bits) {
  if (dt == ORACLE_F32)
    ((uint32_t*)dst)[i] = bits;
  else if (dt == ORACLE_F16)
    ((uint16_t*)dst)[i] = float_bits_to_half_exact(bits);
  else {
    if (bits & 0xFFFFu) std::abort();  // every decoded value must be exact in bf16
    ((uint16_t*)dst)[i] = (uint16_t)(bits >> 16);
  }
}

inline float bits_to_float(uint32_t b) {
  float f;
  std::memcpy(&f, &b, 4);
  return f;
}
inline uint32_t float_to_bits(float f) {
  uint32_t b;
  std::memcpy(&b, &f, 4);
  return b;
}

// Full W-bit code of one element.
uint32_t encode_one(const Format& f, uint32_t bits) {
  const uint32_t sign = bits >> 31;
  const float x = bits_to_float(bits);
  int64_t c;
  if (std::isnan(x) || std::isinf(x))
    c = f.cmax;
  else
    c = magnitude_code(f, std::fabs((double)x));
  return (uint32_t)((sign << (f.X + f.Y)) | (uint32_t)c);
}

// fp32 bit pattern of the value of a full code (exact by construction).
uint32_t decode_one(const Format& f, uint32_t code) {
  const uint32_t sign = (code >> (f.X + f.Y)) & 1u;
  const int64_t c = code & (uint32_t)((((int64_t)1) << (f.X + f.Y)) - 1);
  const float v = (float)code_magnitude(f, c);
  return float_to_bits(v) | (sign << 31);
}

// Segment widths of the power-of-2 decomposition of W, widest first
// (Section 2.2.2: 7 = 4 + 2 + 1, 5 = 4 + 1).
int plane_list(int W, int seg[8]) {
  int n = 0;
  for (int s = 32; s >= 1; s >>= 1)
    if (W & s) seg[n++] = s;
  return n;
}

template <class Fn>
void parallel_ranges(uint64_t n_items, int threads, Fn fn) {
  if (threads <= 1 || n_items < 4096) {
    fn((uint64_t)0, n_items);
    return;
  }
  std::vector<std::thread> pool;
  const uint64_t per = (n_items + threads - 1) / threads;
  for (int t = 0; t < threads; ++t) {
    const uint64_t a = std::min(n_items, per * t), b = std::min(n_items, per * (t + 1));
    if (a < b) pool.emplace_back([=] { fn(a, b); });
  }
  for (auto& th : pool) th.join();
}

// Bit packing, Fig. 2: the codes of groups [g0, g1) go to every plane.
// codes[i - base] is the code of element i.
void pack_groups(const uint32_t* codes, uint64_t base, uint64_t n, int W, uint8_t* out, uint64_t g0, uint64_t g1) {
  const uint64_t G = (n + 7) / 8;
  int seg[8];
  const int np = plane_list(W, seg);
  uint64_t plane_off = 0;
  int lo = 0;
  for (int p = 0; p < np; ++p) {
    const int s = seg[p];
    uint8_t* plane = out + plane_off;
    for (uint64_t g = g0; g < g1; ++g) {
      // one 8s-bit little-endian word per group: element j at bits [s*j, s*j+s)
      for (int b = 0; b < s; ++b) plane[g * s + b] = 0;
      for (int j = 0; j < 8; ++j) {
        const uint64_t i = g * 8 + j;
        const uint32_t code = i < n ? codes[i - base] : 0u;
        const uint32_t field = (uint32_t)(((uint64_t)code >> lo) & (((uint64_t)1 << s) - 1u));
        for (int b = 0; b < s; ++b) {
          const int bit = s * j + b;
          if ((field >> b) & 1u) plane[g * s + bit / 8] |= (uint8_t)(1u << (bit % 8));
        }
      }
    }
    plane_off += G * (uint64_t)s;
    lo += s;
  }
}

void unpack_groups(const uint8_t* in, uint64_t n, int W, uint32_t* codes, uint64_t base, uint64_t g0, uint64_t g1) {
  const uint64_t G = (n + 7) / 8;
  int seg[8];
  const int np = plane_list(W, seg);
  for (uint64_t g = g0; g < g1; ++g)
    for (int j = 0; j < 8; ++j)
      if (g * 8 + j < n) codes[g * 8 + j - base] = 0;
  uint64_t plane_off = 0;
  int lo = 0;
  for (int p = 0; p < np; ++p) {
    const int s = seg[p];
    const uint8_t* plane = in + plane_off;
    for (uint64_t g = g0; g < g1; ++g) {
      for (int j = 0; j < 8; ++j) {
        const uint64_t i = g * 8 + j;
        if (i >= n) continue;
        uint32_t field = 0;
        for (int b = 0; b < s; ++b) {
          const int bit = s * j + b;
          if ((plane[g * s + bit / 8] >> (bit % 8)) & 1u) field |= 1u << b;
        }
        codes[i - base] |= field << lo;
      }
    }
    plane_off += G * (uint64_t)s;
    lo += s;
  }
}

}  // namespace

extern "C" {

// ceil(n/8) * W bytes: perfect compression (Section 2.2.2).
uint64_t exmy_oracle_packed_bytes(uint64_t n, int X, int Y) { return ((n + 7) / 8) * (uint64_t)(1 + X + Y); }

int exmy_oracle_check_format(int dt, int X, int Y, int max_exp, int packed) {
  Format f;
  return check_format(dt, X, Y, max_exp, packed != 0, &f);
}

// Real value of a full code (sign included), for value-set enumeration.
double exmy_oracle_code_value(int X, int Y, int max_exp, uint32_t code) {
  Format f;
  if (check_format(ORACLE_F32, X, Y, max_exp, false, &f) != ORACLE_OK) return NAN;
  const uint32_t sign = (code >> (X + Y)) & 1u;
  const double m = code_magnitude(f, code & (uint32_t)((((int64_t)1) << (X + Y)) - 1));
  return sign ? -m : m;
}

// Step 1 of the codec (Section 2.2.1): float -> eXmY code in a 32-bit container.
int exmy_oracle_to_codes(const void* src, int dt, uint64_t n, int X, int Y, int max_exp, uint32_t* codes,
                         int threads) {
  if ((!src || !codes) && n) return ORACLE_ERR_NULL;
  Format f;
  if (int rc = check_format(dt, X, Y, max_exp, true, &f)) return rc;
  parallel_ranges(n, threads, [&](uint64_t a, uint64_t b) {
    for (uint64_t i = a; i < b; ++i) codes[i] = encode_one(f, load_bits(src, dt, i));
  });
  return ORACLE_OK;
}

// Inverse of step 1: code -> float of type dt.
int exmy_oracle_from_codes(const uint32_t* codes, int dt, uint64_t n, int X, int Y, int max_exp, void* dst,
                           int threads) {
  if ((!dst || !codes) && n) return ORACLE_ERR_NULL;
  Format f;
  if (int rc = check_format(dt, X, Y, max_exp, true, &f)) return rc;
  parallel_ranges(n, threads, [&](uint64_t a, uint64_t b) {
    for (uint64_t i = a; i < b; ++i) store_bits(dst, dt, i, decode_one(f, codes[i]));
  });
  return ORACLE_OK;
}

// Step 2 of the codec (Section 2.2.2): W-bit codes -> planes.
int exmy_oracle_pack(const uint32_t* codes, uint64_t n, int W, uint8_t* out, int threads) {
  if ((!codes || !out) && n) return ORACLE_ERR_NULL;
  if (W < 1 || W > 32) return ORACLE_ERR_FORMAT;
  parallel_ranges((n + 7) / 8, threads, [&](uint64_t a, uint64_t b) { pack_groups(codes, 0, n, W, out, a, b); });
  return ORACLE_OK;
}

int exmy_oracle_unpack(const uint8_t* in, uint64_t n, int W, uint32_t* codes, int threads) {
  if ((!codes || !in) && n) return ORACLE_ERR_NULL;
  if (W < 1 || W > 32) return ORACLE_ERR_FORMAT;
  parallel_ranges((n + 7) / 8, threads, [&](uint64_t a, uint64_t b) { unpack_groups(in, n, W, codes, 0, a, b); });
  return ORACLE_OK;
}

// encode = step 1 then step 2.
int exmy_oracle_encode(const void* src, int dt, uint64_t n, int X, int Y, int max_exp, uint8_t* dst_packed,
                       int threads) {
  if ((!src || !dst_packed) && n) return ORACLE_ERR_NULL;
  Format f;
  if (int rc = check_format(dt, X, Y, max_exp, true, &f)) return rc;
  parallel_ranges((n + 7) / 8, threads, [&](uint64_t g0, uint64_t g1) {
    // convert this range of groups, then pack it; ranges touch disjoint bytes
    const uint64_t a = g0 * 8, b = std::min(n, g1 * 8);
    std::vector<uint32_t> codes(b - a);
    for (uint64_t i = a; i < b; ++i) codes[i - a] = encode_one(f, load_bits(src, dt, i));
    pack_groups(codes.data(), a, n, f.W, dst_packed, g0, g1);
  });
  return ORACLE_OK;
}

int exmy_oracle_decode(const uint8_t* src_packed, int dt, uint64_t n, int X, int Y, int max_exp, void* dst,
                       int threads) {
  if ((!src_packed || !dst) && n) return ORACLE_ERR_NULL;
  Format f;
  if (int rc = check_format(dt, X, Y, max_exp, true, &f)) return rc;
  parallel_ranges((n + 7) / 8, threads, [&](uint64_t g0, uint64_t g1) {
    const uint64_t a = g0 * 8, b = std::min(n, g1 * 8);
    std::vector<uint32_t> codes(b - a);
    unpack_groups(src_packed, n, f.W, codes.data(), a, g0, g1);
    for (uint64_t i = a; i < b; ++i) store_bits(dst, dt, i, decode_one(f, codes[i - a]));
  });
  return ORACLE_OK;
}

// ---------------------------------------------------------------------------
// Records: a second arrangement of the same plane words.  Section 2.2.2 keeps one
// array per power-of-2 segment; here the words of one group follow each other,
// widest segment first, as one record of W bytes ("8 values in W bytes"), and the
// records follow each other in group order.  Not a layout of the paper: the words
// are those of Fig. 2, only their order in memory differs.  Widths up to 16.
static void records_op(bool pack, uint32_t* codes, uint64_t n, int W, uint8_t* blob) {
  const uint64_t G = (n + 7) / 8;
  int seg[8];
  const int np = plane_list(W, seg);
  for (uint64_t g = 0; g < G; ++g) {
    uint8_t* rec = blob + g * (uint64_t)W;
    if (pack)
      for (int b = 0; b < W; ++b) rec[b] = 0;
    int word_off = 0;  // byte offset of the segment's word inside the record
    int lo = 0;        // first code bit of the segment
    for (int p = 0; p < np; ++p) {
      const int s = seg[p];
      for (int j = 0; j < 8; ++j) {
        const uint64_t i = g * 8 + j;
        for (int b = 0; b < s; ++b) {
          const int bit = s * j + b;  // element j at bits [s*j, s*j + s) of the little-endian word
          uint8_t* byte = rec + word_off + bit / 8;
          if (pack) {
            const uint32_t code = i < n ? codes[i] : 0u;
            if ((code >> (lo + b)) & 1u) *byte |= (uint8_t)(1u << (bit % 8));
          } else if (i < n) {
            if ((*byte >> (bit % 8)) & 1u) codes[i] |= 1u << (lo + b);
          }
        }
      }
      word_off += s;
      lo += s;
    }
  }
}

int exmy_oracle_encode_records(const void* src, int dt, uint64_t n, int X, int Y, int max_exp, uint8_t* dst_records) {
  if ((!src || !dst_records) && n) return ORACLE_ERR_NULL;
  Format f;
  if (int rc = check_format(dt, X, Y, max_exp, true, &f)) return rc;
  if (f.W > 16) return ORACLE_ERR_FORMAT;
  std::vector<uint32_t> codes(n);
  for (uint64_t i = 0; i < n; ++i) codes[i] = encode_one(f, load_bits(src, dt, i));
  records_op(true, codes.data(), n, f.W, dst_records);
  return ORACLE_OK;
}

int exmy_oracle_decode_records(const uint8_t* src_records, int dt, uint64_t n, int X, int Y, int max_exp, void* dst) {
  if ((!src_records || !dst) && n) return ORACLE_ERR_NULL;
  Format f;
  if (int rc = check_format(dt, X, Y, max_exp, true, &f)) return rc;
  if (f.W > 16) return ORACLE_ERR_FORMAT;
  std::vector<uint32_t> codes(n, 0u);
  records_op(false, codes.data(), n, f.W, const_cast<uint8_t*>(src_records));
  for (uint64_t i = 0; i < n; ++i) store_bits(dst, dt, i, decode_one(f, codes[i]));
  return ORACLE_OK;
}

// ---------------------------------------------------------------------------
// Reserved code points for NaN and Inf (Section 5: values encoded for training
// would need an encoding for these, which the paper leaves open).  The two
// conventions of the float types in use are offered:
//   specials = 1, IEEE 754 style (fp32, bf16, fp16, e5m2): the top exponent code
//     is reserved; mantissa 0 under it is Inf, anything else NaN.  The finite
//     values are those of the plain format without its top binade.
//   specials = 2, NaN only (OCP e4m3): the all-ones magnitude code is NaN, there
//     is no Inf; the finite values are those of the plain format without its
//     largest one.
// Finite elements round as always and saturate to the largest finite value;
// a NaN takes the all-ones magnitude code under its own sign; Inf takes the Inf
// code, or (NaN only) saturates like any large value.  max_exp keeps its meaning:
// the exponent of the top exponent code, reserved or not.
static int specials_format(int dt, int X, int Y, int max_exp, int specials, bool packed, Format* f) {
  if (specials != 1 && specials != 2) return ORACLE_ERR_FORMAT;
  if (int rc = check_format(dt, X, Y, max_exp, packed, f)) return rc;
  if (packed && f->W > 16) return ORACLE_ERR_FORMAT;
  if (specials == 1) {
    if (X < 1) return ORACLE_ERR_FORMAT;
    f->cmax = ((((int64_t)1 << X) - 1) << Y) - 1;  // below the reserved exponent code
  } else {
    if (X == 8 || X + Y < 1) return ORACLE_ERR_FORMAT;  // exponent code 255 is not a finite binade of any container
    f->cmax = ((int64_t)1 << (X + Y)) - 2;
  }
  return ORACLE_OK;
}

static uint32_t encode_one_specials(const Format& f, int specials, uint32_t bits) {
  const uint32_t sign = bits >> 31;
  const float x = bits_to_float(bits);
  const int64_t all_ones = ((int64_t)1 << (f.X + f.Y)) - 1;
  int64_t c;
  if (std::isnan(x))
    c = all_ones;
  else if (std::isinf(x))
    c = specials == 1 ? ((((int64_t)1 << f.X) - 1) << f.Y) : f.cmax;
  else
    c = magnitude_code(f, std::fabs((double)x));  // saturates to f.cmax, the largest finite code
  return (uint32_t)((sign << (f.X + f.Y)) | (uint32_t)c);
}

// fp32 bits of a full code: finite codes as always; reserved ones give Inf or the quiet NaN 0x7FC00000, signed.
static uint32_t decode_one_specials(const Format& f, int specials, uint32_t code) {
  const uint32_t sign = ((code >> (f.X + f.Y)) & 1u) << 31;
  const int64_t c = code & (uint32_t)((((int64_t)1) << (f.X + f.Y)) - 1);
  if (c <= f.cmax) return float_to_bits((float)code_magnitude(f, c)) | sign;
  if (specials == 1 && c == ((((int64_t)1 << f.X) - 1) << f.Y)) return sign | 0x7F800000u;
  return sign | 0x7FC00000u;
}

static void store_bits_specials(void* dst, int dt, uint64_t i, uint32_t bits) {
  if (dt == ORACLE_F16 && (bits & 0x7FFFFFFFu) > 0x7F800000u)  // the half NaN with the same quiet bit
    ((uint16_t*)dst)[i] = (uint16_t)(((bits >> 31) << 15) | 0x7E00u);
  else
    store_bits(dst, dt, i, bits);
}

int exmy_oracle_encode_specials(const void* src, int dt, uint64_t n, int X, int Y, int max_exp, int specials,
                                uint8_t* dst_packed) {
  if ((!src || !dst_packed) && n) return ORACLE_ERR_NULL;
  Format f;
  if (int rc = specials_format(dt, X, Y, max_exp, specials, true, &f)) return rc;
  std::vector<uint32_t> codes(n);
  for (uint64_t i = 0; i < n; ++i) codes[i] = encode_one_specials(f, specials, load_bits(src, dt, i));
  pack_groups(codes.data(), 0, n, f.W, dst_packed, 0, (n + 7) / 8);
  return ORACLE_OK;
}

int exmy_oracle_decode_specials(const uint8_t* src_packed, int dt, uint64_t n, int X, int Y, int max_exp,
                                int specials, void* dst) {
  if ((!src_packed || !dst) && n) return ORACLE_ERR_NULL;
  Format f;
  if (int rc = specials_format(dt, X, Y, max_exp, specials, true, &f)) return rc;
  std::vector<uint32_t> codes(n);
  unpack_groups(src_packed, n, f.W, codes.data(), 0, 0, (n + 7) / 8);
  for (uint64_t i = 0; i < n; ++i) store_bits_specials(dst, dt, i, decode_one_specials(f, specials, codes[i]));
  return ORACLE_OK;
}

// Emulation: NaN / Inf stay as they are (Section 2.1); finite elements become the nearest finite value of
// the format with reserved code points, saturated.
int exmy_oracle_emulate_specials(void* data, int dt, uint64_t n, int X, int Y, int max_exp, int specials) {
  if (!data && n) return ORACLE_ERR_NULL;
  Format f;
  if (int rc = specials_format(dt, X, Y, max_exp, specials, false, &f)) return rc;
  for (uint64_t i = 0; i < n; ++i) {
    const uint32_t bits = load_bits(data, dt, i);
    const float x = bits_to_float(bits);
    if (std::isnan(x) || std::isinf(x)) continue;
    const float v = (float)code_magnitude(f, magnitude_code(f, std::fabs((double)x)));
    store_bits(data, dt, i, float_to_bits(v) | (bits & 0x80000000u));
  }
  return ORACLE_OK;
}

// Emulation (Section 2.1): quantise and dequantise in the element's own type;
// NaN and +-Inf are returned bit-identical.
int exmy_oracle_emulate(void* data, int dt, uint64_t n, int X, int Y, int max_exp, int threads) {
  if (!data && n) return ORACLE_ERR_NULL;
  Format f;
  if (int rc = check_format(dt, X, Y, max_exp, false, &f)) return rc;
  parallel_ranges(n, threads, [&](uint64_t a, uint64_t b) {
    for (uint64_t i = a; i < b; ++i) {
      const uint32_t bits = load_bits(data, dt, i);
      const float x = bits_to_float(bits);
      if (std::isnan(x) || std::isinf(x)) continue;
      const int64_t c = magnitude_code(f, std::fabs((double)x));
      const float v = (float)code_magnitude(f, c);
      store_bits(data, dt, i, float_to_bits(v) | (bits & 0x80000000u));
    }
  });
  return ORACLE_OK;
}

// 256-bin histogram of the biased exponent field (Section 3.1, Fig. 3): +-0 and
// denormals fall in bin 0, Inf / NaN in bin 255.  Accumulates into hist.
int exmy_oracle_exponent_histogram(const void* src, int dt, uint64_t n, uint64_t* hist256) {
  if ((!src && n) || !hist256) return ORACLE_ERR_NULL;
  if (dt != ORACLE_F32 && dt != ORACLE_BF16 && dt != ORACLE_F16) return ORACLE_ERR_FORMAT;
  for (uint64_t i = 0; i < n; ++i) hist256[(load_bits(src, dt, i) >> 23) & 0xFFu] += 1;
  return ORACLE_OK;
}

// Smallest biased exponent e (0..254) such that at least `coverage` of the
// finite elements have an exponent <= e (Section 3.1: keep the top exponents,
// let the rest saturate or flush).  Returns -1 for an empty histogram.
int exmy_oracle_max_exp_from_histogram(const uint64_t* hist256, double coverage) {
  uint64_t total = 0;
  for (int e = 0; e < 255; ++e) total += hist256[e];
  if (total == 0) return -1;
  uint64_t cum = 0;
  for (int e = 0; e < 255; ++e) {
    cum += hist256[e];
    if ((double)cum >= coverage * (double)total) return e;
  }
  return 254;
}


// ---------------------------------------------------------------------------
// Per-block metadata (Section 2 "Metadata", "Block Size"; Section 2.2.1: a tensor
// of codes plus one 8-bit maximum exponent per block).  The tensor is cut into
// consecutive blocks of `block` elements (a multiple of 8; a row of a row-major
// matrix, or a part of one); the last block may be short.  Valid metadata in
// block mode: 2^X <= max_exp <= 254 for 1 <= X <= 7, 1 <= max_exp <= 253 for
// X = 0 (so that the smallest binade of every block is a normal of the
// container); values outside are clamped into that range.  X = 8 has no
// per-block metadata.

// The per-block, float-scaling and row-packing forms stop at 16-bit codes.
static const int kBlockWidth = 16;

// Y < 0: the caller has no Y (the "before rounding" maximum); the fp16 container then applies
// only the limits that do not depend on it.
static int block_meta_range(int dt, int X, int Y, int* lo, int* hi) {
  if (X < 0 || X > 7) return ORACLE_ERR_FORMAT;
  *lo = X == 0 ? 1 : (1 << X);
  *hi = X == 0 ? 253 : 254;
  if (dt == ORACLE_F16) {  // top binade at most 2^15, quantum at least 2^-24 (see check_format)
    if (X > 5) return ORACLE_ERR_FORMAT;
    *hi = 142;
    if (Y >= 0) *lo = std::max(*lo, X == 0 ? 102 + Y : 101 + Y + (1 << X));
    if (*lo > *hi) return ORACLE_ERR_FORMAT;
  }
  return ORACLE_OK;
}

static int clamp_meta(int m, int lo, int hi) { return m < lo ? lo : (m > hi ? hi : m); }

// "Maximum exponent before rounding": the largest biased exponent among the
// finite elements of each block, clamped into the valid range.
int exmy_oracle_block_max_exp(const void* src, int dt, uint64_t n, uint64_t block, int X, uint8_t* max_exp_out) {
  if ((!src || !max_exp_out) && n) return ORACLE_ERR_NULL;
  if (dt != ORACLE_F32 && dt != ORACLE_BF16 && dt != ORACLE_F16) return ORACLE_ERR_FORMAT;
  if (block == 0 || block % 8) return ORACLE_ERR_FORMAT;
  int lo, hi;
  if (int rc = block_meta_range(dt, X, -1, &lo, &hi)) return rc;
  const uint64_t nb = (n + block - 1) / block;
  for (uint64_t b = 0; b < nb; ++b) {
    int m = 0;
    for (uint64_t i = b * block; i < std::min(n, (b + 1) * block); ++i) {
      const int e = (int)((load_bits(src, dt, i) >> 23) & 0xFFu);
      if (e != 255 && e > m) m = e;
    }
    max_exp_out[b] = (uint8_t)clamp_meta(m, lo, hi);
  }
  return ORACLE_OK;
}

// "Maximum exponent after rounding" (Section 2 "Metadata"; Section 2.1: with this
// scheme 3.9 in e2m1 always rounds up to 4.0).  The block's largest finite
// magnitude is rounded to nearest, ties to even, to the mantissa width of the
// format's top binade; the metadatum is the biased exponent of the result.
// Biased exponent of the magnitude m >= 0 after rounding it to nearest, ties to even, to `bits`
// fraction bits in its own binade (0 for magnitudes below the smallest normal float).
static int biased_exp_after_rounding(double m, int bits) {
  if (!(m >= std::ldexp(1.0, -126))) return 0;
  int e;
  const double frac = std::frexp(m, &e);                         // m = frac * 2^e, frac in [0.5, 1)
  const double k = std::nearbyint(std::ldexp(frac, bits + 1));    // significand with `bits` fraction bits
  std::frexp(std::ldexp(k, e - bits - 1), &e);                   // the rounded value may be 2^e
  return e - 1 + 127;
}

int exmy_oracle_block_max_exp_after_rounding(const void* src, int dt, uint64_t n, uint64_t block, int X, int Y,
                                             uint8_t* max_exp_out) {
  if ((!src || !max_exp_out) && n) return ORACLE_ERR_NULL;
  if (block == 0 || block % 8) return ORACLE_ERR_FORMAT;
  int lo, hi;
  if (int rc = block_meta_range(dt, X, Y, &lo, &hi)) return rc;
  Format f0;
  if (int rc = check_format(dt, X, Y, hi, false, &f0)) return rc;
  const int bits = X == 0 ? (Y > 0 ? Y - 1 : 0) : Y;  // mantissa bits of the top binade
  const uint64_t nb = (n + block - 1) / block;
  for (uint64_t b = 0; b < nb; ++b) {
    double m = 0.0;
    for (uint64_t i = b * block; i < std::min(n, (b + 1) * block); ++i) {
      const double a = std::fabs((double)bits_to_float(load_bits(src, dt, i)));
      if (std::isfinite(a) && a > m) m = a;
    }
    max_exp_out[b] = (uint8_t)clamp_meta(biased_exp_after_rounding(m, bits), lo, hi);
  }
  return ORACLE_OK;
}

// what: 0 = encode (src -> packed), 1 = decode (packed -> dst), 2 = emulate in place (data = src)
static int blocks_op(int what, const void* src, void* dst, int dt, uint64_t n, uint64_t block, int X, int Y,
                     const uint8_t* max_exp, int threads) {
  if (n && (!src || !dst || !max_exp)) return ORACLE_ERR_NULL;
  if (block == 0 || block % 8) return ORACLE_ERR_FORMAT;
  int lo, hi;
  if (int rc = block_meta_range(dt, X, Y, &lo, &hi)) return rc;
  Format f0;
  if (int rc = check_format(dt, X, Y, hi, what != 2, &f0)) return rc;
  if (what != 2 && 1 + X + Y > kBlockWidth) return ORACLE_ERR_FORMAT;
  const uint64_t nb = (n + block - 1) / block;
  const int W = 1 + X + Y;
  std::vector<uint32_t> codes;
  if (what != 2) codes.resize(n);
  if (what == 1) unpack_groups((const uint8_t*)src, n, W, codes.data(), 0, 0, (n + 7) / 8);
  parallel_ranges(nb, threads, [&](uint64_t b0, uint64_t b1) {
    for (uint64_t b = b0; b < b1; ++b) {
      Format f;
      check_format(dt, X, Y, clamp_meta(max_exp[b], lo, hi), what != 2, &f);
      for (uint64_t i = b * block; i < std::min(n, (b + 1) * block); ++i) {
        if (what == 0) {
          codes[i] = encode_one(f, load_bits(src, dt, i));
        } else if (what == 1) {
          store_bits(dst, dt, i, decode_one(f, codes[i]));
        } else {
          const uint32_t bits = load_bits(src, dt, i);
          const float x = bits_to_float(bits);
          if (std::isnan(x) || std::isinf(x)) continue;
          const float v = (float)code_magnitude(f, magnitude_code(f, std::fabs((double)x)));
          store_bits(dst, dt, i, float_to_bits(v) | (bits & 0x80000000u));
        }
      }
    }
  });
  if (what == 0) pack_groups(codes.data(), 0, n, W, (uint8_t*)dst, 0, (n + 7) / 8);
  return ORACLE_OK;
}

int exmy_oracle_encode_blocks(const void* src, int dt, uint64_t n, uint64_t block, int X, int Y,
                              const uint8_t* max_exp, uint8_t* dst_packed, int threads) {
  return blocks_op(0, src, dst_packed, dt, n, block, X, Y, max_exp, threads);
}

int exmy_oracle_decode_blocks(const uint8_t* src_packed, int dt, uint64_t n, uint64_t block, int X, int Y,
                              const uint8_t* max_exp, void* dst, int threads) {
  return blocks_op(1, src_packed, dst, dt, n, block, X, Y, max_exp, threads);
}

int exmy_oracle_emulate_blocks(void* data, int dt, uint64_t n, uint64_t block, int X, int Y, const uint8_t* max_exp,
                               int threads) {
  return blocks_op(2, data, data, dt, n, block, X, Y, max_exp, threads);
}

// ---------------------------------------------------------------------------
// Blocks that are columns or 2-D tiles (the block shapes of Section 2 "Block
// Size" that are not runs of consecutive elements).  src is a row-major
// (rows, cols) matrix; tile (i, j) covers rows [i*tile_rows, (i+1)*tile_rows) and
// columns [j*tile_cols, (j+1)*tile_cols), cut off at the matrix edges; its
// metadatum is byte i * ceil(cols / tile_cols) + j of the metadata array.  A
// column is the tile (rows, 1), a row (1, cols), a sub row (1, k).  Codes are
// packed in the flat layout of the matrix in memory (groups of 8 consecutive
// elements; cols is a multiple of 8, so a group lies inside one row).  Metadata
// range, clamping and widths as for the consecutive blocks above.

static int tiles_shape(uint64_t rows, uint64_t cols, uint64_t tile_rows, uint64_t tile_cols) {
  if (tile_rows == 0 || tile_cols == 0) return ORACLE_ERR_FORMAT;
  if (cols % 8) return ORACLE_ERR_FORMAT;
  (void)rows;
  return ORACLE_OK;
}

// scheme 0: "maximum exponent before rounding" (Y is not used), 1: "after rounding".
int exmy_oracle_tile_max_exp(const void* src, int dt, uint64_t rows, uint64_t cols, uint64_t tile_rows,
                             uint64_t tile_cols, int X, int Y, int scheme, uint8_t* max_exp_out) {
  if ((!src || !max_exp_out) && rows && cols) return ORACLE_ERR_NULL;
  if (dt != ORACLE_F32 && dt != ORACLE_BF16 && dt != ORACLE_F16) return ORACLE_ERR_FORMAT;
  if (scheme != 0 && scheme != 1) return ORACLE_ERR_FORMAT;
  if (int rc = tiles_shape(rows, cols, tile_rows, tile_cols)) return rc;
  int lo, hi;
  if (int rc = block_meta_range(dt, X, scheme ? Y : -1, &lo, &hi)) return rc;
  int bits = 0;
  if (scheme) {
    Format f0;
    if (int rc = check_format(dt, X, Y, hi, false, &f0)) return rc;
    bits = X == 0 ? (Y > 0 ? Y - 1 : 0) : Y;  // mantissa bits of the top binade
  }
  const uint64_t tr_n = (rows + tile_rows - 1) / tile_rows, tc_n = (cols + tile_cols - 1) / tile_cols;
  for (uint64_t ti = 0; ti < tr_n; ++ti) {
    for (uint64_t tj = 0; tj < tc_n; ++tj) {
      double m = 0.0;  // largest finite magnitude of the tile
      for (uint64_t r = ti * tile_rows; r < std::min(rows, (ti + 1) * tile_rows); ++r) {
        for (uint64_t c = tj * tile_cols; c < std::min(cols, (tj + 1) * tile_cols); ++c) {
          const double a = std::fabs((double)bits_to_float(load_bits(src, dt, r * cols + c)));
          if (std::isfinite(a) && a > m) m = a;
        }
      }
      int biased;
      if (scheme) {
        biased = biased_exp_after_rounding(m, bits);
      } else {
        int e;
        (void)std::frexp(m, &e);  // m in [2^(e-1), 2^e)
        biased = m >= std::ldexp(1.0, -126) ? e - 1 + 127 : 0;
      }
      max_exp_out[ti * tc_n + tj] = (uint8_t)clamp_meta(biased, lo, hi);
    }
  }
  return ORACLE_OK;
}

// what: 0 = encode (src -> packed), 1 = decode (packed -> dst), 2 = emulate in place (data = src)
static int tiles_op(int what, const void* src, void* dst, int dt, uint64_t rows, uint64_t cols, uint64_t tile_rows,
                    uint64_t tile_cols, int X, int Y, const uint8_t* max_exp, int threads) {
  const uint64_t n = rows * cols;
  if (n && (!src || !dst || !max_exp)) return ORACLE_ERR_NULL;
  if (int rc = tiles_shape(rows, cols, tile_rows, tile_cols)) return rc;
  int lo, hi;
  if (int rc = block_meta_range(dt, X, Y, &lo, &hi)) return rc;
  Format f0;
  if (int rc = check_format(dt, X, Y, hi, what != 2, &f0)) return rc;
  if (what != 2 && 1 + X + Y > kBlockWidth) return ORACLE_ERR_FORMAT;
  const uint64_t tc_n = (cols + tile_cols - 1) / tile_cols;
  const int W = 1 + X + Y;
  std::vector<uint32_t> codes;
  if (what != 2) codes.resize(n);
  if (what == 1) unpack_groups((const uint8_t*)src, n, W, codes.data(), 0, 0, (n + 7) / 8);
  parallel_ranges(rows, threads, [&](uint64_t r0, uint64_t r1) {
    for (uint64_t r = r0; r < r1; ++r) {
      for (uint64_t c = 0; c < cols; ++c) {
        const uint64_t i = r * cols + c;
        Format f;
        check_format(dt, X, Y, clamp_meta(max_exp[(r / tile_rows) * tc_n + c / tile_cols], lo, hi), what != 2, &f);
        if (what == 0) {
          codes[i] = encode_one(f, load_bits(src, dt, i));
        } else if (what == 1) {
          store_bits(dst, dt, i, decode_one(f, codes[i]));
        } else {
          const uint32_t bits = load_bits(src, dt, i);
          const float x = bits_to_float(bits);
          if (std::isnan(x) || std::isinf(x)) continue;
          const float v = (float)code_magnitude(f, magnitude_code(f, std::fabs((double)x)));
          store_bits(dst, dt, i, float_to_bits(v) | (bits & 0x80000000u));
        }
      }
    }
  });
  if (what == 0) pack_groups(codes.data(), 0, n, W, (uint8_t*)dst, 0, (n + 7) / 8);
  return ORACLE_OK;
}

int exmy_oracle_encode_tiles(const void* src, int dt, uint64_t rows, uint64_t cols, uint64_t tile_rows,
                             uint64_t tile_cols, int X, int Y, const uint8_t* max_exp, uint8_t* dst_packed,
                             int threads) {
  return tiles_op(0, src, dst_packed, dt, rows, cols, tile_rows, tile_cols, X, Y, max_exp, threads);
}

int exmy_oracle_decode_tiles(const uint8_t* src_packed, int dt, uint64_t rows, uint64_t cols, uint64_t tile_rows,
                             uint64_t tile_cols, int X, int Y, const uint8_t* max_exp, void* dst, int threads) {
  return tiles_op(1, src_packed, dst, dt, rows, cols, tile_rows, tile_cols, X, Y, max_exp, threads);
}

int exmy_oracle_emulate_tiles(void* data, int dt, uint64_t rows, uint64_t cols, uint64_t tile_rows,
                              uint64_t tile_cols, int X, int Y, const uint8_t* max_exp, int threads) {
  return tiles_op(2, data, data, dt, rows, cols, tile_rows, tile_cols, X, Y, max_exp, threads);
}

// ---------------------------------------------------------------------------
// Float scaling with maximum exponent 127 (Section 2 "Metadata": an additional
// float32 scaling factor; Section 2.1: this scheme reproduces the largest value
// of the block accurately).  One fp32 scale per block; the codes are those of
// the max_exp = 127 format, whose top binade is [1, 2).

static int scaled_format(int dt, int X, int Y, bool packed, Format* f) {
  if (X < 0 || X > 7) return ORACLE_ERR_FORMAT;
  if (X == 0 && Y == 0) return ORACLE_ERR_FORMAT;  // the only magnitude is 0: nothing to scale
  return check_format(dt, X, Y, 127, packed, f);
}

// A real number r (held exactly in a double) rounded once to nearest, ties to even, onto the bf16 grid
// (8 significant bits, denormals below 2^-126, overflow to Inf), as fp32 bits.
static uint32_t round_to_bf16_bits(double r) {
  if (std::isnan(r) || std::isinf(r) || r == 0.0) return float_to_bits((float)r) & 0xFFFF0000u;
  int e;
  (void)std::frexp(r, &e);                                 // |r| in [2^(e-1), 2^e)
  const int q = std::max(e - 1, -126) - 7;                 // exponent of the bf16 quantum in this binade
  const double k = std::nearbyint(std::ldexp(r, -q));
  return float_to_bits((float)std::ldexp(k, q));           // exact in fp32; 2^128 becomes Inf
}

// The same onto the fp16 grid (11 significant bits, denormals below 2^-14), as the fp32 bits of the half's value.
static uint32_t round_to_half_float_bits(double r) {
  if (std::isnan(r) || std::isinf(r) || r == 0.0) return float_to_bits((float)r);
  int e;
  (void)std::frexp(r, &e);                                 // |r| in [2^(e-1), 2^e)
  const int q = std::max(e - 1, -14) - 10;                 // exponent of the fp16 quantum in this binade
  const double v = std::ldexp(std::nearbyint(std::ldexp(r, -q)), q);
  if (std::fabs(v) >= 65536.0) return float_to_bits(std::copysign(INFINITY, (float)r));  // past the largest half (65504)
  return float_to_bits((float)v);
}

int exmy_oracle_block_scale(const void* src, int dt, uint64_t n, uint64_t block, int X, int Y, float* scale_out) {
  if ((!src || !scale_out) && n) return ORACLE_ERR_NULL;
  if (block == 0 || block % 8) return ORACLE_ERR_FORMAT;
  Format f;
  if (int rc = scaled_format(dt, X, Y, false, &f)) return rc;
  const float vmax = (float)code_magnitude(f, f.cmax);
  const uint64_t nb = (n + block - 1) / block;
  for (uint64_t b = 0; b < nb; ++b) {
    float m = 0.0f;
    for (uint64_t i = b * block; i < std::min(n, (b + 1) * block); ++i) {
      const float a = std::fabs(bits_to_float(load_bits(src, dt, i)));
      if (std::isfinite(a) && a > m) m = a;
    }
    float s = m / vmax;
    if (!(s >= std::ldexp(1.0f, -126))) s = std::ldexp(1.0f, -126);
    scale_out[b] = s;
  }
  return ORACLE_OK;
}

// The bf16 form of the scales: for each block the smallest bf16 value >= the fp32
// scale above, capped at the largest finite bf16; written as bf16 bit patterns.
int exmy_oracle_block_scale_bf16(const void* src, int dt, uint64_t n, uint64_t block, int X, int Y,
                                 uint16_t* scale_out) {
  if ((!src || !scale_out) && n) return ORACLE_ERR_NULL;
  if (block == 0 || block % 8) return ORACLE_ERR_FORMAT;
  const uint64_t nb = (n + block - 1) / block;
  std::vector<float> s32(nb);
  if (int rc = exmy_oracle_block_scale(src, dt, n, block, X, Y, s32.data())) return rc;
  const double bf16_max = std::ldexp(255.0, 127 - 7);  // (2 - 2^-7) * 2^127
  for (uint64_t b = 0; b < nb; ++b) {
    int e;
    (void)std::frexp((double)s32[b], &e);                   // s in [2^(e-1), 2^e), a normal float
    const int q = e - 1 - 7;                                // exponent of the bf16 quantum in this binade
    double up = std::ldexp(std::ceil(std::ldexp((double)s32[b], -q)), q);
    if (up > bf16_max) up = bf16_max;
    scale_out[b] = (uint16_t)(float_to_bits((float)up) >> 16);  // exact: `up` is a bf16 value
  }
  return ORACLE_OK;
}

// what: 0 = encode, 1 = decode, 2 = emulate in place
static int scaled_op(int what, const void* src, void* dst, int dt, uint64_t n, uint64_t block, int X, int Y,
                     const float* scale, int threads) {
  if (n && (!src || !dst || !scale)) return ORACLE_ERR_NULL;
  if (block == 0 || block % 8) return ORACLE_ERR_FORMAT;
  Format f;
  if (int rc = scaled_format(dt, X, Y, what != 2, &f)) return rc;
  if (what != 2 && 1 + X + Y > kBlockWidth) return ORACLE_ERR_FORMAT;
  const uint64_t nb = (n + block - 1) / block;
  const int W = 1 + X + Y;
  std::vector<uint32_t> codes;
  if (what != 2) codes.resize(n);
  if (what == 1) unpack_groups((const uint8_t*)src, n, W, codes.data(), 0, 0, (n + 7) / 8);
  parallel_ranges(nb, threads, [&](uint64_t b0, uint64_t b1) {
    for (uint64_t b = b0; b < b1; ++b) {
      const double s = (double)scale[b];
      for (uint64_t i = b * block; i < std::min(n, (b + 1) * block); ++i) {
        uint32_t code = 0;
        uint32_t bits = 0;
        if (what != 1) {
          bits = load_bits(src, dt, i);
          const float x = bits_to_float(bits);
          // the real quotient |x| / s, to 2^-53: see the header for why that decides the code exactly
          const int64_t c = (std::isnan(x) || std::isinf(x)) ? f.cmax : magnitude_code(f, std::fabs((double)x) / s);
          code = (uint32_t)(((bits >> 31) << (X + Y)) | (uint32_t)c);
        } else {
          code = codes[i];
        }
        if (what == 0) {
          codes[i] = code;
          continue;
        }
        const float x = bits_to_float(bits);
        if (what == 2 && (std::isnan(x) || std::isinf(x))) continue;  // preserved
        // the real product value * s (exact in a double: at most 24 + 24 bits), rounded once into the container
        const double r = code_magnitude(f, code & (uint32_t)((((int64_t)1) << (X + Y)) - 1)) * s;
        uint32_t out = dt == ORACLE_F32 ? float_to_bits((float)r) : (dt == ORACLE_F16 ? round_to_half_float_bits(r) : round_to_bf16_bits(r));
        out |= ((code >> (X + Y)) & 1u) << 31;
        store_bits(dst, dt, i, out);
      }
    }
  });
  if (what == 0) pack_groups(codes.data(), 0, n, W, (uint8_t*)dst, 0, (n + 7) / 8);
  return ORACLE_OK;
}

int exmy_oracle_encode_scaled(const void* src, int dt, uint64_t n, uint64_t block, int X, int Y, const float* scale,
                              uint8_t* dst_packed, int threads) {
  return scaled_op(0, src, dst_packed, dt, n, block, X, Y, scale, threads);
}

int exmy_oracle_decode_scaled(const uint8_t* src_packed, int dt, uint64_t n, uint64_t block, int X, int Y,
                              const float* scale, void* dst, int threads) {
  return scaled_op(1, src_packed, dst, dt, n, block, X, Y, scale, threads);
}

int exmy_oracle_emulate_scaled(void* data, int dt, uint64_t n, uint64_t block, int X, int Y, const float* scale,
                               int threads) {
  return scaled_op(2, data, data, dt, n, block, X, Y, scale, threads);
}

// ---------------------------------------------------------------------------
// Packing along rows (Section 2.2.2, Fig. 2: an array of shape (8R, C) becomes
// arrays of shape (R, C), one per power-of-2 segment).  The matrix is row-major
// with `rows` rows of `cols` elements; R = ceil(rows / 8).  max_exp_rows: one
// metadatum per row of the matrix (Section 2.2.1: the (R, 1) metadata tensor of an
// (R, C) tensor), read with the block-mode range; or null, then `max_exp` holds for
// the whole tensor.

uint64_t exmy_oracle_packed_bytes_rows(uint64_t rows, uint64_t cols, int X, int Y) {
  return ((rows + 7) / 8) * cols * (uint64_t)(1 + X + Y);
}

// what: 0 = encode, 1 = decode
static int rows_op(int what, const void* src, void* dst, int dt, uint64_t rows, uint64_t cols, int X, int Y,
                   int max_exp, const uint8_t* max_exp_rows) {
  const uint64_t n = rows * cols;
  if (n && (!src || !dst)) return ORACLE_ERR_NULL;
  Format f0;
  int lo = 0, hi = 0;
  if (max_exp_rows) {
    if (int rc = block_meta_range(dt, X, Y, &lo, &hi)) return rc;
    if (int rc = check_format(dt, X, Y, hi, true, &f0)) return rc;
  } else {
    if (int rc = check_format(dt, X, Y, max_exp, true, &f0)) return rc;
  }
  const int W = 1 + X + Y;
  if (W > kBlockWidth) return ORACLE_ERR_FORMAT;
  const uint64_t R = (rows + 7) / 8;
  int seg[8];
  const int np = plane_list(W, seg);
  uint8_t* packed = (uint8_t*)(what == 0 ? dst : const_cast<void*>(src));
  for (uint64_t r = 0; r < R; ++r) {
    Format f[8];
    for (int j = 0; j < 8; ++j) {
      f[j] = f0;
      const uint64_t row = 8 * r + j;
      if (max_exp_rows && row < rows) check_format(dt, X, Y, clamp_meta(max_exp_rows[row], lo, hi), true, &f[j]);
    }
    for (uint64_t c = 0; c < cols; ++c) {
      uint32_t code[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      if (what == 0)
        for (int j = 0; j < 8; ++j)
          if (8 * r + j < rows) code[j] = encode_one(f[j], load_bits(src, dt, (8 * r + j) * cols + c));
      // the word of plane p at (r, c): element j at bits [s*j, s*j + s), little-endian bytes
      uint64_t plane_off = 0;
      int lob = 0;
      for (int p = 0; p < np; ++p) {
        const int sb = seg[p];
        uint8_t* word = packed + plane_off + (r * cols + c) * (uint64_t)sb;
        if (what == 0)
          for (int b = 0; b < sb; ++b) word[b] = 0;
        for (int j = 0; j < 8; ++j) {
          for (int b = 0; b < sb; ++b) {
            const int bit = sb * j + b;
            if (what == 0) {
              if ((code[j] >> (lob + b)) & 1u) word[bit / 8] |= (uint8_t)(1u << (bit % 8));
            } else {
              if ((word[bit / 8] >> (bit % 8)) & 1u) code[j] |= 1u << (lob + b);
            }
          }
        }
        plane_off += R * cols * (uint64_t)sb;
        lob += sb;
      }
      if (what == 1)
        for (int j = 0; j < 8; ++j)
          if (8 * r + j < rows) store_bits(dst, dt, (8 * r + j) * cols + c, decode_one(f[j], code[j]));
    }
  }
  return ORACLE_OK;
}

int exmy_oracle_encode_rows(const void* src, int dt, uint64_t rows, uint64_t cols, int X, int Y, int max_exp,
                            const uint8_t* max_exp_rows, uint8_t* dst_packed) {
  return rows_op(0, src, dst_packed, dt, rows, cols, X, Y, max_exp, max_exp_rows);
}

int exmy_oracle_decode_rows(const uint8_t* src_packed, int dt, uint64_t rows, uint64_t cols, int X, int Y,
                            int max_exp, const uint8_t* max_exp_rows, void* dst) {
  return rows_op(1, src_packed, dst, dt, rows, cols, X, Y, max_exp, max_exp_rows);
}

// ---------------------------------------------------------------------------
// Two's complement reading of the X = 0 formats (Section 2 "Format": instead of
// (sign, magnitude) with its double zero, the 1 + Y bits are a two's complement
// number, which gains one encoding: e0m3 as int4 covers [-8, 7]).  The quantum
// is that of e0mY with the same max_exp: 2^(max_exp + 1 - 127 - Y).

static int int_format(int dt, int Y, int max_exp, bool packed, Format* f) {
  if (int rc = check_format(dt, 0, Y, max_exp, packed, f)) return rc;
  if (dt == ORACLE_F16 && max_exp > 141) return ORACLE_ERR_MAX_EXP;  // -2^Y quanta = -2^(max_exp - 126) must be a half
  if (packed && 1 + Y > kBlockWidth) return ORACLE_ERR_FORMAT;
  // -2^Y quanta = -2^(max_exp + 1 - 127) must be a value of the container (it always is), and Y >= 1
  // keeps at least one magnitude bit (with Y = 0 the range would be [-1, 0])
  if (Y < 1) return ORACLE_ERR_FORMAT;
  return ORACLE_OK;
}

static int64_t int_code(const Format& f, uint32_t bits) {
  const float x = bits_to_float(bits);
  const int64_t lo = -((int64_t)1 << f.Y), hi = ((int64_t)1 << f.Y) - 1;
  const bool neg = (bits >> 31) != 0;
  if (std::isnan(x) || std::isinf(x)) return neg ? lo : hi;
  const double k = std::nearbyint(std::ldexp((double)x, -(f.emin8 - 127 - f.Y)));  // x / quantum is exact
  return k < (double)lo ? lo : (k > (double)hi ? hi : (int64_t)k);
}

static float int_value(const Format& f, int64_t k) { return (float)std::ldexp((double)k, f.emin8 - 127 - f.Y); }

int exmy_oracle_to_codes_int(const void* src, int dt, uint64_t n, int Y, int max_exp, uint32_t* codes) {
  if ((!src || !codes) && n) return ORACLE_ERR_NULL;
  Format f;
  if (int rc = int_format(dt, Y, max_exp, true, &f)) return rc;
  for (uint64_t i = 0; i < n; ++i) codes[i] = (uint32_t)int_code(f, load_bits(src, dt, i)) & ((2u << Y) - 1u);
  return ORACLE_OK;
}

int exmy_oracle_from_codes_int(const uint32_t* codes, int dt, uint64_t n, int Y, int max_exp, void* dst) {
  if ((!dst || !codes) && n) return ORACLE_ERR_NULL;
  Format f;
  if (int rc = int_format(dt, Y, max_exp, true, &f)) return rc;
  for (uint64_t i = 0; i < n; ++i) {
    int64_t k = codes[i] & ((2u << Y) - 1u);
    if (k >> Y) k -= (int64_t)2 << Y;  // sign extension of the (1 + Y)-bit number
    store_bits(dst, dt, i, float_to_bits(int_value(f, k)));
  }
  return ORACLE_OK;
}

int exmy_oracle_encode_int(const void* src, int dt, uint64_t n, int Y, int max_exp, uint8_t* dst_packed) {
  if ((!src || !dst_packed) && n) return ORACLE_ERR_NULL;
  std::vector<uint32_t> codes(n);
  if (int rc = exmy_oracle_to_codes_int(src, dt, n, Y, max_exp, codes.data())) return rc;
  pack_groups(codes.data(), 0, n, 1 + Y, dst_packed, 0, (n + 7) / 8);
  return ORACLE_OK;
}

int exmy_oracle_decode_int(const uint8_t* src_packed, int dt, uint64_t n, int Y, int max_exp, void* dst) {
  if ((!src_packed || !dst) && n) return ORACLE_ERR_NULL;
  Format f;
  if (int rc = int_format(dt, Y, max_exp, true, &f)) return rc;
  std::vector<uint32_t> codes(n);
  unpack_groups(src_packed, n, 1 + Y, codes.data(), 0, 0, (n + 7) / 8);
  return exmy_oracle_from_codes_int(codes.data(), dt, n, Y, max_exp, dst);
}

// In place; Inf / NaN are left bit-identical (Section 2.1).
int exmy_oracle_emulate_int(void* data, int dt, uint64_t n, int Y, int max_exp) {
  if (!data && n) return ORACLE_ERR_NULL;
  Format f;
  if (int rc = int_format(dt, Y, max_exp, false, &f)) return rc;
  for (uint64_t i = 0; i < n; ++i) {
    const uint32_t bits = load_bits(data, dt, i);
    const float x = bits_to_float(bits);
    if (std::isnan(x) || std::isinf(x)) continue;
    store_bits(data, dt, i, float_to_bits(int_value(f, int_code(f, bits))));
  }
  return ORACLE_OK;
}

// fp32 -> bf16 / fp16 roundings used above, exported so that they can be pinned on their own.
uint32_t exmy_oracle_round_to_bf16_bits(double r) { return round_to_bf16_bits(r); }
uint32_t exmy_oracle_round_to_half_float_bits(double r) { return round_to_half_float_bits(r); }

}  // extern "C"
