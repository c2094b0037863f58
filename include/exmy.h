/*
 * exmy.h - C ABI of the MI355X (gfx950) eXmY tensor codec.
 *
 * eXmY (arxiv 2405.13938) is a float format with 1 sign bit, X exponent bits
 * and Y mantissa bits, any width W = 1 + X + Y, subnormals, a software-defined
 * exponent bias and no code points reserved for Inf / NaN (Section 2 "Format",
 * "Subnormals", "Exponent Bias"; Section 5).  This library converts bf16 / fp32
 * tensors to packed W-bit codes and back, and emulates the format in place.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - All data pointers are DEVICE pointers owned by the caller.  The library
 *    allocates and frees no device memory and never synchronises: work is enqueued
 *    on `stream` (a hipStream_t passed as void*; NULL = the default stream) and
 *    the call returns at once.  Arguments are validated on the host before any
 *    launch; a failed validation launches nothing.
 *  - Element pointers and packed pointers must be 16-byte aligned.
 *  - `max_exp` is the paper's metadatum (Section 2 "Metadata"): the biased
 *    (bias 127, as in fp32 / bf16) exponent that the top exponent code of the
 *    format stands for.  The paper's exponent bias is 2^X - 1 + 127 - max_exp.
 *    Valid: 2^X - 1 <= max_exp <= 254 for 1 <= X <= 7; 0 <= max_exp <= 253 for
 *    X = 0 (and >= 1 when Y is one more than the container's mantissa);
 *    max_exp = 255 exactly for X = 8 (identity exponent map).
 *  - A format fits a container when X <= 8 and Y <= 7 (bf16) / 23 (fp32), or
 *    X <= 5 and Y <= 10 (fp16) (Section 2.1); with X = 0 one more mantissa bit
 *    is allowed.  With the fp16 container (EXMY_F16) max_exp must also keep the
 *    format's top binade and its quantum inside fp16: max_exp <= 142 and
 *    max_exp - 2^X + 2 - 127 - Y >= -24 (EXMY_ERR_MAX_EXP), so that every
 *    decoded value is an fp16 value (e5m10 therefore has no valid max_exp, and
 *    float scaling, whose formats sit at max_exp = 127, needs Y + 2^X <= 26);
 *    per-block metadata bytes are read as the nearest value of that narrower
 *    range; the exponent histogram of fp16 data bins the exponent of the value
 *    as an fp32.  Packed codes
 *    are limited to W <= 32 (segments of 16, 8, 4, 2 and 1 bits; widths above
 *    16 need the fp32 container; 32 is e8m23 alone, one 32-bit segment: the
 *    packed form is then the array of codes, which are the elements' own bits
 *    with Inf / NaN clamped) in exmy_encode / exmy_decode and their batch
 *    and histogram forms, and to W <= 16 in the per-block, float-scaling and
 *    row-packing entry points.  e0m24 has no packed form (use e1m23, which it
 *    equals bit for bit).
 *  - Rounding is round-to-nearest-even to Y mantissa bits (Section 2
 *    "Rounding"); a tie goes to the even multiple of the quantum of the value's
 *    binade.  Values under the smallest normal are rounded on the subnormal
 *    grid and may flush to (signed) zero; values over the largest normal
 *    saturate to it (Section 2.1).
 *  - Code bit order: sign at bit W-1, then exponent, mantissa in the low Y
 *    bits.
 *
 * Packed layout (Section 2.2.2 "Power-of-2 Decomposition", Fig. 2)
 * ----------------------------------------------------------------
 *  Elements are taken in groups of 8 consecutive values; G = ceil(n / 8); a
 *  ragged last group is padded with zero codes.  W is split into its powers of
 *  two, s_0 > s_1 > ... (7 = 4 + 2 + 1).  Walking the code from bit 0 upwards,
 *  the widest segment takes the lowest bits.  Plane p is an array of G
 *  little-endian words of s_p bytes (8 elements x s_p bits), element j of the
 *  group at bits [s_p*j, s_p*j + s_p).  The planes lie back to back, widest
 *  first: total G * W bytes.  For W = 7: G int32, then G int16, then G int8.
 *  A shard [a, b) of the elements (a, b multiples of 8) is the slice
 *  [a/8, b/8) of every plane.
 */
#ifndef EXMY_H_
#define EXMY_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { EXMY_F32 = 0, EXMY_BF16 = 1, EXMY_F16 = 2 } exmy_dtype_t;

typedef enum {
  EXMY_OK = 0,
  EXMY_ERR_NULL = 1,    /* a required pointer is NULL (and n > 0) */
  EXMY_ERR_FORMAT = 2,  /* X, Y, W or dtype out of domain, or the dtype cannot hold the format */
  EXMY_ERR_MAX_EXP = 3, /* max_exp outside the range valid for X */
  EXMY_ERR_COUNT = 4,   /* n above EXMY_MAX_ELEMENTS */
  EXMY_ERR_ALIGN = 5,   /* a pointer is not 16-byte aligned */
  EXMY_ERR_DEVICE = 6,  /* the HIP runtime reported an error at launch */
  EXMY_ERR_BLOCK = 7,   /* metadata block size not a multiple of 8 in [8, EXMY_MAX_BLOCK] */
  EXMY_ERR_SHAPE = 8    /* matrices: cols not a multiple of 8 or above EXMY_MAX_COLS, rows above EXMY_MAX_ROWS */
} exmy_status_t;

#define EXMY_MAX_ELEMENTS ((uint64_t)1 << 40)
#define EXMY_MAX_BLOCK ((uint64_t)1 << 31)
#define EXMY_MAX_COLS ((uint64_t)1 << 26)
#define EXMY_MAX_ROWS ((uint64_t)1 << 31)

/* Bytes of the packed form of n elements: ceil(n / 8) * (1 + X + Y)
 * (perfect compression, Section 2.2.2).  Host only; no validation. */
size_t exmy_packed_bytes(uint64_t n, int X, int Y);

/* Host-side validation of (dtype, X, Y, max_exp) as described above.  `packed`
 * non-zero also applies the W <= 32 limit of the packed form. */
exmy_status_t exmy_check_format(exmy_dtype_t dt, int X, int Y, int max_exp, int packed);

/* Encode (Sections 2.2.1 + 2.2.2 fused): round n elements of type dt at `src`
 * to eXmY codes and write the packed planes to `dst_packed`
 * (exmy_packed_bytes(n, X, Y) bytes).  +-Inf and NaN become sign + largest
 * magnitude code.  src and dst_packed must not overlap. */
exmy_status_t exmy_encode(const void* src, exmy_dtype_t dt, uint64_t n, int X, int Y, int max_exp,
                          void* dst_packed, void* stream);

/* Decode (inverse of the above): unpack n codes from `src_packed` and write
 * their values as type dt_out to `dst` (n elements).  Every code is a finite
 * value, exactly representable in dt_out.  With X = 8 an exponent code of 255
 * decodes to the largest finite value. */
exmy_status_t exmy_decode(const void* src_packed, exmy_dtype_t dt_out, uint64_t n, int X, int Y, int max_exp,
                          void* dst, void* stream);

/* One tensor of a batched call.  For exmy_encode_batch `src` holds n elements
 * and `dst` receives exmy_packed_bytes(n, X, Y) bytes; for exmy_decode_batch
 * `src` holds the packed bytes and `dst` receives n elements.  Both are device
 * pointers, 16-byte aligned; the array of descriptors itself is HOST memory and
 * is read before the call returns. */
typedef struct {
  const void* src;
  void* dst;
  uint64_t n;
  int32_t max_exp; /* this tensor's metadatum (Section 2 "Metadata": one per block; here block = tensor) */
} exmy_tensor_t;

/* exmy_encode / exmy_decode over `count` tensors that share dtype, X and Y but
 * carry their own max_exp: a checkpoint-shaped stream (the paper names tensor
 * and checkpoint codecs) enqueued as a few launches instead of one per tensor,
 * so that small tensors do not pay a launch each.  Results are identical to
 * calling the single-tensor entry point on every tensor in order.  All tensors
 * are validated first; on any error nothing is launched.  Tensors with n = 0 are
 * skipped. */
exmy_status_t exmy_encode_batch(const exmy_tensor_t* tensors, size_t count, exmy_dtype_t dt, int X, int Y,
                                void* stream);
exmy_status_t exmy_decode_batch(const exmy_tensor_t* tensors, size_t count, exmy_dtype_t dt_out, int X, int Y,
                                void* stream);

/* Emulate (Section 2.1): replace each of the n elements at `data_inout` by the
 * eXmY value nearest to it, kept in the same type; NaN and +-Inf are left
 * bit-identical.  No width limit beyond the container's (Y <= 7 / 23). */
exmy_status_t exmy_emulate(void* data_inout, exmy_dtype_t dt, uint64_t n, int X, int Y, int max_exp, void* stream);

/* 256-bin histogram of the biased exponent field (Section 3.1, Fig. 3): +-0 and
 * denormals count in bin 0, Inf / NaN in bin 255.  ACCUMULATES into
 * hist256_dev (256 uint64 on the device, 8-byte aligned): the caller zeroes it. */
exmy_status_t exmy_exponent_histogram(const void* src, exmy_dtype_t dt, uint64_t n, uint64_t* hist256_dev,
                                      void* stream);

/* exmy_encode and exmy_exponent_histogram in one pass over src. */
exmy_status_t exmy_encode_with_histogram(const void* src, exmy_dtype_t dt, uint64_t n, int X, int Y, int max_exp,
                                         void* dst_packed, uint64_t* hist256_dev, void* stream);

/* ---------------------------------------------------------------------------
 * Per-block metadata (Section 2 "Metadata" and "Block Size"; Section 2.2.1: the
 * encoded tensor is the codes plus one 8-bit max_exp per block).
 *
 * The n elements are cut into consecutive blocks of `block` elements; the last
 * block may be short; there are exmy_block_count(n, block) of them.  With a
 * row-major matrix, block = the row length gives per-row (per-channel)
 * metadata, a divisor of it gives sub-row blocks (e.g. 32 or 64 elements).
 * `block` is a multiple of 8 in [8, EXMY_MAX_BLOCK], else EXMY_ERR_BLOCK;
 * every such size runs at the same rate (a block need not be a power of two).
 *
 * max_exp_dev is a DEVICE array of one byte per block.  Valid metadata here is
 * 2^X <= max_exp <= 254 for 1 <= X <= 7 and 1 <= max_exp <= 253 for X = 0 (the
 * smallest binade of every block is then a normal of the container); bytes
 * outside are read as the nearest valid value, so no byte is an error.  X = 8
 * has nothing for a block to choose and is EXMY_ERR_FORMAT here.  The packed
 * layout is the per-tensor one: block b's codes are groups
 * [b*block/8, (b+1)*block/8) of every plane.  Results equal the per-tensor
 * entry points applied to each block with its own max_exp.
 * Pointers, alignment, n = 0, streams and errors as for exmy_encode. */

/* Number of blocks (bytes of metadata): ceil(n / block); 0 if block = 0.  Host only. */
size_t exmy_block_count(uint64_t n, uint64_t block);

/* "Maximum exponent before rounding" (Section 2 "Metadata"): max_exp_dev[b] =
 * the largest biased exponent among the finite elements of block b (0 if none),
 * brought into the valid range for X given above.  Writes every byte. */
exmy_status_t exmy_block_max_exp(const void* src, exmy_dtype_t dt, uint64_t n, uint64_t block, int X,
                                 uint8_t* max_exp_dev, void* stream);

/* "Maximum exponent after rounding" (Section 2 "Metadata"; Section 2.1: with
 * it 3.9 in e2m1 always becomes 4.0): as above, but the block's largest finite
 * magnitude is first rounded to nearest (ties to even) to the mantissa width
 * of the format's top binade (Y bits; Y - 1 for X = 0), so the block maximum
 * is rounded like any other value and never cut off by saturation.  Differs
 * from the scheme above (by +1) only where that rounding carries into the next
 * binade.  No width limit on Y beyond the container's. */
exmy_status_t exmy_block_max_exp_after_rounding(const void* src, exmy_dtype_t dt, uint64_t n, uint64_t block, int X,
                                                int Y, uint8_t* max_exp_dev, void* stream);

/* exmy_encode / exmy_decode / exmy_emulate with block b using max_exp_dev[b]. */
exmy_status_t exmy_encode_blocks(const void* src, exmy_dtype_t dt, uint64_t n, uint64_t block, int X, int Y,
                                 const uint8_t* max_exp_dev, void* dst_packed, void* stream);
exmy_status_t exmy_decode_blocks(const void* src_packed, exmy_dtype_t dt_out, uint64_t n, uint64_t block, int X,
                                 int Y, const uint8_t* max_exp_dev, void* dst, void* stream);
exmy_status_t exmy_emulate_blocks(void* data_inout, exmy_dtype_t dt, uint64_t n, uint64_t block, int X, int Y,
                                  const uint8_t* max_exp_dev, void* stream);

/* The pipeline of Section 2.2.1 in one call: the metadata of `scheme` is
 * computed from src into max_exp_dev (an OUTPUT here, one byte per block; the
 * bytes are already inside the range valid for (X, Y) and the container) and
 * src is encoded with it.  Blocks of 8, 16, ..., 512 elements and blocks of 520
 * to 65536 (16-bit types) / 32768 (fp32) elements take one launch that reads src
 * from memory once (the block stays in registers, the longest ones in the L2
 * cache, between the two steps); other sizes take two
 * launches on `stream` and read src twice.  Same results either way. */
typedef enum { EXMY_MAX_EXP_BEFORE_ROUNDING = 0, EXMY_MAX_EXP_AFTER_ROUNDING = 1 } exmy_scheme_t;
exmy_status_t exmy_encode_blocks_auto(const void* src, exmy_dtype_t dt, uint64_t n, uint64_t block, int X, int Y,
                                      exmy_scheme_t scheme, uint8_t* max_exp_dev, void* dst_packed, void* stream);

/* ---------------------------------------------------------------------------
 * Reserved code points for NaN and Inf (Section 5 "Limitations": values encoded
 * for training need an encoding for these, which the paper leaves open).  The two
 * conventions of the float types in use are offered:
 *   EXMY_SPECIALS_IEEE      the top exponent code is reserved (as in fp32, bf16,
 *                           fp16, e5m2): mantissa 0 under it is Inf, any other
 *                           mantissa NaN; X >= 1 (X = 8 is allowed: e8m7 is then
 *                           bf16 itself).  The finite values are those of the
 *                           plain format without its top binade;
 *   EXMY_SPECIALS_NAN_ONLY  only the all-ones magnitude code is reserved (as in
 *                           OCP e4m3): it is NaN, there is no Inf; X <= 7,
 *                           X + Y >= 1.  The finite values are those of the plain
 *                           format without its largest one.
 * max_exp keeps its meaning (the exponent of the top exponent code, reserved or
 * not; e5m2 with IEEE bias 15 is max_exp 143, OCP e4m3 with bias 7 is 135).
 * Encode: finite elements round as in exmy_encode and saturate to the largest
 * finite value (Section 2.1), NaN takes the all-ones magnitude code under its own
 * sign, Inf the Inf code or (NaN only) the largest finite code.  Decode: finite
 * codes as in exmy_decode; reserved codes give Inf or the quiet NaN (0x7FC00000,
 * 0x7FC0, 0x7E00 in fp32 / bf16 / fp16) under the code's sign.  Emulate leaves
 * Inf / NaN bit-identical and saturates finite elements.  Planar layout of
 * exmy_encode, W <= 16 (emulate: any width); everything else as there. */
typedef enum { EXMY_SPECIALS_IEEE = 1, EXMY_SPECIALS_NAN_ONLY = 2 } exmy_specials_t;
exmy_status_t exmy_encode_specials(const void* src, exmy_dtype_t dt, uint64_t n, int X, int Y, int max_exp,
                                   exmy_specials_t specials, void* dst_packed, void* stream);
exmy_status_t exmy_decode_specials(const void* src_packed, exmy_dtype_t dt_out, uint64_t n, int X, int Y, int max_exp,
                                   exmy_specials_t specials, void* dst, void* stream);
exmy_status_t exmy_emulate_specials(void* data_inout, exmy_dtype_t dt, uint64_t n, int X, int Y, int max_exp,
                                    exmy_specials_t specials, void* stream);

/* ---------------------------------------------------------------------------
 * Records: the plane words of Section 2.2.2 / Fig. 2 in another order.  The
 * words of one group follow each other, widest segment first, as one record of
 * W = 1 + X + Y bytes, and the records follow each other in group order: for
 * W = 7, bytes 0-3 of record g are the int32 word of the group's low nibbles,
 * bytes 4-5 its int16 word, byte 6 its int8 word ("8 values in 7 bytes").  One
 * stream instead of one per segment; the shard [a, b) of the elements (a, b
 * multiples of 8) is the byte range [a / 8 * W, b / 8 * W).  This is not a
 * layout of the paper; the words are the paper's.  Size exmy_packed_bytes(n, X,
 * Y); W <= 16 (for W = 8 and 16, which have one segment, records and planes
 * coincide); everything else (formats, max_exp, rounding, Inf / NaN, n not a
 * multiple of 8, pointers, alignment, errors, stream) as exmy_encode /
 * exmy_decode. */
exmy_status_t exmy_encode_records(const void* src, exmy_dtype_t dt, uint64_t n, int X, int Y, int max_exp,
                                  void* dst_records, void* stream);
exmy_status_t exmy_decode_records(const void* src_records, exmy_dtype_t dt_out, uint64_t n, int X, int Y, int max_exp,
                                  void* dst, void* stream);

/* ---------------------------------------------------------------------------
 * Blocks that are columns or 2-D tiles: the block shapes of Section 2 "Block
 * Size" that are not runs of consecutive elements.
 *
 * src is a row-major matrix of `rows` rows of `cols` elements.  Tile (i, j)
 * covers rows [i * tile_rows, (i + 1) * tile_rows) and columns
 * [j * tile_cols, (j + 1) * tile_cols), cut off at the matrix edges; its
 * metadatum is byte i * ceil(cols / tile_cols) + j of max_exp_dev
 * (exmy_tile_count(...) bytes, row-major over the tiles).  A column is the tile
 * (rows, 1), a part of a column (k, 1), a row (1, cols), a sub row (1, k); tile
 * sizes beyond the matrix mean "all of it".  The codes are packed in the flat
 * layout of the matrix in memory, exactly as exmy_encode packs its rows * cols
 * elements (groups of 8 consecutive elements, which lie inside one row because
 * cols is a multiple of 8); metadata bytes are read as in exmy_encode_blocks
 * (same valid range, clamped; X <= 7, codes of at most 16 bits).
 *
 * cols is a multiple of 8, at most EXMY_MAX_COLS, rows at most EXMY_MAX_ROWS
 * (EXMY_ERR_SHAPE); tile_rows >= 1; tile_cols is 1, a multiple of 8, or >= cols
 * (EXMY_ERR_BLOCK); rows * cols <= EXMY_MAX_ELEMENTS; rows = 0 or cols = 0 is
 * a no-op.  All arrays, max_exp_dev included, are DEVICE memory aligned to 16
 * bytes.  exmy_tile_max_exp writes the metadata under either scheme of Section
 * 2 "Metadata" (Y is used by the "after rounding" scheme only) in up to three
 * launches on `stream`: it clears the array's whole 4-byte words, folds partial
 * maxima into them with 32-bit atomic operations, and computes the 1-3 bytes
 * of a last partial word (a tile count that is not a multiple of 4) one
 * workgroup per tile with byte stores; no byte outside the exmy_tile_count(...)
 * bytes of max_exp_dev is read or written.  Tiles
 * that are runs of consecutive elements (tile_cols >= cols, or tile_rows = 1
 * with tile_cols dividing cols) take the kernels of the consecutive-block entry
 * points above. */
size_t exmy_tile_count(uint64_t rows, uint64_t cols, uint64_t tile_rows, uint64_t tile_cols);
exmy_status_t exmy_tile_max_exp(const void* src, exmy_dtype_t dt, uint64_t rows, uint64_t cols, uint64_t tile_rows,
                                uint64_t tile_cols, int X, int Y, exmy_scheme_t scheme, uint8_t* max_exp_dev,
                                void* stream);
exmy_status_t exmy_encode_tiles(const void* src, exmy_dtype_t dt, uint64_t rows, uint64_t cols, uint64_t tile_rows,
                                uint64_t tile_cols, int X, int Y, const uint8_t* max_exp_dev, void* dst_packed,
                                void* stream);
exmy_status_t exmy_decode_tiles(const void* src_packed, exmy_dtype_t dt_out, uint64_t rows, uint64_t cols,
                                uint64_t tile_rows, uint64_t tile_cols, int X, int Y, const uint8_t* max_exp_dev,
                                void* dst, void* stream);
exmy_status_t exmy_emulate_tiles(void* data_inout, exmy_dtype_t dt, uint64_t rows, uint64_t cols, uint64_t tile_rows,
                                 uint64_t tile_cols, int X, int Y, const uint8_t* max_exp_dev, void* stream);

/* ---------------------------------------------------------------------------
 * Float scaling with maximum exponent 127 (Section 2 "Metadata": an additional
 * bfloat16 or float32 scaling factor; Section 2.1: the third scheme of the
 * emulation example, which reproduces the largest value of a block accurately).
 *
 * Every block has one scale in the DEVICE array scale_dev
 * (exmy_block_count(n, block) entries of type scale_dt: EXMY_F32, 4-byte
 * aligned, or EXMY_BF16, 2-byte aligned; EXMY_F16 gives EXMY_ERR_FORMAT)
 * instead of a metadata byte; the codes are those of the format with
 * max_exp = 127, whose top binade is [1, 2).  The paper prints no formulas;
 * this library computes:
 *   scale   s = max(m / vmax, FLT_MIN) rounded once to fp32, m = largest finite
 *               |x| of the block (0 if none), vmax = largest value of the format
 *               at max_exp = 127; a bf16 scale is the smallest bf16 value >= s
 *               (so the block maximum still lands on the largest code), at most
 *               the largest finite bf16;
 *   encode  the code, in that format, of the real quotient |x| / s (nearest
 *           grid point, ties to even, saturating), under the sign of x
 *           (Inf / NaN: sign + largest magnitude code, as in exmy_encode);
 *   decode  the real product value * s rounded once, to nearest even, to dt;
 *   emulate decode(encode(x)) with Inf / NaN left bit-identical.
 * A bf16 scale enters this arithmetic widened exactly to fp32.  Scales given to
 * encode / decode / emulate need not come from exmy_block_scale but must be
 * finite and >= FLT_MIN (else the result is unspecified, without any fault).
 * 1 <= X <= 7 or (X = 0, Y >= 1); block, layout, pointers, n = 0, streams and
 * errors as for the entry points above. */
exmy_status_t exmy_block_scale(const void* src, exmy_dtype_t dt, uint64_t n, uint64_t block, int X, int Y,
                               void* scale_dev, exmy_dtype_t scale_dt, void* stream);
exmy_status_t exmy_encode_scaled(const void* src, exmy_dtype_t dt, uint64_t n, uint64_t block, int X, int Y,
                                 const void* scale_dev, exmy_dtype_t scale_dt, void* dst_packed, void* stream);
exmy_status_t exmy_decode_scaled(const void* src_packed, exmy_dtype_t dt_out, uint64_t n, uint64_t block, int X,
                                 int Y, const void* scale_dev, exmy_dtype_t scale_dt, void* dst, void* stream);
exmy_status_t exmy_emulate_scaled(void* data_inout, exmy_dtype_t dt, uint64_t n, uint64_t block, int X, int Y,
                                  const void* scale_dev, exmy_dtype_t scale_dt, void* stream);

/* ---------------------------------------------------------------------------
 * Packing along rows (Section 2.2.2 and Fig. 2: an array of shape (8R, C) is
 * packed into one array of shape (R, C) per power-of-2 segment).
 *
 * src is a row-major matrix of `rows` rows of `cols` elements.  The group of
 * output position (r, c) is the 8 elements (8r + j, c), j = 0..7; element j
 * sits at bits [s*j, s*j + s) of the plane word as in the layout above.
 * R = ceil(rows / 8); rows past the end count as zero codes.  Each plane is a
 * row-major (R, C) array of little-endian words of s bytes; the planes lie
 * back to back, widest first: exmy_packed_bytes_rows = R * cols * W bytes.
 * Rows [8a, 8b) of the matrix are rows [a, b) of every plane, columns
 * [a, b) are columns [a, b) of every plane: the matrix can be sharded either
 * way before or after packing.
 * Metadata: max_exp_rows_dev == NULL: `max_exp` holds for the whole tensor
 * (range as for exmy_encode, X = 8 included).  Else it is a DEVICE array of
 * one byte per row of the matrix (Section 2.2.1: the (R, 1) metadata tensor of
 * an (R, C) tensor), read as for exmy_encode_blocks (exmy_block_max_exp with
 * block = cols computes it), and `max_exp` is ignored.
 * cols must be a multiple of 8 and at most EXMY_MAX_COLS (EXMY_ERR_SHAPE);
 * rows * cols <= EXMY_MAX_ELEMENTS.  Values and codes equal those of the
 * entry points above; only the grouping differs.  Pointers, alignment, empty
 * input, streams and errors as for exmy_encode. */
size_t exmy_packed_bytes_rows(uint64_t rows, uint64_t cols, int X, int Y);
exmy_status_t exmy_encode_rows(const void* src, exmy_dtype_t dt, uint64_t rows, uint64_t cols, int X, int Y,
                               int max_exp, const uint8_t* max_exp_rows_dev, void* dst_packed, void* stream);
exmy_status_t exmy_decode_rows(const void* src_packed, exmy_dtype_t dt_out, uint64_t rows, uint64_t cols, int X,
                               int Y, int max_exp, const uint8_t* max_exp_rows_dev, void* dst, void* stream);

/* ---------------------------------------------------------------------------
 * Two's complement reading of the X = 0 formats (Section 2 "Format": e0m3 read
 * as a two's complement number is int4 and represents [-8, 7], one encoding
 * more than the (sign, magnitude) form with its double zero).
 *
 * The W = 1 + Y bits of a code are a two's complement integer k in
 * [-2^Y, 2^Y - 1]; the value is k quanta, the quantum being that of e0mY with
 * the same max_exp: 2^(max_exp + 1 - 127 - Y) (max_exp = 126 + Y makes it 1).
 * encode: k = round-half-even(x / quantum), clamped to the range; +-Inf and NaN
 * go to the end of the range on the side of their sign bit; -0 and negative
 * values that round to 0 give k = 0.  decode: k * quantum (k = 0 is +0).
 * emulate: decode(encode(x)), Inf / NaN left bit-identical.  Packed layout as
 * for exmy_encode with W = 1 + Y.
 * 1 <= Y <= 8 (bf16) / 11 (fp16) / 21 (fp32), 1 + Y <= 16 for the packed form;
 * 0 <= max_exp <= min(253, 230 + Y), and 102 + Y <= max_exp <= 141 inside fp16
 * (EXMY_ERR_MAX_EXP).  Pointers, alignment,
 * n = 0, streams and errors as for exmy_encode. */
exmy_status_t exmy_encode_int(const void* src, exmy_dtype_t dt, uint64_t n, int Y, int max_exp, void* dst_packed,
                              void* stream);
exmy_status_t exmy_decode_int(const void* src_packed, exmy_dtype_t dt_out, uint64_t n, int Y, int max_exp, void* dst,
                              void* stream);
exmy_status_t exmy_emulate_int(void* data_inout, exmy_dtype_t dt, uint64_t n, int Y, int max_exp, void* stream);

/* Host helper for Section 3.1's technique (keep the top exponents, let the
 * tail go): the smallest biased exponent e in [0, 254] such that at least
 * `coverage` (0..1) of the finite elements counted in the HOST array
 * hist256_host have an exponent <= e.  Returns -1 when no finite element was
 * counted or the pointer is NULL. */
int exmy_max_exp_from_histogram(const uint64_t* hist256_host, double coverage);

const char* exmy_status_string(exmy_status_t status);

#ifdef __cplusplus
}
#endif

#endif /* EXMY_H_ */
