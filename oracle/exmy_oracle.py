"""ctypes binding of the scalar C++ oracle (``exmy_oracle.cpp``).

Test infrastructure only.  Arrays are numpy: fp32 tensors as ``float32`` (or
``uint32`` bit patterns), bf16 tensors as ``uint16`` bit patterns.
"""
import ctypes
import os

import numpy as np

from . import build as _build

F32, BF16, F16 = 0, 1, 2
_STATUS = {0: "ok", 1: "null pointer", 2: "bad format", 3: "bad max_exp"}

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        L = ctypes.CDLL(path)
        u64, i32, vp, dbl = ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p, ctypes.c_double
        L.exmy_oracle_packed_bytes.restype = u64
        L.exmy_oracle_packed_bytes.argtypes = [u64, i32, i32]
        L.exmy_oracle_check_format.restype = i32
        L.exmy_oracle_check_format.argtypes = [i32, i32, i32, i32, i32]
        L.exmy_oracle_code_value.restype = dbl
        L.exmy_oracle_code_value.argtypes = [i32, i32, i32, ctypes.c_uint32]
        L.exmy_oracle_to_codes.argtypes = [vp, i32, u64, i32, i32, i32, vp, i32]
        L.exmy_oracle_from_codes.argtypes = [vp, i32, u64, i32, i32, i32, vp, i32]
        L.exmy_oracle_pack.argtypes = [vp, u64, i32, vp, i32]
        L.exmy_oracle_unpack.argtypes = [vp, u64, i32, vp, i32]
        L.exmy_oracle_encode.argtypes = [vp, i32, u64, i32, i32, i32, vp, i32]
        L.exmy_oracle_decode.argtypes = [vp, i32, u64, i32, i32, i32, vp, i32]
        L.exmy_oracle_emulate.argtypes = [vp, i32, u64, i32, i32, i32, i32]
        L.exmy_oracle_exponent_histogram.argtypes = [vp, i32, u64, vp]
        L.exmy_oracle_encode_specials.argtypes = [vp, i32, u64, i32, i32, i32, i32, vp]
        L.exmy_oracle_decode_specials.argtypes = [vp, i32, u64, i32, i32, i32, i32, vp]
        L.exmy_oracle_emulate_specials.argtypes = [vp, i32, u64, i32, i32, i32, i32]
        L.exmy_oracle_encode_records.argtypes = [vp, i32, u64, i32, i32, i32, vp]
        L.exmy_oracle_decode_records.argtypes = [vp, i32, u64, i32, i32, i32, vp]
        L.exmy_oracle_block_max_exp.argtypes = [vp, i32, u64, u64, i32, vp]
        L.exmy_oracle_block_max_exp_after_rounding.argtypes = [vp, i32, u64, u64, i32, i32, vp]
        L.exmy_oracle_encode_blocks.argtypes = [vp, i32, u64, u64, i32, i32, vp, vp, i32]
        L.exmy_oracle_decode_blocks.argtypes = [vp, i32, u64, u64, i32, i32, vp, vp, i32]
        L.exmy_oracle_emulate_blocks.argtypes = [vp, i32, u64, u64, i32, i32, vp, i32]
        L.exmy_oracle_tile_max_exp.argtypes = [vp, i32, u64, u64, u64, u64, i32, i32, i32, vp]
        L.exmy_oracle_encode_tiles.argtypes = [vp, i32, u64, u64, u64, u64, i32, i32, vp, vp, i32]
        L.exmy_oracle_decode_tiles.argtypes = [vp, i32, u64, u64, u64, u64, i32, i32, vp, vp, i32]
        L.exmy_oracle_emulate_tiles.argtypes = [vp, i32, u64, u64, u64, u64, i32, i32, vp, i32]
        L.exmy_oracle_block_scale.argtypes = [vp, i32, u64, u64, i32, i32, vp]
        L.exmy_oracle_block_scale_bf16.argtypes = [vp, i32, u64, u64, i32, i32, vp]
        L.exmy_oracle_encode_scaled.argtypes = [vp, i32, u64, u64, i32, i32, vp, vp, i32]
        L.exmy_oracle_decode_scaled.argtypes = [vp, i32, u64, u64, i32, i32, vp, vp, i32]
        L.exmy_oracle_emulate_scaled.argtypes = [vp, i32, u64, u64, i32, i32, vp, i32]
        L.exmy_oracle_round_to_bf16_bits.restype = ctypes.c_uint32
        L.exmy_oracle_round_to_bf16_bits.argtypes = [ctypes.c_double]
        L.exmy_oracle_round_to_half_float_bits.restype = ctypes.c_uint32
        L.exmy_oracle_round_to_half_float_bits.argtypes = [ctypes.c_double]
        L.exmy_oracle_packed_bytes_rows.restype = u64
        L.exmy_oracle_packed_bytes_rows.argtypes = [u64, u64, i32, i32]
        L.exmy_oracle_encode_rows.argtypes = [vp, i32, u64, u64, i32, i32, i32, vp, vp]
        L.exmy_oracle_decode_rows.argtypes = [vp, i32, u64, u64, i32, i32, i32, vp, vp]
        L.exmy_oracle_to_codes_int.argtypes = [vp, i32, u64, i32, i32, vp]
        L.exmy_oracle_from_codes_int.argtypes = [vp, i32, u64, i32, i32, vp]
        L.exmy_oracle_encode_int.argtypes = [vp, i32, u64, i32, i32, vp]
        L.exmy_oracle_decode_int.argtypes = [vp, i32, u64, i32, i32, vp]
        L.exmy_oracle_emulate_int.argtypes = [vp, i32, u64, i32, i32]
        L.exmy_oracle_max_exp_from_histogram.restype = i32
        L.exmy_oracle_max_exp_from_histogram.argtypes = [vp, dbl]
        _lib = L
    return _lib


class OracleError(ValueError):
    pass


def _check(rc):
    if rc != 0:
        raise OracleError(_STATUS.get(rc, "status %d" % rc))


def default_threads():
    return len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)


def _src(a):
    """Return (contiguous array, dtype enum) for an fp32 / bf16-bits array."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float32 or a.dtype == np.uint32:
        return a, F32
    if a.dtype == np.uint16:
        return a, BF16
    if a.dtype == np.float16:
        return a, F16
    raise TypeError("expected float32/uint32 (fp32), uint16 (bf16 bits) or float16, got %s" % a.dtype)


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _out_dtype(dt):
    return np.float32 if dt == F32 else (np.float16 if dt == F16 else np.uint16)


def packed_bytes(n, X, Y):
    return int(lib().exmy_oracle_packed_bytes(n, X, Y))


def check_format(dt, X, Y, max_exp, packed=True):
    return int(lib().exmy_oracle_check_format(dt, X, Y, max_exp, int(packed)))


def code_value(X, Y, max_exp, code):
    return float(lib().exmy_oracle_code_value(X, Y, max_exp, int(code)))


def to_codes(src, X, Y, max_exp, threads=1):
    a, dt = _src(src)
    codes = np.empty(a.size, dtype=np.uint32)
    _check(lib().exmy_oracle_to_codes(_ptr(a), dt, a.size, X, Y, max_exp, _ptr(codes), threads))
    return codes


def from_codes(codes, dt, X, Y, max_exp, threads=1):
    codes = np.ascontiguousarray(codes, dtype=np.uint32)
    out = np.empty(codes.size, dtype=_out_dtype(dt))
    _check(lib().exmy_oracle_from_codes(_ptr(codes), dt, codes.size, X, Y, max_exp, _ptr(out), threads))
    return out


def pack(codes, W, threads=1):
    codes = np.ascontiguousarray(codes, dtype=np.uint32)
    out = np.empty(((codes.size + 7) // 8) * W, dtype=np.uint8)
    _check(lib().exmy_oracle_pack(_ptr(codes), codes.size, W, _ptr(out), threads))
    return out


def unpack(packed, n, W, threads=1):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    assert packed.size == ((n + 7) // 8) * W
    codes = np.empty(n, dtype=np.uint32)
    _check(lib().exmy_oracle_unpack(_ptr(packed), n, W, _ptr(codes), threads))
    return codes


def encode(src, X, Y, max_exp, threads=1):
    a, dt = _src(src)
    out = np.empty(packed_bytes(a.size, X, Y), dtype=np.uint8)
    _check(lib().exmy_oracle_encode(_ptr(a), dt, a.size, X, Y, max_exp, _ptr(out), threads))
    return out


def decode(packed, dt, n, X, Y, max_exp, threads=1):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    assert packed.size == packed_bytes(n, X, Y)
    out = np.empty(n, dtype=_out_dtype(dt))
    _check(lib().exmy_oracle_decode(_ptr(packed), dt, n, X, Y, max_exp, _ptr(out), threads))
    return out


def encode_records(src, X, Y, max_exp):
    """The plane words of each group as one record of W bytes, records in group order."""
    a, dt = _src(src)
    out = np.empty(packed_bytes(a.size, X, Y), dtype=np.uint8)
    _check(lib().exmy_oracle_encode_records(_ptr(a), dt, a.size, X, Y, max_exp, _ptr(out)))
    return out


def decode_records(records, dt, n, X, Y, max_exp):
    records = np.ascontiguousarray(records, dtype=np.uint8)
    assert records.size == packed_bytes(n, X, Y)
    out = np.empty(n, dtype=_out_dtype(dt))
    _check(lib().exmy_oracle_decode_records(_ptr(records), dt, n, X, Y, max_exp, _ptr(out)))
    return out


IEEE, NAN_ONLY = 1, 2


def encode_specials(src, X, Y, max_exp, specials):
    """Codes with reserved NaN / Inf code points (specials: IEEE or NAN_ONLY), planar layout."""
    a, dt = _src(src)
    out = np.empty(packed_bytes(a.size, X, Y), dtype=np.uint8)
    _check(lib().exmy_oracle_encode_specials(_ptr(a), dt, a.size, X, Y, max_exp, specials, _ptr(out)))
    return out


def decode_specials(packed, dt, n, X, Y, max_exp, specials):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    assert packed.size == packed_bytes(n, X, Y)
    out = np.empty(n, dtype=_out_dtype(dt))
    _check(lib().exmy_oracle_decode_specials(_ptr(packed), dt, n, X, Y, max_exp, specials, _ptr(out)))
    return out


def emulate_specials(src, X, Y, max_exp, specials):
    a, dt = _src(src)
    out = a.copy()
    _check(lib().exmy_oracle_emulate_specials(_ptr(out), dt, out.size, X, Y, max_exp, specials))
    return out


def emulate(src, X, Y, max_exp, threads=1):
    """Returns a new array; the input is left alone."""
    a, dt = _src(src)
    out = a.copy()
    _check(lib().exmy_oracle_emulate(_ptr(out), dt, out.size, X, Y, max_exp, threads))
    return out


def exponent_histogram(src, hist=None):
    a, dt = _src(src)
    if hist is None:
        hist = np.zeros(256, dtype=np.uint64)
    _check(lib().exmy_oracle_exponent_histogram(_ptr(a), dt, a.size, _ptr(hist)))
    return hist


def max_exp_from_histogram(hist, coverage):
    hist = np.ascontiguousarray(hist, dtype=np.uint64)
    assert hist.size == 256
    return int(lib().exmy_oracle_max_exp_from_histogram(_ptr(hist), float(coverage)))


# ------------------------------------------------------------ per-block metadata


def block_max_exp(src, block, X):
    a, dt = _src(src)
    out = np.empty((a.size + block - 1) // block, dtype=np.uint8)
    _check(lib().exmy_oracle_block_max_exp(_ptr(a), dt, a.size, block, X, _ptr(out)))
    return out


def block_max_exp_after_rounding(src, block, X, Y):
    a, dt = _src(src)
    out = np.empty((a.size + block - 1) // block, dtype=np.uint8)
    _check(lib().exmy_oracle_block_max_exp_after_rounding(_ptr(a), dt, a.size, block, X, Y, _ptr(out)))
    return out


def _meta(max_exp, n, block):
    m = np.ascontiguousarray(max_exp, dtype=np.uint8)
    assert m.size == (n + block - 1) // block
    return m


def encode_blocks(src, block, X, Y, max_exp, threads=1):
    a, dt = _src(src)
    m = _meta(max_exp, a.size, block)
    out = np.empty(packed_bytes(a.size, X, Y), dtype=np.uint8)
    _check(lib().exmy_oracle_encode_blocks(_ptr(a), dt, a.size, block, X, Y, _ptr(m), _ptr(out), threads))
    return out


def decode_blocks(packed, dt, n, block, X, Y, max_exp, threads=1):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    assert packed.size == packed_bytes(n, X, Y)
    m = _meta(max_exp, n, block)
    out = np.empty(n, dtype=_out_dtype(dt))
    _check(lib().exmy_oracle_decode_blocks(_ptr(packed), dt, n, block, X, Y, _ptr(m), _ptr(out), threads))
    return out


def emulate_blocks(src, block, X, Y, max_exp, threads=1):
    a, dt = _src(src)
    m = _meta(max_exp, a.size, block)
    out = a.copy()
    _check(lib().exmy_oracle_emulate_blocks(_ptr(out), dt, out.size, block, X, Y, _ptr(m), threads))
    return out


# ------------------------------------------------------------ blocks that are columns or 2-D tiles


def tile_count(rows, cols, tile_rows, tile_cols):
    return ((rows + tile_rows - 1) // tile_rows) * ((cols + tile_cols - 1) // tile_cols)


def _matrix(src):
    a, dt = _src(src)
    assert a.ndim == 2
    return a, dt


def tile_max_exp(src, tile_rows, tile_cols, X, Y=0, after_rounding=False):
    """src: 2-D array.  Returns the row-major (ceil(rows/tile_rows), ceil(cols/tile_cols)) metadata, flat."""
    a, dt = _matrix(src)
    rows, cols = a.shape
    out = np.empty(tile_count(rows, cols, tile_rows, tile_cols), dtype=np.uint8)
    _check(lib().exmy_oracle_tile_max_exp(_ptr(a), dt, rows, cols, tile_rows, tile_cols, X, Y, int(after_rounding), _ptr(out)))
    return out


def _tile_meta(max_exp, rows, cols, tile_rows, tile_cols):
    m = np.ascontiguousarray(max_exp, dtype=np.uint8).reshape(-1)
    assert m.size == tile_count(rows, cols, tile_rows, tile_cols)
    return m


def encode_tiles(src, tile_rows, tile_cols, X, Y, max_exp, threads=1):
    a, dt = _matrix(src)
    rows, cols = a.shape
    m = _tile_meta(max_exp, rows, cols, tile_rows, tile_cols)
    out = np.empty(packed_bytes(a.size, X, Y), dtype=np.uint8)
    _check(lib().exmy_oracle_encode_tiles(_ptr(a), dt, rows, cols, tile_rows, tile_cols, X, Y, _ptr(m), _ptr(out), threads))
    return out


def decode_tiles(packed, dt, rows, cols, tile_rows, tile_cols, X, Y, max_exp, threads=1):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    assert packed.size == packed_bytes(rows * cols, X, Y)
    m = _tile_meta(max_exp, rows, cols, tile_rows, tile_cols)
    out = np.empty((rows, cols), dtype=_out_dtype(dt))
    _check(lib().exmy_oracle_decode_tiles(_ptr(packed), dt, rows, cols, tile_rows, tile_cols, X, Y, _ptr(m), _ptr(out), threads))
    return out


def emulate_tiles(src, tile_rows, tile_cols, X, Y, max_exp, threads=1):
    a, dt = _matrix(src)
    rows, cols = a.shape
    m = _tile_meta(max_exp, rows, cols, tile_rows, tile_cols)
    out = a.copy()
    _check(lib().exmy_oracle_emulate_tiles(_ptr(out), dt, rows, cols, tile_rows, tile_cols, X, Y, _ptr(m), threads))
    return out


# ------------------------------------------------------------ float scaling, max_exp = 127


def _scales(scale, n, block):
    """fp32 scales as they are; bf16 scales (uint16 bit patterns) widened exactly to fp32."""
    scale = np.asarray(scale)
    if scale.dtype == np.uint16:
        s = (scale.astype(np.uint32) << 16).view(np.float32)
    else:
        s = np.ascontiguousarray(scale, dtype=np.float32)
    assert s.size == (n + block - 1) // block
    return np.ascontiguousarray(s)


def block_scale(src, block, X, Y, bf16=False):
    """One scale per block: float32 values, or with ``bf16`` the uint16 bit patterns of bf16 scales."""
    a, dt = _src(src)
    nb = (a.size + block - 1) // block
    if bf16:
        out = np.empty(nb, dtype=np.uint16)
        _check(lib().exmy_oracle_block_scale_bf16(_ptr(a), dt, a.size, block, X, Y, _ptr(out)))
        return out
    out = np.empty(nb, dtype=np.float32)
    _check(lib().exmy_oracle_block_scale(_ptr(a), dt, a.size, block, X, Y, _ptr(out)))
    return out


def encode_scaled(src, block, X, Y, scale, threads=1):
    a, dt = _src(src)
    s = _scales(scale, a.size, block)
    out = np.empty(packed_bytes(a.size, X, Y), dtype=np.uint8)
    _check(lib().exmy_oracle_encode_scaled(_ptr(a), dt, a.size, block, X, Y, _ptr(s), _ptr(out), threads))
    return out


def decode_scaled(packed, dt, n, block, X, Y, scale, threads=1):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    assert packed.size == packed_bytes(n, X, Y)
    s = _scales(scale, n, block)
    out = np.empty(n, dtype=_out_dtype(dt))
    _check(lib().exmy_oracle_decode_scaled(_ptr(packed), dt, n, block, X, Y, _ptr(s), _ptr(out), threads))
    return out


def emulate_scaled(src, block, X, Y, scale, threads=1):
    a, dt = _src(src)
    s = _scales(scale, a.size, block)
    out = a.copy()
    _check(lib().exmy_oracle_emulate_scaled(_ptr(out), dt, out.size, block, X, Y, _ptr(s), threads))
    return out


def round_to_half_float_bits(r):
    return int(lib().exmy_oracle_round_to_half_float_bits(float(r)))


def round_to_bf16_bits(r):
    return int(lib().exmy_oracle_round_to_bf16_bits(float(r)))


# ------------------------------------------------------------ packing along rows


def packed_bytes_rows(rows, cols, X, Y):
    return int(lib().exmy_oracle_packed_bytes_rows(rows, cols, X, Y))


def _row_meta(max_exp_rows, rows):
    if max_exp_rows is None:
        return None
    m = np.ascontiguousarray(max_exp_rows, dtype=np.uint8)
    assert m.size == rows
    return m


def encode_rows(src, rows, cols, X, Y, max_exp=0, max_exp_rows=None):
    a, dt = _src(src)
    assert a.size == rows * cols
    m = _row_meta(max_exp_rows, rows)
    out = np.empty(packed_bytes_rows(rows, cols, X, Y), dtype=np.uint8)
    _check(lib().exmy_oracle_encode_rows(_ptr(a), dt, rows, cols, X, Y, max_exp, _ptr(m) if m is not None else None,
                                         _ptr(out)))
    return out


def decode_rows(packed, dt, rows, cols, X, Y, max_exp=0, max_exp_rows=None):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    assert packed.size == packed_bytes_rows(rows, cols, X, Y)
    m = _row_meta(max_exp_rows, rows)
    out = np.empty(rows * cols, dtype=_out_dtype(dt))
    _check(lib().exmy_oracle_decode_rows(_ptr(packed), dt, rows, cols, X, Y, max_exp,
                                         _ptr(m) if m is not None else None, _ptr(out)))
    return out


# ------------------------------------------------------------ two's complement reading of X = 0


def to_codes_int(src, Y, max_exp):
    a, dt = _src(src)
    out = np.empty(a.size, dtype=np.uint32)
    _check(lib().exmy_oracle_to_codes_int(_ptr(a), dt, a.size, Y, max_exp, _ptr(out)))
    return out


def from_codes_int(codes, dt, Y, max_exp):
    codes = np.ascontiguousarray(codes, dtype=np.uint32)
    out = np.empty(codes.size, dtype=_out_dtype(dt))
    _check(lib().exmy_oracle_from_codes_int(_ptr(codes), dt, codes.size, Y, max_exp, _ptr(out)))
    return out


def encode_int(src, Y, max_exp):
    a, dt = _src(src)
    out = np.empty(packed_bytes(a.size, 0, Y), dtype=np.uint8)
    _check(lib().exmy_oracle_encode_int(_ptr(a), dt, a.size, Y, max_exp, _ptr(out)))
    return out


def decode_int(packed, dt, n, Y, max_exp):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    assert packed.size == packed_bytes(n, 0, Y)
    out = np.empty(n, dtype=_out_dtype(dt))
    _check(lib().exmy_oracle_decode_int(_ptr(packed), dt, n, Y, max_exp, _ptr(out)))
    return out


def emulate_int(src, Y, max_exp):
    a, dt = _src(src)
    out = a.copy()
    _check(lib().exmy_oracle_emulate_int(_ptr(out), dt, out.size, Y, max_exp))
    return out
