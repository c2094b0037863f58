"""Thin ctypes binding of ``libexmy.so`` (the C ABI of ``include/exmy.h``).

Argument marshalling only: every step of the codec runs in the HIP kernels.
PyTorch is used for device memory and streams.  There is no fallback: if the
library is not built, or a call fails, an exception is raised.
"""
import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libexmy.so")

F32, BF16, F16 = 0, 1, 2
SYMBOLS = [
    "exmy_packed_bytes",
    "exmy_check_format",
    "exmy_encode",
    "exmy_decode",
    "exmy_encode_batch",
    "exmy_decode_batch",
    "exmy_emulate",
    "exmy_exponent_histogram",
    "exmy_encode_with_histogram",
    "exmy_max_exp_from_histogram",
    "exmy_block_count",
    "exmy_block_max_exp",
    "exmy_block_max_exp_after_rounding",
    "exmy_encode_blocks_auto",
    "exmy_encode_blocks",
    "exmy_decode_blocks",
    "exmy_emulate_blocks",
    "exmy_encode_specials",
    "exmy_decode_specials",
    "exmy_emulate_specials",
    "exmy_encode_records",
    "exmy_decode_records",
    "exmy_tile_count",
    "exmy_tile_max_exp",
    "exmy_encode_tiles",
    "exmy_decode_tiles",
    "exmy_emulate_tiles",
    "exmy_block_scale",
    "exmy_encode_scaled",
    "exmy_decode_scaled",
    "exmy_emulate_scaled",
    "exmy_packed_bytes_rows",
    "exmy_encode_rows",
    "exmy_decode_rows",
    "exmy_encode_int",
    "exmy_decode_int",
    "exmy_emulate_int",
    "exmy_status_string",
]

_lib = None


class TensorDesc(ctypes.Structure):
    """exmy_tensor_t"""

    _fields_ = [("src", ctypes.c_void_p), ("dst", ctypes.c_void_p), ("n", ctypes.c_uint64),
                ("max_exp", ctypes.c_int32)]


class ExmyError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("exmy: %s (status %d)" % (text, status))
        self.status = status


def lib():
    """Load the shared library (building it first if it has never been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from . import build as _build

            _build.build()
        L = ctypes.CDLL(LIB_PATH)
        u64, i32, vp, dbl = ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p, ctypes.c_double
        L.exmy_packed_bytes.restype = ctypes.c_size_t
        L.exmy_packed_bytes.argtypes = [u64, i32, i32]
        L.exmy_check_format.restype = i32
        L.exmy_check_format.argtypes = [i32, i32, i32, i32, i32]
        L.exmy_encode.restype = i32
        L.exmy_encode.argtypes = [vp, i32, u64, i32, i32, i32, vp, vp]
        L.exmy_decode.restype = i32
        L.exmy_decode.argtypes = [vp, i32, u64, i32, i32, i32, vp, vp]
        L.exmy_encode_batch.restype = i32
        L.exmy_encode_batch.argtypes = [vp, ctypes.c_size_t, i32, i32, i32, vp]
        L.exmy_decode_batch.restype = i32
        L.exmy_decode_batch.argtypes = [vp, ctypes.c_size_t, i32, i32, i32, vp]
        L.exmy_emulate.restype = i32
        L.exmy_emulate.argtypes = [vp, i32, u64, i32, i32, i32, vp]
        L.exmy_exponent_histogram.restype = i32
        L.exmy_exponent_histogram.argtypes = [vp, i32, u64, vp, vp]
        L.exmy_encode_with_histogram.restype = i32
        L.exmy_encode_with_histogram.argtypes = [vp, i32, u64, i32, i32, i32, vp, vp, vp]
        L.exmy_max_exp_from_histogram.restype = i32
        L.exmy_max_exp_from_histogram.argtypes = [vp, dbl]
        L.exmy_block_count.restype = ctypes.c_size_t
        L.exmy_block_count.argtypes = [u64, u64]
        L.exmy_block_max_exp.restype = i32
        L.exmy_block_max_exp.argtypes = [vp, i32, u64, u64, i32, vp, vp]
        L.exmy_block_max_exp_after_rounding.restype = i32
        L.exmy_block_max_exp_after_rounding.argtypes = [vp, i32, u64, u64, i32, i32, vp, vp]
        L.exmy_encode_blocks_auto.restype = i32
        L.exmy_encode_blocks_auto.argtypes = [vp, i32, u64, u64, i32, i32, i32, vp, vp, vp]
        L.exmy_encode_blocks.restype = i32
        L.exmy_encode_blocks.argtypes = [vp, i32, u64, u64, i32, i32, vp, vp, vp]
        L.exmy_decode_blocks.restype = i32
        L.exmy_decode_blocks.argtypes = [vp, i32, u64, u64, i32, i32, vp, vp, vp]
        L.exmy_emulate_blocks.restype = i32
        L.exmy_emulate_blocks.argtypes = [vp, i32, u64, u64, i32, i32, vp, vp]
        L.exmy_encode_specials.restype = i32
        L.exmy_encode_specials.argtypes = [vp, i32, u64, i32, i32, i32, i32, vp, vp]
        L.exmy_decode_specials.restype = i32
        L.exmy_decode_specials.argtypes = [vp, i32, u64, i32, i32, i32, i32, vp, vp]
        L.exmy_emulate_specials.restype = i32
        L.exmy_emulate_specials.argtypes = [vp, i32, u64, i32, i32, i32, i32, vp]
        L.exmy_encode_records.restype = i32
        L.exmy_encode_records.argtypes = [vp, i32, u64, i32, i32, i32, vp, vp]
        L.exmy_decode_records.restype = i32
        L.exmy_decode_records.argtypes = [vp, i32, u64, i32, i32, i32, vp, vp]
        L.exmy_tile_count.restype = ctypes.c_size_t
        L.exmy_tile_count.argtypes = [u64, u64, u64, u64]
        L.exmy_tile_max_exp.restype = i32
        L.exmy_tile_max_exp.argtypes = [vp, i32, u64, u64, u64, u64, i32, i32, i32, vp, vp]
        L.exmy_encode_tiles.restype = i32
        L.exmy_encode_tiles.argtypes = [vp, i32, u64, u64, u64, u64, i32, i32, vp, vp, vp]
        L.exmy_decode_tiles.restype = i32
        L.exmy_decode_tiles.argtypes = [vp, i32, u64, u64, u64, u64, i32, i32, vp, vp, vp]
        L.exmy_emulate_tiles.restype = i32
        L.exmy_emulate_tiles.argtypes = [vp, i32, u64, u64, u64, u64, i32, i32, vp, vp]
        L.exmy_block_scale.restype = i32
        L.exmy_block_scale.argtypes = [vp, i32, u64, u64, i32, i32, vp, i32, vp]
        L.exmy_encode_scaled.restype = i32
        L.exmy_encode_scaled.argtypes = [vp, i32, u64, u64, i32, i32, vp, i32, vp, vp]
        L.exmy_decode_scaled.restype = i32
        L.exmy_decode_scaled.argtypes = [vp, i32, u64, u64, i32, i32, vp, i32, vp, vp]
        L.exmy_emulate_scaled.restype = i32
        L.exmy_emulate_scaled.argtypes = [vp, i32, u64, u64, i32, i32, vp, i32, vp]
        L.exmy_packed_bytes_rows.restype = ctypes.c_size_t
        L.exmy_packed_bytes_rows.argtypes = [u64, u64, i32, i32]
        L.exmy_encode_rows.restype = i32
        L.exmy_encode_rows.argtypes = [vp, i32, u64, u64, i32, i32, i32, vp, vp, vp]
        L.exmy_decode_rows.restype = i32
        L.exmy_decode_rows.argtypes = [vp, i32, u64, u64, i32, i32, i32, vp, vp, vp]
        L.exmy_encode_int.restype = i32
        L.exmy_encode_int.argtypes = [vp, i32, u64, i32, i32, vp, vp]
        L.exmy_decode_int.restype = i32
        L.exmy_decode_int.argtypes = [vp, i32, u64, i32, i32, vp, vp]
        L.exmy_emulate_int.restype = i32
        L.exmy_emulate_int.argtypes = [vp, i32, u64, i32, i32, vp]
        L.exmy_status_string.restype = ctypes.c_char_p
        L.exmy_status_string.argtypes = [i32]
        _lib = L
    return _lib


def _check(status):
    if status != 0:
        raise ExmyError(status, lib().exmy_status_string(status).decode())


def _dtype_enum(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float16:
        return F16
    raise TypeError("exmy: tensors must be float32, bfloat16 or float16, got %s" % t.dtype)


def _torch_dtype(dt):
    if dt in (F16, torch.float16):
        return torch.float16
    return torch.float32 if dt in (F32, torch.float32) else torch.bfloat16


def _device_tensor(t, name):
    if not t.is_cuda:
        raise ValueError("exmy: %s must be a GPU tensor (no CPU path exists)" % name)
    if not t.is_contiguous():
        raise ValueError("exmy: %s must be contiguous" % name)
    return t


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def packed_bytes(n, X, Y):
    return int(lib().exmy_packed_bytes(n, X, Y))


def check_format(dt, X, Y, max_exp, packed=True):
    """Status code of the host-side validation (0 = valid)."""
    return int(lib().exmy_check_format(dt, X, Y, max_exp, int(packed)))


def status_string(status):
    return lib().exmy_status_string(status).decode()


def encode(src, X, Y, max_exp, out=None):
    """exmy_encode: returns the packed uint8 tensor (``out`` if given)."""
    _device_tensor(src, "src")
    n = src.numel()
    nbytes = packed_bytes(n, X, Y)
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=src.device)
    else:
        _device_tensor(out, "out")
        if out.dtype != torch.uint8 or out.numel() != nbytes:
            raise ValueError("exmy: out must be uint8 with %d elements" % nbytes)
    _check(lib().exmy_encode(src.data_ptr(), _dtype_enum(src), n, X, Y, max_exp, out.data_ptr(), _stream()))
    return out


def decode(packed, dtype, n, X, Y, max_exp, out=None):
    """exmy_decode: returns a flat tensor of ``n`` values of ``dtype``."""
    _device_tensor(packed, "packed")
    tdt = _torch_dtype(dtype)
    if packed.dtype != torch.uint8 or packed.numel() != packed_bytes(n, X, Y):
        raise ValueError("exmy: packed must be uint8 with %d elements" % packed_bytes(n, X, Y))
    if out is None:
        out = torch.empty(n, dtype=tdt, device=packed.device)
    else:
        _device_tensor(out, "out")
        if out.dtype != tdt or out.numel() != n:
            raise ValueError("exmy: out must be %s with %d elements" % (tdt, n))
    _check(lib().exmy_decode(packed.data_ptr(), _dtype_enum(out), n, X, Y, max_exp, out.data_ptr(), _stream()))
    return out


class Batch:
    """A prepared array of exmy_tensor_t descriptors (host memory), reusable across
    calls.  Holds references to the tensors so their memory stays alive."""

    def __init__(self, elems, packeds, max_exps, X, Y, decode=False):
        elems, packeds, max_exps = list(elems), list(packeds), list(max_exps)
        if not (len(elems) == len(packeds) == len(max_exps)):
            raise ValueError("exmy: batch lists differ in length")
        self.count = len(elems)
        self.X, self.Y, self.decode = X, Y, decode
        self.dtype = elems[0].dtype if elems else torch.bfloat16
        self._keep = (elems, packeds)
        self.array = (TensorDesc * max(self.count, 1))()
        for i, (e, p, m) in enumerate(zip(elems, packeds, max_exps)):
            _device_tensor(e, "element tensor")
            _device_tensor(p, "packed tensor")
            if e.dtype != self.dtype:
                raise TypeError("exmy: all tensors of a batch share one dtype")
            if p.dtype != torch.uint8 or p.numel() != packed_bytes(e.numel(), X, Y):
                raise ValueError("exmy: packed tensor %d must be uint8 with %d elements" % (i, packed_bytes(e.numel(), X, Y)))
            d = self.array[i]
            d.src, d.dst = (p.data_ptr(), e.data_ptr()) if decode else (e.data_ptr(), p.data_ptr())
            d.n, d.max_exp = e.numel(), int(m)

    def run(self):
        L = lib()
        fn = L.exmy_decode_batch if self.decode else L.exmy_encode_batch
        dt = _dtype_enum(self._keep[0][0]) if self.count else BF16
        _check(fn(ctypes.cast(self.array, ctypes.c_void_p), self.count, dt, self.X, self.Y, _stream()))


def encode_batch(srcs, X, Y, max_exps, outs=None):
    """exmy_encode_batch over a list of tensors; returns the list of packed tensors."""
    srcs = [s.reshape(-1) for s in srcs]
    if outs is None:
        outs = [torch.empty(packed_bytes(s.numel(), X, Y), dtype=torch.uint8, device=s.device) for s in srcs]
    Batch(srcs, outs, max_exps, X, Y, decode=False).run()
    return outs


def decode_batch(packeds, dtype, ns, X, Y, max_exps, outs=None):
    """exmy_decode_batch over a list of packed tensors; returns the list of decoded tensors."""
    tdt = _torch_dtype(dtype)
    if outs is None:
        outs = [torch.empty(n, dtype=tdt, device=p.device) for p, n in zip(packeds, ns)]
    Batch(outs, packeds, max_exps, X, Y, decode=True).run()
    return outs


def emulate(data, X, Y, max_exp):
    """exmy_emulate: in place; returns ``data``."""
    _device_tensor(data, "data")
    _check(lib().exmy_emulate(data.data_ptr(), _dtype_enum(data), data.numel(), X, Y, max_exp, _stream()))
    return data


def _hist_tensor(hist, device):
    if hist is None:
        return torch.zeros(256, dtype=torch.int64, device=device)
    _device_tensor(hist, "hist")
    if hist.dtype != torch.int64 or hist.numel() != 256:
        raise ValueError("exmy: hist must be int64 with 256 elements")
    return hist


def exponent_histogram(src, hist=None):
    """exmy_exponent_histogram: accumulates into ``hist`` (int64[256] on the GPU;
    a zeroed one is made if None) and returns it."""
    _device_tensor(src, "src")
    hist = _hist_tensor(hist, src.device)
    _check(lib().exmy_exponent_histogram(src.data_ptr(), _dtype_enum(src), src.numel(), hist.data_ptr(), _stream()))
    return hist


def encode_with_histogram(src, X, Y, max_exp, out=None, hist=None):
    """exmy_encode_with_histogram: returns (packed, hist)."""
    _device_tensor(src, "src")
    n = src.numel()
    nbytes = packed_bytes(n, X, Y)
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=src.device)
    else:
        _device_tensor(out, "out")
        if out.dtype != torch.uint8 or out.numel() != nbytes:
            raise ValueError("exmy: out must be uint8 with %d elements" % nbytes)
    hist = _hist_tensor(hist, src.device)
    _check(lib().exmy_encode_with_histogram(src.data_ptr(), _dtype_enum(src), n, X, Y, max_exp, out.data_ptr(),
                                            hist.data_ptr(), _stream()))
    return out, hist


def max_exp_from_histogram(hist, coverage):
    """exmy_max_exp_from_histogram on a host copy of ``hist``."""
    h = hist.detach().to("cpu", torch.int64).contiguous()
    if h.numel() != 256:
        raise ValueError("exmy: hist must have 256 elements")
    return int(lib().exmy_max_exp_from_histogram(h.data_ptr(), float(coverage)))


# ------------------------------------------------------------ per-block metadata


def block_count(n, block):
    return int(lib().exmy_block_count(n, block))


def _meta_tensor(meta, n, block, name="max_exps"):
    _device_tensor(meta, name)
    if meta.dtype != torch.uint8 or meta.numel() != block_count(n, block):
        raise ValueError("exmy: %s must be uint8 with %d elements" % (name, block_count(n, block)))
    return meta


def block_max_exp(src, block, X, out=None):
    """exmy_block_max_exp: returns the uint8 tensor of one max_exp per block."""
    _device_tensor(src, "src")
    n = src.numel()
    if out is None:
        out = torch.empty(block_count(n, block), dtype=torch.uint8, device=src.device)
    else:
        _meta_tensor(out, n, block, "out")
    _check(lib().exmy_block_max_exp(src.data_ptr(), _dtype_enum(src), n, block, X, out.data_ptr(), _stream()))
    return out


BEFORE_ROUNDING, AFTER_ROUNDING = 0, 1


def block_max_exp_after_rounding(src, block, X, Y, out=None):
    """exmy_block_max_exp_after_rounding: returns the uint8 tensor of one max_exp per block."""
    _device_tensor(src, "src")
    n = src.numel()
    if out is None:
        out = torch.empty(block_count(n, block), dtype=torch.uint8, device=src.device)
    else:
        _meta_tensor(out, n, block, "out")
    _check(lib().exmy_block_max_exp_after_rounding(src.data_ptr(), _dtype_enum(src), n, block, X, Y, out.data_ptr(),
                                                   _stream()))
    return out


def encode_blocks_auto(src, block, X, Y, scheme=BEFORE_ROUNDING, max_exps=None, out=None):
    """exmy_encode_blocks_auto: returns (packed, max_exps)."""
    _device_tensor(src, "src")
    n = src.numel()
    if max_exps is None:
        max_exps = torch.empty(block_count(n, block), dtype=torch.uint8, device=src.device)
    else:
        _meta_tensor(max_exps, n, block)
    nbytes = packed_bytes(n, X, Y)
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=src.device)
    else:
        _device_tensor(out, "out")
        if out.dtype != torch.uint8 or out.numel() != nbytes:
            raise ValueError("exmy: out must be uint8 with %d elements" % nbytes)
    _check(lib().exmy_encode_blocks_auto(src.data_ptr(), _dtype_enum(src), n, block, X, Y, int(scheme),
                                         max_exps.data_ptr(), out.data_ptr(), _stream()))
    return out, max_exps


def encode_blocks(src, block, X, Y, max_exps, out=None):
    """exmy_encode_blocks: returns the packed uint8 tensor (``out`` if given)."""
    _device_tensor(src, "src")
    n = src.numel()
    _meta_tensor(max_exps, n, block)
    nbytes = packed_bytes(n, X, Y)
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=src.device)
    else:
        _device_tensor(out, "out")
        if out.dtype != torch.uint8 or out.numel() != nbytes:
            raise ValueError("exmy: out must be uint8 with %d elements" % nbytes)
    _check(lib().exmy_encode_blocks(src.data_ptr(), _dtype_enum(src), n, block, X, Y, max_exps.data_ptr(),
                                    out.data_ptr(), _stream()))
    return out


def decode_blocks(packed, dtype, n, block, X, Y, max_exps, out=None):
    """exmy_decode_blocks: returns a flat tensor of ``n`` values of ``dtype``."""
    _device_tensor(packed, "packed")
    _meta_tensor(max_exps, n, block)
    tdt = _torch_dtype(dtype)
    if packed.dtype != torch.uint8 or packed.numel() != packed_bytes(n, X, Y):
        raise ValueError("exmy: packed must be uint8 with %d elements" % packed_bytes(n, X, Y))
    if out is None:
        out = torch.empty(n, dtype=tdt, device=packed.device)
    else:
        _device_tensor(out, "out")
        if out.dtype != tdt or out.numel() != n:
            raise ValueError("exmy: out must be %s with %d elements" % (tdt, n))
    _check(lib().exmy_decode_blocks(packed.data_ptr(), _dtype_enum(out), n, block, X, Y, max_exps.data_ptr(),
                                    out.data_ptr(), _stream()))
    return out


def emulate_blocks(data, block, X, Y, max_exps):
    """exmy_emulate_blocks: in place; returns ``data``."""
    _device_tensor(data, "data")
    _meta_tensor(max_exps, data.numel(), block)
    _check(lib().exmy_emulate_blocks(data.data_ptr(), _dtype_enum(data), data.numel(), block, X, Y,
                                     max_exps.data_ptr(), _stream()))
    return data


# ------------------------------------------------------------ reserved NaN / Inf code points

SPECIALS_IEEE, SPECIALS_NAN_ONLY = 1, 2


def encode_specials(src, X, Y, max_exp, specials, out=None):
    """exmy_encode_specials: returns the packed uint8 tensor (``out`` if given)."""
    _device_tensor(src, "src")
    n = src.numel()
    nbytes = packed_bytes(n, X, Y)
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=src.device)
    else:
        _device_tensor(out, "out")
        if out.dtype != torch.uint8 or out.numel() != nbytes:
            raise ValueError("exmy: out must be uint8 with %d elements" % nbytes)
    _check(lib().exmy_encode_specials(src.data_ptr(), _dtype_enum(src), n, X, Y, max_exp, int(specials), out.data_ptr(),
                                      _stream()))
    return out


def decode_specials(packed, dtype, n, X, Y, max_exp, specials, out=None):
    """exmy_decode_specials: returns a flat tensor of ``n`` values of ``dtype``."""
    _device_tensor(packed, "packed")
    tdt = _torch_dtype(dtype)
    if packed.dtype != torch.uint8 or packed.numel() != packed_bytes(n, X, Y):
        raise ValueError("exmy: packed must be uint8 with %d elements" % packed_bytes(n, X, Y))
    if out is None:
        out = torch.empty(n, dtype=tdt, device=packed.device)
    else:
        _device_tensor(out, "out")
        if out.dtype != tdt or out.numel() != n:
            raise ValueError("exmy: out must be %s with %d elements" % (tdt, n))
    _check(lib().exmy_decode_specials(packed.data_ptr(), _dtype_enum(out), n, X, Y, max_exp, int(specials),
                                      out.data_ptr(), _stream()))
    return out


def emulate_specials(data, X, Y, max_exp, specials):
    """exmy_emulate_specials: in place; returns ``data``."""
    _device_tensor(data, "data")
    _check(lib().exmy_emulate_specials(data.data_ptr(), _dtype_enum(data), data.numel(), X, Y, max_exp, int(specials),
                                       _stream()))
    return data


# ------------------------------------------------------------ records (W bytes per group)


def encode_records(src, X, Y, max_exp, out=None):
    """exmy_encode_records: returns the uint8 tensor of records (``out`` if given)."""
    _device_tensor(src, "src")
    n = src.numel()
    nbytes = packed_bytes(n, X, Y)
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=src.device)
    else:
        _device_tensor(out, "out")
        if out.dtype != torch.uint8 or out.numel() != nbytes:
            raise ValueError("exmy: out must be uint8 with %d elements" % nbytes)
    _check(lib().exmy_encode_records(src.data_ptr(), _dtype_enum(src), n, X, Y, max_exp, out.data_ptr(), _stream()))
    return out


def decode_records(records, dtype, n, X, Y, max_exp, out=None):
    """exmy_decode_records: returns a flat tensor of ``n`` values of ``dtype``."""
    _device_tensor(records, "records")
    tdt = _torch_dtype(dtype)
    if records.dtype != torch.uint8 or records.numel() != packed_bytes(n, X, Y):
        raise ValueError("exmy: records must be uint8 with %d elements" % packed_bytes(n, X, Y))
    if out is None:
        out = torch.empty(n, dtype=tdt, device=records.device)
    else:
        _device_tensor(out, "out")
        if out.dtype != tdt or out.numel() != n:
            raise ValueError("exmy: out must be %s with %d elements" % (tdt, n))
    _check(lib().exmy_decode_records(records.data_ptr(), _dtype_enum(out), n, X, Y, max_exp, out.data_ptr(), _stream()))
    return out


# ------------------------------------------------------------ blocks that are columns or 2-D tiles


def tile_count(rows, cols, tile_rows, tile_cols):
    return int(lib().exmy_tile_count(rows, cols, tile_rows, tile_cols))


def _matrix(t, name):
    _device_tensor(t, name)
    if t.dim() != 2:
        raise ValueError("exmy: %s must be a 2-D tensor" % name)
    return t.shape[0], t.shape[1]


def _tile_meta_tensor(meta, rows, cols, tile_rows, tile_cols, name="max_exps"):
    _device_tensor(meta, name)
    if meta.dtype != torch.uint8 or meta.numel() != tile_count(rows, cols, tile_rows, tile_cols):
        raise ValueError("exmy: %s must be uint8 with %d elements" % (name, tile_count(rows, cols, tile_rows, tile_cols)))
    return meta


def tile_max_exp(src, tile_rows, tile_cols, X, Y=0, scheme=BEFORE_ROUNDING, out=None):
    """exmy_tile_max_exp: returns the flat uint8 tensor of one max_exp per tile, row-major over the tiles."""
    rows, cols = _matrix(src, "src")
    if out is None:
        out = torch.empty(tile_count(rows, cols, tile_rows, tile_cols), dtype=torch.uint8, device=src.device)
    else:
        _tile_meta_tensor(out, rows, cols, tile_rows, tile_cols, "out")
    _check(lib().exmy_tile_max_exp(src.data_ptr(), _dtype_enum(src), rows, cols, tile_rows, tile_cols, X, Y, int(scheme),
                                   out.data_ptr(), _stream()))
    return out


def encode_tiles(src, tile_rows, tile_cols, X, Y, max_exps, out=None):
    """exmy_encode_tiles: returns the packed uint8 tensor (``out`` if given)."""
    rows, cols = _matrix(src, "src")
    _tile_meta_tensor(max_exps, rows, cols, tile_rows, tile_cols)
    nbytes = packed_bytes(rows * cols, X, Y)
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=src.device)
    else:
        _device_tensor(out, "out")
        if out.dtype != torch.uint8 or out.numel() != nbytes:
            raise ValueError("exmy: out must be uint8 with %d elements" % nbytes)
    _check(lib().exmy_encode_tiles(src.data_ptr(), _dtype_enum(src), rows, cols, tile_rows, tile_cols, X, Y,
                                   max_exps.data_ptr(), out.data_ptr(), _stream()))
    return out


def decode_tiles(packed, dtype, rows, cols, tile_rows, tile_cols, X, Y, max_exps, out=None):
    """exmy_decode_tiles: returns a (rows, cols) tensor of ``dtype``."""
    _device_tensor(packed, "packed")
    _tile_meta_tensor(max_exps, rows, cols, tile_rows, tile_cols)
    tdt = _torch_dtype(dtype)
    if packed.dtype != torch.uint8 or packed.numel() != packed_bytes(rows * cols, X, Y):
        raise ValueError("exmy: packed must be uint8 with %d elements" % packed_bytes(rows * cols, X, Y))
    if out is None:
        out = torch.empty((rows, cols), dtype=tdt, device=packed.device)
    else:
        _device_tensor(out, "out")
        if out.dtype != tdt or tuple(out.shape) != (rows, cols):
            raise ValueError("exmy: out must be %s of shape (%d, %d)" % (tdt, rows, cols))
    _check(lib().exmy_decode_tiles(packed.data_ptr(), _dtype_enum(out), rows, cols, tile_rows, tile_cols, X, Y,
                                   max_exps.data_ptr(), out.data_ptr(), _stream()))
    return out


def emulate_tiles(data, tile_rows, tile_cols, X, Y, max_exps):
    """exmy_emulate_tiles: in place; returns ``data``."""
    rows, cols = _matrix(data, "data")
    _tile_meta_tensor(max_exps, rows, cols, tile_rows, tile_cols)
    _check(lib().exmy_emulate_tiles(data.data_ptr(), _dtype_enum(data), rows, cols, tile_rows, tile_cols, X, Y,
                                    max_exps.data_ptr(), _stream()))
    return data


# ------------------------------------------------------------ float scaling, max_exp = 127


def _scale_tensor(scale, n, block, name="scales"):
    _device_tensor(scale, name)
    if scale.dtype not in (torch.float32, torch.bfloat16) or scale.numel() != block_count(n, block):
        raise ValueError("exmy: %s must be float32 or bfloat16 with %d elements" % (name, block_count(n, block)))
    return scale


def block_scale(src, block, X, Y, out=None, scale_dtype=torch.float32):
    """exmy_block_scale: returns the tensor of one scale per block (``scale_dtype``: float32 or bfloat16)."""
    _device_tensor(src, "src")
    n = src.numel()
    if out is None:
        out = torch.empty(block_count(n, block), dtype=scale_dtype, device=src.device)
    _scale_tensor(out, n, block, "out")
    _check(lib().exmy_block_scale(src.data_ptr(), _dtype_enum(src), n, block, X, Y, out.data_ptr(), _dtype_enum(out),
                                  _stream()))
    return out


def encode_scaled(src, block, X, Y, scales, out=None):
    """exmy_encode_scaled: returns the packed uint8 tensor (``out`` if given)."""
    _device_tensor(src, "src")
    n = src.numel()
    _scale_tensor(scales, n, block)
    nbytes = packed_bytes(n, X, Y)
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=src.device)
    else:
        _device_tensor(out, "out")
        if out.dtype != torch.uint8 or out.numel() != nbytes:
            raise ValueError("exmy: out must be uint8 with %d elements" % nbytes)
    _check(lib().exmy_encode_scaled(src.data_ptr(), _dtype_enum(src), n, block, X, Y, scales.data_ptr(),
                                    _dtype_enum(scales), out.data_ptr(), _stream()))
    return out


def decode_scaled(packed, dtype, n, block, X, Y, scales, out=None):
    """exmy_decode_scaled: returns a flat tensor of ``n`` values of ``dtype``."""
    _device_tensor(packed, "packed")
    _scale_tensor(scales, n, block)
    tdt = _torch_dtype(dtype)
    if packed.dtype != torch.uint8 or packed.numel() != packed_bytes(n, X, Y):
        raise ValueError("exmy: packed must be uint8 with %d elements" % packed_bytes(n, X, Y))
    if out is None:
        out = torch.empty(n, dtype=tdt, device=packed.device)
    else:
        _device_tensor(out, "out")
        if out.dtype != tdt or out.numel() != n:
            raise ValueError("exmy: out must be %s with %d elements" % (tdt, n))
    _check(lib().exmy_decode_scaled(packed.data_ptr(), _dtype_enum(out), n, block, X, Y, scales.data_ptr(),
                                    _dtype_enum(scales), out.data_ptr(), _stream()))
    return out


def emulate_scaled(data, block, X, Y, scales):
    """exmy_emulate_scaled: in place; returns ``data``."""
    _device_tensor(data, "data")
    _scale_tensor(scales, data.numel(), block)
    _check(lib().exmy_emulate_scaled(data.data_ptr(), _dtype_enum(data), data.numel(), block, X, Y,
                                     scales.data_ptr(), _dtype_enum(scales), _stream()))
    return data


# ------------------------------------------------------------ packing along rows


def packed_bytes_rows(rows, cols, X, Y):
    return int(lib().exmy_packed_bytes_rows(rows, cols, X, Y))


def _row_meta_ptr(max_exp_rows, rows):
    if max_exp_rows is None:
        return None
    _device_tensor(max_exp_rows, "max_exp_rows")
    if max_exp_rows.dtype != torch.uint8 or max_exp_rows.numel() != rows:
        raise ValueError("exmy: max_exp_rows must be uint8 with %d elements" % rows)
    return max_exp_rows.data_ptr()


def encode_rows(src, X, Y, max_exp=0, max_exp_rows=None, out=None):
    """exmy_encode_rows on a 2-D tensor (rows, cols); returns the packed uint8 tensor."""
    _device_tensor(src, "src")
    if src.dim() != 2:
        raise ValueError("exmy: src must be a matrix")
    rows, cols = src.shape
    nbytes = packed_bytes_rows(rows, cols, X, Y)
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=src.device)
    else:
        _device_tensor(out, "out")
        if out.dtype != torch.uint8 or out.numel() != nbytes:
            raise ValueError("exmy: out must be uint8 with %d elements" % nbytes)
    _check(lib().exmy_encode_rows(src.data_ptr(), _dtype_enum(src), rows, cols, X, Y, max_exp,
                                  _row_meta_ptr(max_exp_rows, rows), out.data_ptr(), _stream()))
    return out


def decode_rows(packed, dtype, rows, cols, X, Y, max_exp=0, max_exp_rows=None, out=None):
    """exmy_decode_rows: returns a (rows, cols) tensor of ``dtype``."""
    _device_tensor(packed, "packed")
    tdt = _torch_dtype(dtype)
    if packed.dtype != torch.uint8 or packed.numel() != packed_bytes_rows(rows, cols, X, Y):
        raise ValueError("exmy: packed must be uint8 with %d elements" % packed_bytes_rows(rows, cols, X, Y))
    if out is None:
        out = torch.empty((rows, cols), dtype=tdt, device=packed.device)
    else:
        _device_tensor(out, "out")
        if out.dtype != tdt or tuple(out.shape) != (rows, cols):
            raise ValueError("exmy: out must be %s of shape (%d, %d)" % (tdt, rows, cols))
    _check(lib().exmy_decode_rows(packed.data_ptr(), _dtype_enum(out), rows, cols, X, Y, max_exp,
                                  _row_meta_ptr(max_exp_rows, rows), out.data_ptr(), _stream()))
    return out


# ------------------------------------------------------------ two's complement reading of X = 0


def encode_int(src, Y, max_exp, out=None):
    """exmy_encode_int: returns the packed uint8 tensor of (1 + Y)-bit two's complement codes."""
    _device_tensor(src, "src")
    n = src.numel()
    nbytes = packed_bytes(n, 0, Y)
    if out is None:
        out = torch.empty(nbytes, dtype=torch.uint8, device=src.device)
    else:
        _device_tensor(out, "out")
        if out.dtype != torch.uint8 or out.numel() != nbytes:
            raise ValueError("exmy: out must be uint8 with %d elements" % nbytes)
    _check(lib().exmy_encode_int(src.data_ptr(), _dtype_enum(src), n, Y, max_exp, out.data_ptr(), _stream()))
    return out


def decode_int(packed, dtype, n, Y, max_exp, out=None):
    """exmy_decode_int: returns a flat tensor of ``n`` values of ``dtype``."""
    _device_tensor(packed, "packed")
    tdt = _torch_dtype(dtype)
    if packed.dtype != torch.uint8 or packed.numel() != packed_bytes(n, 0, Y):
        raise ValueError("exmy: packed must be uint8 with %d elements" % packed_bytes(n, 0, Y))
    if out is None:
        out = torch.empty(n, dtype=tdt, device=packed.device)
    else:
        _device_tensor(out, "out")
        if out.dtype != tdt or out.numel() != n:
            raise ValueError("exmy: out must be %s with %d elements" % (tdt, n))
    _check(lib().exmy_decode_int(packed.data_ptr(), _dtype_enum(out), n, Y, max_exp, out.data_ptr(), _stream()))
    return out


def emulate_int(data, Y, max_exp):
    """exmy_emulate_int: in place; returns ``data``."""
    _device_tensor(data, "data")
    _check(lib().exmy_emulate_int(data.data_ptr(), _dtype_enum(data), data.numel(), Y, max_exp, _stream()))
    return data
