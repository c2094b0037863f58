"""CPU-only checks of the C-ABI library: it loads, exports every symbol that
include/exmy.h declares, and its host-side logic (sizes, validation, error
codes, the histogram helper) agrees with the oracle.  No kernel is launched."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import exmy_oracle as O
from paper_2405_13938_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "exmy.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(exmy_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert set(names) == set(B.SYMBOLS)
    L = B.lib()
    for name in names:
        assert getattr(L, name) is not None


def test_packed_bytes():
    for n in (0, 1, 7, 8, 9, 1 << 20, (1 << 40) - 3):
        for X, Y in ((3, 3), (0, 2), (8, 7), (4, 0)):
            assert B.packed_bytes(n, X, Y) == ((n + 7) // 8) * (1 + X + Y) == O.packed_bytes(n, X, Y)
    assert B.packed_bytes(1 << 20, 3, 3) == 917504  # configuration 1


def test_format_validation_matches_oracle_over_the_whole_domain():
    for dt in (B.F32, B.BF16, B.F16):
        for X in range(-1, 10):
            for Y in range(-1, 26):
                for max_exp in (-1, 0, 1, (1 << max(X, 0)) - 2, (1 << max(X, 0)) - 1, 100 + Y + (1 << max(X, 0)),
                                101 + Y + (1 << max(X, 0)), 102 + Y, 127, 142, 143, 253, 254, 255, 256):
                    for packed in (False, True):
                        got = B.check_format(dt, X, Y, max_exp, packed)
                        want = O.check_format(dt, X, Y, max_exp, packed)
                        assert (got == 0) == (want == 0), (dt, X, Y, max_exp, packed)
                        if got and want:
                            assert got == want, (dt, X, Y, max_exp, packed)  # same error class (format / max_exp)


def test_error_codes_without_launch():
    L = B.lib()
    ok_ptr = ctypes.c_void_p(0x1000)
    odd_ptr = ctypes.c_void_p(0x1004)
    assert L.exmy_encode(ok_ptr, B.F32, 0, 3, 3, 130, ok_ptr, None) == 0  # n = 0: nothing to do
    assert L.exmy_encode(None, B.F32, 8, 3, 3, 130, ok_ptr, None) == 1
    assert L.exmy_decode(ok_ptr, B.F32, 8, 3, 3, 130, None, None) == 1
    assert L.exmy_emulate(None, B.BF16, 8, 3, 3, 130, None) == 1
    assert L.exmy_encode(ok_ptr, B.F32, 8, 9, 3, 130, ok_ptr, None) == 2
    assert L.exmy_encode(ok_ptr, 7, 8, 3, 3, 130, ok_ptr, None) == 2
    assert L.exmy_encode(ok_ptr, B.BF16, 8, 3, 8, 130, ok_ptr, None) == 2  # bf16 cannot hold 8 mantissa bits
    assert L.exmy_encode(ok_ptr, B.F32, 0, 4, 12, 130, ok_ptr, None) == 0  # W = 17 packs (fp32 only)
    assert L.exmy_encode(ok_ptr, B.F32, 0, 8, 22, 255, ok_ptr, None) == 0  # W = 31
    assert L.exmy_encode(ok_ptr, B.F32, 0, 8, 23, 255, ok_ptr, None) == 0  # W = 32, the widest packed form
    assert L.exmy_encode(ok_ptr, B.F32, 0, 8, 23, 254, ok_ptr, None) == 3
    assert L.exmy_emulate(ok_ptr, B.F32, 0, 8, 23, 255, None) == 0  # emulate has no width limit
    assert L.exmy_encode(ok_ptr, B.F32, 8, 3, 3, 6, ok_ptr, None) == 3
    assert L.exmy_decode(ok_ptr, B.F32, 8, 8, 3, 254, ok_ptr, None) == 3
    assert L.exmy_encode(ok_ptr, B.F32, (1 << 40) + 1, 3, 3, 130, ok_ptr, None) == 4
    assert L.exmy_encode(odd_ptr, B.F32, 8, 3, 3, 130, ok_ptr, None) == 5
    assert L.exmy_encode(ok_ptr, B.F32, 8, 3, 3, 130, odd_ptr, None) == 5
    assert L.exmy_decode(odd_ptr, B.BF16, 8, 3, 3, 130, ok_ptr, None) == 5
    assert L.exmy_emulate(odd_ptr, B.BF16, 8, 3, 3, 130, None) == 5
    assert L.exmy_exponent_histogram(ok_ptr, B.F32, 8, None, None) == 1
    assert L.exmy_exponent_histogram(ok_ptr, B.F32, 8, odd_ptr, None) == 5
    assert L.exmy_encode_with_histogram(ok_ptr, B.F32, 8, 3, 3, 130, ok_ptr, None, None) == 1
    # batches: validated as a whole before anything is launched
    descs = (B.TensorDesc * 2)()
    descs[0].src, descs[0].dst, descs[0].n, descs[0].max_exp = 0x1000, 0x2000, 8, 130
    descs[1].src, descs[1].dst, descs[1].n, descs[1].max_exp = 0x1000, 0x2000, 8, 3
    p = ctypes.cast(descs, ctypes.c_void_p)
    assert L.exmy_encode_batch(p, 2, B.BF16, 3, 3, None) == 3  # second tensor's max_exp
    descs[1].max_exp, descs[1].dst = 130, 0x2004
    assert L.exmy_decode_batch(p, 2, B.BF16, 3, 3, None) == 5
    descs[1].dst, descs[1].src = 0x2000, 0
    assert L.exmy_encode_batch(p, 2, B.BF16, 3, 3, None) == 1
    assert L.exmy_encode_batch(None, 2, B.BF16, 3, 3, None) == 1
    assert L.exmy_encode_batch(None, 0, B.BF16, 3, 3, None) == 0
    assert L.exmy_encode_batch(None, 0, B.BF16, 3, 9, None) == 2
    descs[0].n = descs[1].n = 0
    assert L.exmy_encode_batch(p, 2, B.BF16, 3, 3, None) == 0  # empty tensors: nothing to do
    for st in range(0, 7):
        assert B.status_string(st)
    assert "max_exp" in B.status_string(3)


def test_max_exp_from_histogram_matches_oracle():
    import torch

    rng = np.random.default_rng(5)
    for _ in range(50):
        hist = np.zeros(256, dtype=np.uint64)
        idx = rng.integers(0, 256, size=rng.integers(1, 40))
        hist[idx] = rng.integers(1, 1 << 40, size=idx.size, dtype=np.uint64)
        for cov in (0.0, 0.5, 0.9, 0.99, 0.999, 1.0):
            got = B.max_exp_from_histogram(torch.from_numpy(hist.view(np.int64)), cov)
            assert got == O.max_exp_from_histogram(hist, cov)
    assert B.max_exp_from_histogram(torch.zeros(256, dtype=torch.int64), 0.5) == -1


def test_cpu_tensors_are_rejected():
    import torch

    with pytest.raises(ValueError):
        B.encode(torch.zeros(8), 3, 3, 130)
    with pytest.raises(TypeError):
        B._dtype_enum(torch.zeros(8, dtype=torch.float64))


def test_block_entry_points_validate_without_launch():
    L = B.lib()
    ok, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1008)
    for n, block in ((0, 8), (1, 8), (100, 32), (4096, 4096), (4097, 4096)):
        assert B.block_count(n, block) == (n + block - 1) // block
    assert B.block_count(5, 0) == 0
    enc = lambda *a: L.exmy_encode_blocks(*a)
    assert enc(ok, B.BF16, 0, 32, 3, 3, ok, ok, None) == 0  # n = 0: nothing to do
    assert enc(None, B.BF16, 64, 32, 3, 3, ok, ok, None) == 1
    assert enc(ok, B.BF16, 64, 32, 3, 3, None, ok, None) == 1
    assert enc(ok, B.BF16, 64, 32, 3, 3, ok, None, None) == 1
    assert enc(odd, B.BF16, 64, 32, 3, 3, ok, ok, None) == 5
    assert enc(ok, B.BF16, 64, 32, 3, 3, ok, odd, None) == 5
    assert enc(ok, B.BF16, 64, 32, 8, 3, ok, ok, None) == 2  # X = 8 has no per-block metadata
    assert enc(ok, B.BF16, 64, 32, 3, 8, ok, ok, None) == 2  # bf16 holds 7 mantissa bits
    assert enc(ok, B.F32, 64, 32, 3, 13, ok, ok, None) == 2  # packed form stops at 16 bits
    for block in (0, 4, 12, 33, (1 << 31) + 8, 1 << 32):
        assert enc(ok, B.BF16, 64, block, 3, 3, ok, ok, None) == 7
        assert L.exmy_block_max_exp(ok, B.BF16, 64, block, 3, ok, None) == 7
        assert L.exmy_decode_blocks(ok, B.BF16, 64, block, 3, 3, ok, ok, None) == 7
        assert L.exmy_emulate_blocks(ok, B.BF16, 64, block, 3, 3, ok, None) == 7
    assert enc(ok, B.BF16, (1 << 40) + 1, 32, 3, 3, ok, ok, None) == 4
    assert L.exmy_emulate_blocks(ok, B.F32, 0, 32, 2, 22, ok, None) == 0  # emulation has no width limit
    assert L.exmy_emulate_blocks(None, B.F32, 8, 32, 2, 22, ok, None) == 1
    assert L.exmy_block_max_exp(ok, B.F32, 8, 8, 9, ok, None) == 2
    assert L.exmy_block_max_exp(ok, B.F32, 8, 8, 3, None, None) == 1
    assert B.status_string(7).startswith("block size")
    # the oracle rejects the same block sizes and X = 8
    x = np.zeros(64, dtype=np.float32)
    for block in (0, 4, 12, 33):
        with pytest.raises(Exception):
            O.block_max_exp(x, block, 3)


def test_after_rounding_and_auto_entry_points_validate_without_launch():
    L = B.lib()
    ok, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1008)
    mx = L.exmy_block_max_exp_after_rounding
    assert mx(ok, B.F32, 0, 8, 3, 3, ok, None) == 0
    assert mx(None, B.F32, 8, 8, 3, 3, ok, None) == 1
    assert mx(ok, B.F32, 8, 8, 3, 3, None, None) == 1
    assert mx(ok, B.F32, 8, 8, 3, 24, ok, None) == 2
    assert mx(ok, B.F32, 0, 8, 3, 23, ok, None) == 0  # no width limit beyond the container's
    assert mx(ok, B.BF16, 0, 8, 8, 3, ok, None) == 2
    assert mx(ok, B.BF16, 8, 12, 3, 3, ok, None) == 7
    assert mx(odd, B.BF16, 8, 8, 3, 3, ok, None) == 5
    auto = L.exmy_encode_blocks_auto
    assert auto(ok, B.BF16, 0, 32, 3, 3, 0, ok, ok, None) == 0
    assert auto(ok, B.BF16, 0, 32, 3, 3, 1, ok, ok, None) == 0
    assert auto(ok, B.BF16, 0, 32, 3, 3, 2, ok, ok, None) == 2  # unknown scheme
    assert auto(ok, B.BF16, 64, 32, 3, 3, 0, ok, None, None) == 1
    assert auto(ok, B.BF16, 64, 32, 3, 3, 0, None, ok, None) == 1
    assert auto(None, B.BF16, 64, 32, 3, 3, 0, ok, ok, None) == 1
    assert auto(ok, B.BF16, 64, 32, 3, 3, 0, ok, odd, None) == 5
    assert auto(ok, B.F32, 64, 32, 3, 13, 0, ok, ok, None) == 2  # packed form stops at 16 bits
    assert auto(ok, B.BF16, 64, 20, 3, 3, 0, ok, ok, None) == 7


def test_float_scaling_entry_points_validate_without_launch():
    L = B.lib()
    ok, odd16, odd4 = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1008), ctypes.c_void_p(0x1002)

    def with_scale_dtype(fn):  # the scale's dtype follows the scale pointer (argument 6); fp32 unless given
        return lambda *a, sdt=B.F32: fn(*a[:7], sdt, *a[7:])

    sc, enc, dec, emu = (with_scale_dtype(f) for f in (L.exmy_block_scale, L.exmy_encode_scaled, L.exmy_decode_scaled, L.exmy_emulate_scaled))
    assert sc(ok, B.F32, 0, 8, 3, 3, ok, None) == 0
    assert sc(None, B.F32, 8, 8, 3, 3, ok, None) == 1
    assert sc(ok, B.F32, 8, 8, 3, 3, None, None) == 1
    assert sc(ok, B.F32, 8, 8, 3, 3, odd4, None) == 5  # scales are 4-byte aligned
    assert sc(odd16, B.F32, 8, 8, 3, 3, ok, None) == 5
    for X, Y in ((8, 3), (0, 0), (9, 1), (-1, 2)):
        assert sc(ok, B.F32, 0, 8, X, Y, ok, None) == 2
        assert enc(ok, B.F32, 0, 8, X, Y, ok, ok, None) == 2
        assert dec(ok, B.F32, 0, 8, X, Y, ok, ok, None) == 2
        assert emu(ok, B.F32, 0, 8, X, Y, ok, None) == 2
    assert enc(ok, B.F32, 0, 8, 3, 13, ok, ok, None) == 2   # packed form stops at 16 bits
    assert emu(ok, B.F32, 0, 8, 3, 13, ok, None) == 0       # emulation does not
    assert sc(ok, B.F32, 0, 8, 3, 23, ok, None) == 0
    assert sc(ok, B.BF16, 0, 8, 3, 8, ok, None) == 2
    assert enc(ok, B.BF16, 64, 12, 3, 3, ok, ok, None) == 7
    assert enc(ok, B.BF16, 64, 16, 3, 3, None, ok, None) == 1
    assert enc(ok, B.BF16, 64, 16, 3, 3, ok, None, None) == 1
    assert dec(ok, B.BF16, 64, 16, 3, 3, ok, None, None) == 1
    assert dec(odd16, B.BF16, 64, 16, 3, 3, ok, ok, None) == 5
    assert emu(ok, B.BF16, 64, 16, 3, 3, odd4, None) == 5
    assert emu(ok, B.BF16, (1 << 40) + 8, 16, 3, 3, ok, None) == 4
    # bf16 scales: 2-byte aligned; fp16 scales are not offered
    odd1 = ctypes.c_void_p(0x1001)
    assert sc(ok, B.F32, 0, 8, 3, 3, ok, None, sdt=B.BF16) == 0
    assert sc(ok, B.F32, 0, 8, 3, 3, ok, None, sdt=B.F16) == 2
    assert enc(ok, B.BF16, 0, 16, 3, 3, ok, ok, None, sdt=B.F16) == 2
    assert dec(ok, B.BF16, 0, 16, 3, 3, ok, ok, None, sdt=7) == 2
    assert emu(ok, B.BF16, 64, 16, 3, 3, odd1, None, sdt=B.BF16) == 5
    assert sc(ok, B.BF16, 64, 16, 3, 3, odd1, None, sdt=B.BF16) == 5
    assert emu(ok, B.BF16, 64, 16, 3, 3, None, None, sdt=B.BF16) == 1


def test_row_packing_entry_points_validate_without_launch():
    L = B.lib()
    ok, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1008)
    for rows, cols in ((0, 8), (1, 8), (8, 8), (9, 16), (4096, 11008)):
        assert B.packed_bytes_rows(rows, cols, 3, 3) == ((rows + 7) // 8) * cols * 7 == O.packed_bytes_rows(rows, cols, 3, 3)
    enc, dec = L.exmy_encode_rows, L.exmy_decode_rows
    assert enc(ok, B.BF16, 0, 64, 3, 3, 130, None, ok, None) == 0
    assert enc(ok, B.BF16, 64, 0, 3, 3, 130, None, ok, None) == 0
    assert enc(None, B.BF16, 8, 8, 3, 3, 130, None, ok, None) == 1
    assert enc(ok, B.BF16, 8, 8, 3, 3, 130, None, None, None) == 1
    assert dec(ok, B.BF16, 8, 8, 3, 3, 130, None, None, None) == 1
    assert enc(odd, B.BF16, 8, 8, 3, 3, 130, None, ok, None) == 5
    assert dec(ok, B.BF16, 8, 8, 3, 3, 130, None, odd, None) == 5
    assert enc(ok, B.BF16, 8, 8, 3, 3, 5, None, ok, None) == 3       # max_exp below 2^X - 1
    assert enc(ok, B.BF16, 0, 8, 8, 7, 255, None, ok, None) == 0     # X = 8 with its fixed metadatum
    assert enc(ok, B.BF16, 0, 8, 8, 7, 255, ok, ok, None) == 2       # but not with per-row metadata
    assert enc(ok, B.BF16, 0, 8, 3, 3, 5, ok, ok, None) == 0         # max_exp is ignored with per-row metadata
    assert enc(ok, B.F32, 8, 8, 3, 13, 130, None, ok, None) == 2
    for cols in (1, 4, 12, 8 * 11 + 4, (1 << 26) + 8):
        assert enc(ok, B.BF16, 8, cols, 3, 3, 130, None, ok, None) == 8
        assert dec(ok, B.BF16, 8, cols, 3, 3, 130, None, ok, None) == 8
    assert enc(ok, B.BF16, 1 << 30, 1 << 20, 3, 3, 130, None, ok, None) == 4
    assert B.status_string(8).startswith("column count")


def test_twos_complement_entry_points_validate_without_launch():
    L = B.lib()
    ok, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1008)
    enc, dec, emu = L.exmy_encode_int, L.exmy_decode_int, L.exmy_emulate_int
    assert enc(ok, B.F32, 0, 7, 133, ok, None) == 0
    assert enc(None, B.F32, 8, 7, 133, ok, None) == 1
    assert dec(ok, B.F32, 8, 7, 133, None, None) == 1
    assert emu(None, B.F32, 8, 7, 133, None) == 1
    assert enc(odd, B.F32, 8, 7, 133, ok, None) == 5
    assert dec(ok, B.F32, 8, 7, 133, odd, None) == 5
    assert emu(odd, B.BF16, 8, 7, 133, None) == 5
    for Y in (0, -1, 16, 25):
        assert enc(ok, B.F32, 0, Y, 133, ok, None) == 2
    assert enc(ok, B.BF16, 0, 9, 133, ok, None) == 2    # bf16 holds 8 significant bits
    assert enc(ok, B.BF16, 0, 8, 133, ok, None) == 0
    assert emu(ok, B.F32, 0, 21, 133, None) == 0         # emulation goes beyond the packed widths ...
    assert emu(ok, B.F32, 0, 22, 133, None) == 2         # ... up to what one fp32 rounding addend covers
    assert enc(ok, B.F32, 0, 7, 254, ok, None) == 3
    assert enc(ok, B.F32, 0, 7, -1, ok, None) == 3
    assert enc(ok, B.F32, 0, 7, 238, ok, None) == 3      # above 230 + Y the rounding addend would overflow
    assert enc(ok, B.F32, 0, 7, 237, ok, None) == 0
    assert enc(ok, B.F32, (1 << 40) + 1, 7, 133, ok, None) == 4


def test_fp16_container_limits():
    L = B.lib()
    ok = ctypes.c_void_p(0x1000)
    assert L.exmy_encode(ok, B.F16, 0, 3, 3, 130, ok, None) == 0
    assert L.exmy_decode(ok, B.F16, 0, 3, 3, 130, ok, None) == 0
    assert L.exmy_emulate(ok, B.F16, 0, 4, 10, 130, None) == 0
    assert L.exmy_exponent_histogram(ok, B.F16, 0, ok, None) == 0
    assert L.exmy_encode(ok, B.F16, 0, 6, 3, 130, ok, None) == 2       # X <= 5
    assert L.exmy_encode(ok, B.F16, 0, 3, 11, 130, ok, None) == 2      # Y <= 10
    assert L.exmy_encode(ok, B.F16, 0, 3, 3, 143, ok, None) == 3       # top binade above 2^15
    assert L.exmy_encode(ok, B.F16, 0, 3, 3, 111, ok, None) == 3       # quantum below 2^-24
    assert L.exmy_encode(ok, B.F16, 0, 3, 3, 112, ok, None) == 0
    # per-block forms: the same formats, unless no metadatum keeps them inside fp16
    assert L.exmy_block_max_exp(ok, B.F16, 0, 8, 3, ok, None) == 0
    assert L.exmy_block_max_exp(ok, B.F16, 0, 8, 6, ok, None) == 2
    assert L.exmy_block_max_exp_after_rounding(ok, B.F16, 0, 8, 3, 3, ok, None) == 0
    assert L.exmy_encode_blocks(ok, B.F16, 0, 8, 3, 3, ok, ok, None) == 0
    assert L.exmy_encode_blocks(ok, B.F16, 0, 8, 5, 9, ok, ok, None) == 0
    assert L.exmy_encode_blocks(ok, B.F16, 0, 8, 5, 10, ok, ok, None) != 0
    assert L.exmy_encode_blocks_auto(ok, B.F16, 0, 8, 3, 3, 0, ok, ok, None) == 0
    assert L.exmy_block_scale(ok, B.F16, 0, 8, 3, 3, ok, B.F32, None) == 0
    assert L.exmy_block_scale(ok, B.F16, 0, 8, 4, 10, ok, B.BF16, None) == 0
    assert L.exmy_block_scale(ok, B.F16, 0, 8, 5, 2, ok, B.F32, None) != 0    # max_exp = 127 lies under e5m2's fp16 range
    assert L.exmy_encode_rows(ok, B.F16, 0, 8, 3, 3, 130, None, ok, None) == 0
    assert L.exmy_encode_rows(ok, B.F16, 0, 8, 3, 3, 143, None, ok, None) == 3
    assert L.exmy_encode_rows(ok, B.F16, 0, 8, 3, 3, 0, ok, ok, None) == 0
    assert L.exmy_encode_int(ok, B.F16, 0, 7, 133, ok, None) == 0
    assert L.exmy_encode_int(ok, B.F16, 0, 7, 142, ok, None) == 3      # -2^16 is not a half
    assert L.exmy_encode_int(ok, B.F16, 0, 7, 108, ok, None) == 3      # quantum 2^-25
    assert L.exmy_encode_int(ok, B.F16, 0, 12, 133, ok, None) == 2


def test_tile_entry_points_validate_without_launch():
    L = B.lib()
    ok, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1008)
    mx, enc, dec, emu = L.exmy_tile_max_exp, L.exmy_encode_tiles, L.exmy_decode_tiles, L.exmy_emulate_tiles
    for rows, cols, tr, tc in ((9, 24, 4, 16), (4096, 4096, 128, 128), (64, 64, 64, 1), (0, 64, 8, 8), (5, 8, 100, 100)):
        assert B.tile_count(rows, cols, tr, tc) == O.tile_count(rows, cols, tr, tc)
    assert B.tile_count(8, 8, 0, 8) == 0
    assert mx(ok, B.BF16, 0, 64, 8, 8, 3, 0, 0, ok, None) == 0
    assert mx(ok, B.BF16, 8, 0, 8, 8, 3, 0, 0, ok, None) == 0
    assert mx(ok, B.BF16, 8, 60, 8, 8, 3, 0, 0, ok, None) == 8            # cols not a multiple of 8
    assert mx(ok, B.BF16, 8, (1 << 26) + 8, 8, 8, 3, 0, 0, ok, None) == 8
    assert mx(ok, B.BF16, (1 << 31) + 1, 8, 8, 8, 3, 0, 0, ok, None) == 8
    assert mx(ok, B.BF16, 8, 64, 8, 12, 3, 0, 0, ok, None) == 7           # tile width neither 1 nor a multiple of 8
    assert mx(ok, B.BF16, 8, 64, 0, 8, 3, 0, 0, ok, None) == 7
    assert mx(ok, B.BF16, 8, 64, 8, 0, 3, 0, 0, ok, None) == 7
    assert mx(ok, B.BF16, 1 << 20, 1 << 21, 8, 8, 3, 0, 0, ok, None) == 4  # more than 2^40 elements
    assert mx(None, B.BF16, 8, 64, 4, 8, 3, 0, 0, ok, None) == 1
    assert mx(ok, B.BF16, 8, 64, 4, 8, 3, 0, 0, None, None) == 1
    assert mx(ok, B.BF16, 8, 64, 4, 8, 3, 0, 0, odd, None) == 5           # the metadata array is 16-byte aligned too
    assert mx(odd, B.BF16, 8, 64, 4, 8, 3, 0, 0, ok, None) == 5
    assert mx(ok, B.BF16, 8, 64, 4, 8, 8, 0, 0, ok, None) == 2            # X = 8 has no per-block metadata
    assert mx(ok, B.BF16, 8, 64, 4, 8, 3, 0, 2, ok, None) == 2            # no such scheme
    assert mx(ok, B.BF16, 0, 64, 4, 8, 3, 9, 1, ok, None) == 2            # "after rounding" needs a valid Y
    assert mx(ok, B.BF16, 0, 64, 4, 8, 3, 9, 0, ok, None) == 0            # "before rounding" ignores it
    assert enc(ok, B.F32, 0, 64, 4, 8, 3, 13, ok, ok, None) == 2          # packed form stops at 16 bits
    assert emu(ok, B.F32, 0, 64, 4, 8, 3, 13, ok, None) == 0
    assert enc(ok, B.BF16, 8, 64, 4, 8, 3, 3, ok, None, None) == 1
    assert dec(ok, B.BF16, 8, 64, 4, 8, 3, 3, ok, None, None) == 1
    assert dec(ok, B.BF16, 8, 64, 4, 8, 3, 3, ok, odd, None) == 5
    assert emu(ok, B.F16, 0, 64, 4, 8, 5, 2, ok, None) == 0
    assert emu(ok, B.F16, 0, 64, 4, 8, 6, 2, ok, None) == 2


def test_record_entry_points_validate_without_launch():
    L = B.lib()
    ok, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1008)
    enc, dec = L.exmy_encode_records, L.exmy_decode_records
    for f in (enc, dec):
        assert f(ok, B.BF16, 0, 3, 3, 130, ok, None) == 0
        assert f(None, B.BF16, 8, 3, 3, 130, ok, None) == 1
        assert f(ok, B.BF16, 8, 3, 3, 130, None, None) == 1
        assert f(odd, B.BF16, 8, 3, 3, 130, ok, None) == 5
        assert f(ok, B.BF16, 8, 3, 3, 130, odd, None) == 5
        assert f(ok, B.F32, 0, 4, 12, 130, ok, None) == 2   # records stop at 16 bits
        assert f(ok, B.F32, 0, 5, 10, 130, ok, None) == 0
        assert f(ok, B.BF16, 0, 3, 3, 6, ok, None) == 3
        assert f(ok, B.BF16, (1 << 40) + 8, 3, 3, 130, ok, None) == 4


def test_reserved_code_entry_points_validate_without_launch():
    L = B.lib()
    ok, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1008)
    enc, dec, emu = L.exmy_encode_specials, L.exmy_decode_specials, L.exmy_emulate_specials
    IEEE, NAN_ONLY = B.SPECIALS_IEEE, B.SPECIALS_NAN_ONLY
    for f in (enc, dec):
        assert f(ok, B.BF16, 0, 5, 2, 143, IEEE, ok, None) == 0
        assert f(ok, B.BF16, 0, 4, 3, 135, NAN_ONLY, ok, None) == 0
        assert f(ok, B.BF16, 0, 8, 7, 255, IEEE, ok, None) == 0      # bf16 itself
        assert f(ok, B.BF16, 0, 8, 7, 255, NAN_ONLY, ok, None) == 2
        assert f(ok, B.BF16, 0, 0, 3, 130, IEEE, ok, None) == 2      # no exponent code to reserve
        assert f(ok, B.BF16, 0, 0, 3, 130, NAN_ONLY, ok, None) == 0
        assert f(ok, B.BF16, 0, 0, 0, 130, NAN_ONLY, ok, None) == 2
        assert f(ok, B.BF16, 0, 3, 3, 130, 0, ok, None) == 2
        assert f(ok, B.BF16, 0, 3, 3, 130, 3, ok, None) == 2
        assert f(ok, B.F32, 0, 4, 12, 130, IEEE, ok, None) == 2      # packed form stops at 16 bits
        assert f(ok, B.BF16, 0, 3, 3, 6, IEEE, ok, None) == 3
        assert f(None, B.BF16, 8, 3, 3, 130, IEEE, ok, None) == 1
        assert f(ok, B.BF16, 8, 3, 3, 130, IEEE, None, None) == 1
        assert f(odd, B.BF16, 8, 3, 3, 130, IEEE, ok, None) == 5
        assert f(ok, B.BF16, (1 << 40) + 8, 3, 3, 130, IEEE, ok, None) == 4
    assert emu(ok, B.F32, 0, 4, 12, 130, IEEE, None) == 0
    assert emu(None, B.F32, 8, 4, 12, 130, IEEE, None) == 1
    assert emu(odd, B.F32, 8, 4, 12, 130, NAN_ONLY, None) == 5
