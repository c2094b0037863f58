"""Blocks that are columns or 2-D tiles (Section 2 "Block Size") on the GPU, against the CPU oracle,
bit for bit: metadata under both schemes, encode, decode and emulate."""
import numpy as np
import pytest
import torch

import paper_2405_13938_amd as exmy
from oracle import exmy_oracle as O
from paper_2405_13938_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
THREADS = min(O.default_threads(), 16)
ODT = {torch.float32: O.F32, torch.bfloat16: O.BF16, torch.float16: O.F16}


def ubits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else (a.view(np.uint16) if a.dtype == np.float16 else a)


def tbits(t):
    return ubits(synth.bits_numpy(t))


def matrix(rows, cols, dtype, seed, spread=10, specials=True):
    g = torch.Generator(DEV).manual_seed(seed)
    x = torch.randn(rows, cols, device=DEV, generator=g) * torch.exp2(torch.randint(-spread, spread, (rows, cols), device=DEV, generator=g).float())
    # tiles of different magnitude, so that a wrong tile index changes results
    x = x * torch.exp2(((torch.arange(rows, device=DEV)[:, None] // 5 * 3 + torch.arange(cols, device=DEV)[None, :] // 8) % 7).float())
    if dtype == torch.float32:
        x = x * 1.0009765625
    if specials:
        x[torch.rand(rows, cols, device=DEV, generator=g) < 0.003] = float("inf")
        x[torch.rand(rows, cols, device=DEV, generator=g) < 0.003] = float("nan")
        x[torch.rand(rows, cols, device=DEV, generator=g) < 0.01] = 0.0
    return x.to(dtype).contiguous()


def check_tiles(x, tr, tc, X, Y, what=("max", "encode", "decode", "emulate")):
    rows, cols = x.shape
    host = synth.bits_numpy(x).reshape(rows, cols)
    label = "e%dm%d %dx%d tile %dx%d %s" % (X, Y, rows, cols, tr, tc, x.dtype)
    if "max" in what:
        for scheme in (exmy.binding.BEFORE_ROUNDING, exmy.binding.AFTER_ROUNDING):
            got = exmy.tile_max_exp(x, tr, tc, X, Y, scheme)
            torch.cuda.synchronize()
            want = O.tile_max_exp(host, tr, tc, X, Y, bool(scheme))
            assert np.array_equal(got.cpu().numpy(), want), "tile_max_exp scheme %d %s" % (scheme, label)
    meta = O.tile_max_exp(host, tr, tc, X)
    rng = np.random.default_rng(rows * 31 + cols + tr)
    meta = (meta.astype(np.int32) + rng.integers(-3, 2, meta.size)).clip(0, 255).astype(np.uint8)
    meta[rng.random(meta.size) < 0.02] = 0      # out-of-range bytes are clamped
    meta[rng.random(meta.size) < 0.02] = 255
    meta_dev = torch.from_numpy(meta).to(DEV)
    if 1 + X + Y <= 16 and ("encode" in what or "decode" in what):
        want_packed = O.encode_tiles(host, tr, tc, X, Y, meta, threads=THREADS)
        if "encode" in what:
            got = exmy.encode_tiles(x, tr, tc, X, Y, meta_dev)
            torch.cuda.synchronize()
            assert np.array_equal(got.cpu().numpy(), want_packed), "encode_tiles " + label
        if "decode" in what:
            got = exmy.decode_tiles(torch.from_numpy(want_packed).to(DEV), x.dtype, rows, cols, tr, tc, X, Y, meta_dev)
            torch.cuda.synchronize()
            want = O.decode_tiles(want_packed, ODT[x.dtype], rows, cols, tr, tc, X, Y, meta, threads=THREADS)
            assert np.array_equal(tbits(got), ubits(want).reshape(-1)), "decode_tiles " + label
    if "emulate" in what:
        got = exmy.emulate_tiles(x.clone(), tr, tc, X, Y, meta_dev)
        torch.cuda.synchronize()
        want = O.emulate_tiles(host, tr, tc, X, Y, meta, threads=THREADS)
        assert np.array_equal(tbits(got), ubits(want).reshape(-1)), "emulate_tiles " + label


SHAPES = [  # rows, cols, tile_rows, tile_cols
    (64, 64, 8, 8), (300, 1024, 32, 64), (257, 520, 16, 8), (1030, 72, 128, 24), (37, 72, 8, 16), (19, 88, 5, 8),
    (96, 4096, 32, 256), (513, 264, 100, 40), (2000, 8, 3, 8), (9, 2056, 4, 2048),
    (64, 4096, 64, 1), (513, 264, 100, 1), (2000, 8, 2000, 1), (300, 1024, 7, 1), (48, 8200, 48, 1),
]


@pytest.mark.parametrize("rows,cols,tr,tc", SHAPES)
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32, torch.float16])
def test_tile_shapes(rows, cols, tr, tc, dtype):
    x = matrix(rows, cols, dtype, seed=rows + cols + tr + tc, spread=6 if dtype == torch.float16 else 10)
    for X, Y in ((3, 3), (2, 1), (0, 3)):
        check_tiles(x, tr, tc, X, Y)


@pytest.mark.parametrize("W", range(2, 17))
def test_every_width(W):
    x16 = matrix(130, 528, torch.bfloat16, seed=W)
    x32 = matrix(130, 528, torch.float32, seed=W + 100)
    for X in range(0, min(W - 1, 7) + 1):
        Y = W - 1 - X
        if (X, Y) == (0, 0):
            continue
        for tr, tc in ((16, 48), (130, 1)):
            if Y <= (7 if X else 8):
                check_tiles(x16, tr, tc, X, Y, what=("encode", "decode", "emulate"))
            check_tiles(x32, tr, tc, X, Y, what=("encode", "decode", "emulate"))


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_wide_formats_emulate_only(dtype):
    x = matrix(70, 264, dtype, seed=3)
    for X, Y in ((7, 0), (1, 7), (0, 8)) if dtype == torch.bfloat16 else ((5, 18), (2, 22), (3, 23), (0, 24), (7, 15)):
        for tr, tc in ((8, 24), (70, 1)):
            check_tiles(x, tr, tc, X, Y, what=("max", "emulate"))


def test_weight_matrix_tiles_and_columns():
    x = synth.gaussian_bf16(4096 * 4096, std=0.02, seed=41, device=DEV).view(4096, 4096)
    x[::97, ::89] *= 50.0
    for tr, tc in ((128, 128), (32, 32), (4096, 1), (64, 1), (1, 4096), (16, 4096), (1, 64)):
        check_tiles(x, tr, tc, 3, 3)
        check_tiles(x, tr, tc, 2, 1, what=("max", "encode"))


def test_consecutive_tiles_equal_the_block_entry_points():
    x = matrix(64, 1024, torch.bfloat16, seed=8)
    flat = x.view(-1)
    for tr, tc, block in ((1, 1024, 1024), (1, 64, 64), (4, 1024, 4096), (1, 5000, 1024)):
        meta = exmy.tile_max_exp(x, tr, tc, 3)
        assert torch.equal(meta, exmy.block_max_exp(flat, block, 3))
        assert torch.equal(exmy.encode_tiles(x, tr, tc, 3, 3, meta), exmy.encode_blocks(flat, block, 3, 3, meta))
        check_tiles(x, tr, tc, 3, 3)


def test_empty_and_single_tile():
    e = torch.empty((0, 64), dtype=torch.bfloat16, device=DEV)
    assert exmy.tile_max_exp(e, 8, 8, 3).numel() == 0
    assert exmy.encode_tiles(e, 8, 8, 3, 3, torch.empty(0, dtype=torch.uint8, device=DEV)).numel() == 0
    x = matrix(24, 64, torch.bfloat16, seed=2)
    check_tiles(x, 1 << 20, 1 << 20, 3, 3)   # one tile = the tensor
    check_tiles(x, 24, 64, 2, 1)
    with pytest.raises(exmy.ExmyError):
        exmy.tile_max_exp(x, 8, 12, 3)        # tile width neither 1 nor a multiple of 8
    with pytest.raises(exmy.ExmyError):
        exmy.tile_max_exp(x[:, :60].contiguous(), 8, 8, 3)  # cols not a multiple of 8


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("rows,cols,tr,tc", [(40, 40, 8, 8), (37, 24, 37, 8), (100, 16, 10, 8), (300, 56, 128, 8),
                                            (7, 48, 3, 16), (5000, 24, 5000, 8), (64, 88, 16, 8), (9, 8, 4, 8)])
def test_tile_max_exp_writes_only_its_own_bytes(dtype, rows, cols, tr, tc):
    """The metadata array of these shapes is not a multiple of 4 bytes long (5, 3, 10 x 2 ... tiles), or shorter
    than one word.  It is placed inside a larger buffer of guard bytes, 16-byte aligned as the call asks, with
    the bytes right behind it checked for being untouched."""
    x = matrix(rows, cols, dtype, seed=rows + cols)
    count = exmy.tile_count(rows, cols, tr, tc)
    want = O.tile_max_exp(synth.bits_numpy(x).reshape(rows, cols), tr, tc, 3)
    for scheme in (0, 1):
        if scheme:
            want = O.tile_max_exp(synth.bits_numpy(x).reshape(rows, cols), tr, tc, 3, 2, True)
        buf = torch.full((count + 64,), 0xA5, dtype=torch.uint8, device=DEV)
        out = buf[:count]
        exmy.tile_max_exp(x, tr, tc, 3, 2, scheme, out=out)
        torch.cuda.synchronize()
        got = buf.cpu().numpy()
        assert np.array_equal(got[:count], want)
        assert (got[count:] == 0xA5).all(), "bytes behind the metadata array were written"
