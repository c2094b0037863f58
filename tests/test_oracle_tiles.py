"""Pins of the CPU oracle's column / 2-D tile blocks (the block shapes of Section 2 "Block Size" that are not
runs of consecutive elements).  The tile functions walk (row, column) indices of their own; each
pin reaches the same result through a function that is pinned elsewhere and a numpy reshape / transpose,
so a wrong tile index, a transposed metadata array or a mishandled edge shows up."""
import numpy as np
import pytest
import torch

from oracle import exmy_oracle as O
from paper_2405_13938_amd import synth


def matrix(rows, cols, dtype=torch.bfloat16, seed=0, spread=12):
    g = torch.Generator().manual_seed(seed)
    x = torch.randn(rows, cols, generator=g) * torch.exp2(torch.randint(-spread, spread, (rows, cols), generator=g).float())
    x[torch.rand(rows, cols, generator=g) < 0.01] = float("inf")
    x[torch.rand(rows, cols, generator=g) < 0.01] = float("nan")
    x[torch.rand(rows, cols, generator=g) < 0.02] = 0.0
    return synth.bits_numpy(x.to(dtype)).reshape(rows, cols)


def ubits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else a


def tiles_as_blocks(a, tr, tc):
    """(rows, cols) with rows % tr == cols % tc == 0 -> flat array in which every tile is one run of tr*tc elements,
    tiles in row-major tile order (the order of the metadata array)."""
    rows, cols = a.shape
    return np.ascontiguousarray(a.reshape(rows // tr, tr, cols // tc, tc).transpose(0, 2, 1, 3)).reshape(-1)


def blocks_as_tiles(flat, rows, cols, tr, tc):
    return np.ascontiguousarray(flat.reshape(rows // tr, cols // tc, tr, tc).transpose(0, 2, 1, 3)).reshape(rows, cols)


def padded(a, tr, tc):
    rows, cols = a.shape
    R, C = -(-rows // tr) * tr, -(-cols // tc) * tc
    out = np.zeros((R, C), dtype=a.dtype)
    out[:rows, :cols] = a
    return out


SHAPES = [  # rows, cols, tile_rows, tile_cols (tile element counts are multiples of 8 so the block functions apply)
    (64, 64, 8, 8), (64, 128, 16, 32), (96, 64, 32, 16), (40, 72, 8, 24), (64, 64, 64, 1), (64, 64, 16, 1),
    (24, 64, 24, 64), (16, 64, 1, 16), (37, 72, 8, 16), (50, 40, 16, 1), (19, 88, 5, 8), (64, 64, 128, 256),
]


@pytest.mark.parametrize("rows,cols,tr,tc", SHAPES)
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_tiles_are_blocks_of_the_rearranged_matrix(rows, cols, tr, tc, dtype):
    a = matrix(rows, cols, dtype, seed=rows + cols + tr)
    p = padded(a, tr, tc)  # zeros change neither a maximum nor the other elements' results
    if (tr * tc) % 8:
        pytest.skip("tile of %d elements: the block functions need multiples of 8" % (tr * tc))
    flat = tiles_as_blocks(p, tr, tc)
    for X, Y in ((2, 1), (3, 3), (0, 3), (4, 2)):
        for after in (False, True):
            got = O.tile_max_exp(a, tr, tc, X, Y, after)
            want = O.block_max_exp_after_rounding(flat, tr * tc, X, Y) if after else O.block_max_exp(flat, tr * tc, X)
            assert np.array_equal(got, want), (X, Y, after)
        meta = O.tile_max_exp(a, tr, tc, X)
        meta = (meta.astype(np.int32) + np.random.default_rng(rows).integers(-3, 2, meta.size)).clip(0, 255).astype(np.uint8)
        emu = O.emulate_tiles(a, tr, tc, X, Y, meta)
        want = blocks_as_tiles(O.emulate_blocks(flat, tr * tc, X, Y, meta), p.shape[0], p.shape[1], tr, tc)[:rows, :cols]
        assert np.array_equal(ubits(emu), ubits(want)), (X, Y)
        packed = O.encode_tiles(a, tr, tc, X, Y, meta)
        dec = O.decode_tiles(packed, O.F32 if dtype == torch.float32 else O.BF16, rows, cols, tr, tc, X, Y, meta)
        fin = np.isfinite(synth_float(a))
        assert np.array_equal(ubits(dec)[fin], ubits(emu)[fin]), (X, Y)


def synth_float(a):
    return a if a.dtype == np.float32 else (a.astype(np.uint32) << 16).view(np.float32)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_column_blocks_are_row_blocks_of_the_transpose(dtype):
    rows, cols = 48, 64
    a = matrix(rows, cols, dtype, seed=5)
    at = np.ascontiguousarray(a.T)  # (cols, rows): a column of `a` is a row of `at`
    for X, Y in ((2, 1), (3, 3), (0, 3)):
        for tr in (rows, 16, 8):  # whole columns and parts of columns
            meta = O.tile_max_exp(a, tr, 1, X)
            want = O.block_max_exp(at.reshape(-1), tr, X).reshape(cols, rows // tr).T  # [column][part] -> [part][column]
            assert np.array_equal(meta.reshape(rows // tr, cols), want), (X, Y, tr)
            emu = O.emulate_tiles(a, tr, 1, X, Y, meta)
            want = O.emulate_blocks(at.reshape(-1), tr, X, Y, np.ascontiguousarray(want.T).reshape(-1)).reshape(cols, rows).T
            assert np.array_equal(ubits(emu), ubits(np.ascontiguousarray(want))), (X, Y, tr)


def test_rows_sub_rows_and_the_whole_tensor_reduce_to_the_flat_functions():
    rows, cols = 24, 96
    a = matrix(rows, cols, torch.bfloat16, seed=6)
    flat = a.reshape(-1)
    for X, Y in ((2, 1), (3, 3), (0, 3), (4, 3)):
        for tc in (cols, 32, 8):  # (1, tc) tiles are consecutive blocks of tc elements
            meta = O.tile_max_exp(a, 1, tc, X)
            assert np.array_equal(meta, O.block_max_exp(flat, tc, X))
            assert np.array_equal(O.encode_tiles(a, 1, tc, X, Y, meta), O.encode_blocks(flat, tc, X, Y, meta))
            dec = O.decode_tiles(O.encode_tiles(a, 1, tc, X, Y, meta), O.BF16, rows, cols, 1, tc, X, Y, meta)
            assert np.array_equal(dec.reshape(-1), O.decode_blocks(O.encode_blocks(flat, tc, X, Y, meta), O.BF16, flat.size, tc, X, Y, meta))
        # one tile = the tensor: the per-tensor codec with that metadatum
        meta = O.tile_max_exp(a, rows, cols, X)
        assert meta.size == 1
        assert np.array_equal(O.encode_tiles(a, rows, cols, X, Y, meta), O.encode(flat, X, Y, int(meta[0])))
        assert np.array_equal(O.emulate_tiles(a, rows, cols, X, Y, meta).reshape(-1), O.emulate(flat, X, Y, int(meta[0])))


def test_metadata_array_is_row_major_over_tiles():
    # one large element in tile (1, 2) of a 3 x 4 tile grid
    a = np.full((24, 64), 0x3C00, dtype=np.uint16)  # bf16 2^-7 = biased exponent 120
    a[8 + 3, 32 + 5] = 0x4300                       # 128 = biased exponent 134
    meta = O.tile_max_exp(a, 8, 16, 3).reshape(3, 4)
    want = np.full((3, 4), 120, dtype=np.uint8)
    want[1, 2] = 134
    assert np.array_equal(meta, want)
    # and each element is coded with its own tile's metadatum: 2^-7 is the top binade at 120 but flushes at 134 (e3m3)
    emu = O.emulate_tiles(a, 8, 16, 3, 3, meta)
    assert emu[8 + 3, 32 + 5] == 0x4300
    inside = np.zeros((24, 64), dtype=bool)
    inside[8:16, 32:48] = True
    inside[8 + 3, 32 + 5] = False
    assert (emu[inside] == 0).all() and (emu[~inside & (a == 0x3C00)] == 0x3C00).all()


def test_tile_validation():
    a = np.zeros((8, 16), dtype=np.uint16)
    with pytest.raises(Exception):
        O.tile_max_exp(np.zeros((8, 12), dtype=np.uint16), 4, 4, 3)  # cols not a multiple of 8
    with pytest.raises(Exception):
        O.tile_max_exp(a, 0, 8, 3)
    with pytest.raises(Exception):
        O.tile_max_exp(a, 8, 0, 3)
    with pytest.raises(Exception):
        O.tile_max_exp(a, 8, 8, 8)  # X = 8 has no per-block metadata
    with pytest.raises(Exception):
        O.encode_tiles(np.zeros((8, 16), dtype=np.float32), 8, 8, 3, 13, np.zeros(2, dtype=np.uint8))  # 17-bit codes
    assert O.tile_max_exp(np.zeros((0, 16), dtype=np.uint16), 8, 8, 3).size == 0
    assert O.tile_count(9, 24, 4, 16) == 3 * 2
