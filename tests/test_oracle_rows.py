"""Pins of the CPU oracle's packing along rows ((8R, C) -> planes of shape (R, C)):
the paper's stated shapes and sizes, the flat packer applied to the permuted
matrix, sharding along rows and columns, and the per-tensor / per-block functions
for the values."""
import numpy as np
import pytest
import torch

from oracle import exmy_oracle as O
from paper_2405_13938_amd import synth

F32, BF16 = O.F32, O.BF16


def as_np(t):
    return synth.bits_numpy(t)


def test_plane_shapes_of_the_paper():
    # Section 2.2.2: (8R, C) with 7-bit elements -> int32, int16 and int8 arrays of shape (R, C);
    # 5-bit elements -> int32 and int8; 8 elements of 7 bits use exactly 56 bits
    R, C = 5, 24
    assert O.packed_bytes_rows(8 * R, C, 3, 3) == R * C * (4 + 2 + 1)
    assert O.packed_bytes_rows(8 * R, C, 2, 2) == R * C * (4 + 1)
    assert O.packed_bytes_rows(8, 1, 3, 3) * 8 == 56
    # Fig. 2: an (8, 1) array of 7-bit codes c_j: int32 holds the low 4 bits of every c_j (element j at
    # bits 4j..4j+3), int16 the next 2 bits, int8 the top bit
    vals = np.array([1.0, -1.5, 0.25, 6.0, -0.125, 3.5, 0.0, -7.5], dtype=np.float32)
    codes = O.to_codes(vals, 3, 3, 129)
    p = O.encode_rows(vals, 8, 1, 3, 3, 129)
    w32 = int.from_bytes(p[0:4].tobytes(), "little")
    w16 = int.from_bytes(p[4:6].tobytes(), "little")
    w8 = int(p[6])
    for j, c in enumerate(codes.tolist()):
        assert (w32 >> (4 * j)) & 0xF == c & 0xF
        assert (w16 >> (2 * j)) & 0x3 == (c >> 4) & 0x3
        assert (w8 >> j) & 1 == (c >> 6) & 1


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("X,Y", [(3, 3), (2, 2), (1, 1), (4, 4), (0, 2), (5, 7), (8, 7), (7, 0)])
@pytest.mark.parametrize("rows,cols", [(8, 1), (16, 8), (24, 40), (13, 16), (7, 8), (64, 3)])
def test_rows_layout_is_the_flat_layout_of_the_permuted_matrix(dtype, X, Y, rows, cols):
    g = torch.Generator().manual_seed(rows * 100 + cols)
    x = (torch.randn(rows * cols, generator=g) * 4).to(dtype)
    xn = as_np(x)
    me = 255 if X == 8 else 130
    R = (rows + 7) // 8
    codes = O.to_codes(xn, X, Y, me).reshape(rows, cols)
    padded = np.zeros((8 * R, cols), dtype=codes.dtype)
    padded[:rows] = codes
    # group (r, c) = rows 8r..8r+7 of column c; flat groups in (r, c) order
    flat = padded.reshape(R, 8, cols).transpose(0, 2, 1).reshape(-1)
    want = O.pack(flat, 1 + X + Y)
    got = O.encode_rows(xn, rows, cols, X, Y, me)
    assert np.array_equal(got, want)
    dec = O.decode_rows(got, F32 if dtype == torch.float32 else BF16, rows, cols, X, Y, me)
    assert np.array_equal(dec.view(np.uint8), O.from_codes(codes.reshape(-1), F32 if dtype == torch.float32 else BF16, X, Y, me).view(np.uint8))


def test_sharding_along_rows_and_columns_commutes_with_packing():
    # Section 2.2.2: "sharded along rows or columns, before or after packing"
    rows, cols, X, Y, me = 32, 24, 3, 3, 128
    W = 7
    x = torch.randn(rows * cols, generator=torch.Generator().manual_seed(4)).float().numpy()
    full = O.encode_rows(x, rows, cols, X, Y, me)
    R = rows // 8
    planes, off = [], 0
    for s in (4, 2, 1):
        planes.append(full[off: off + R * cols * s].reshape(R, cols * s))
        off += R * cols * s
    m = x.reshape(rows, cols)
    # rows [8, 24): plane rows [1, 3)
    part = O.encode_rows(np.ascontiguousarray(m[8:24]).reshape(-1), 16, cols, X, Y, me)
    assert np.array_equal(part, np.concatenate([p[1:3].reshape(-1) for p in planes]))
    # columns [8, 16): plane columns [8, 16) (s bytes each)
    part = O.encode_rows(np.ascontiguousarray(m[:, 8:16]).reshape(-1), rows, 8, X, Y, me)
    assert np.array_equal(part, np.concatenate([p[:, 8 * s: 16 * s].reshape(-1) for p, s in zip(planes, (4, 2, 1))]))
    assert full.size == rows * cols * W // 8


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_per_row_metadata_is_the_block_scheme_with_block_equal_to_the_row(dtype):
    rows, cols = 21, 32
    g = torch.Generator().manual_seed(8)
    x = (torch.randn(rows, cols, generator=g) * torch.exp2(torch.randint(-8, 8, (rows, 1), generator=g).float())).to(dtype).reshape(-1)
    xn = as_np(x)
    dt = F32 if dtype == torch.float32 else BF16
    for X, Y in ((3, 3), (2, 1), (0, 3), (4, 2)):
        meta = O.block_max_exp(xn, cols, X)  # one metadatum per row
        meta[3], meta[5] = 0, 255              # out-of-range bytes are read as the nearest valid value
        packed = O.encode_rows(xn, rows, cols, X, Y, max_exp_rows=meta)
        # values: the per-block functions with block = one row
        want_vals = O.decode_blocks(O.encode_blocks(xn, cols, X, Y, meta), dt, rows * cols, cols, X, Y, meta)
        got_vals = O.decode_rows(packed, dt, rows, cols, X, Y, max_exp_rows=meta)
        assert np.array_equal(got_vals.view(np.uint8), want_vals.view(np.uint8))
        # layout: codes of the block scheme, permuted, through the flat packer
        codes = O.unpack(O.encode_blocks(xn, cols, X, Y, meta), rows * cols, 1 + X + Y).reshape(rows, cols)
        R = (rows + 7) // 8
        padded = np.zeros((8 * R, cols), dtype=codes.dtype)
        padded[:rows] = codes
        assert np.array_equal(packed, O.pack(padded.reshape(R, 8, cols).transpose(0, 2, 1).reshape(-1), 1 + X + Y))


def test_rows_validation():
    x = np.zeros(64, dtype=np.float32)
    with pytest.raises(Exception):
        O.encode_rows(x, 8, 8, 9, 1, 130)
    with pytest.raises(Exception):
        O.encode_rows(x, 8, 8, 3, 3, 300)
    with pytest.raises(Exception):
        O.encode_rows(x, 8, 8, 8, 3, 0, max_exp_rows=np.zeros(8, dtype=np.uint8))  # X = 8 has no per-row metadata
    assert O.encode_rows(np.zeros(0, dtype=np.float32), 0, 8, 3, 3, 130).size == 0
