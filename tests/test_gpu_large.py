"""Tensors larger than 2^32 elements / 2^33 bytes: 64-bit group and byte offsets in every
kernel.  The oracle checks 8-aligned shards at the start, across the 2^32 boundary and at
the ragged end, through the slice of each plane that the shard owns; the histogram is
compared whole."""
import numpy as np
import pytest
import torch

import paper_2405_13938_amd as exmy
from oracle import exmy_oracle as O
from paper_2405_13938_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
THREADS = min(O.default_threads(), 16)


def plane_sizes(W):
    return [s for s in (16, 8, 4, 2, 1) if W & s]


def shards(n):
    mid = 1 << 32
    out = [(0, 1 << 20), (mid - (1 << 19), mid + (1 << 19)), (n - (n % 8) - (1 << 19), n)]
    return [(a, b) for a, b in out if 0 <= a < b <= n]


@pytest.mark.parametrize("dtype,n", [(torch.bfloat16, (1 << 32) + 4096 * 3 + 5), (torch.float32, (1 << 31) + 4096 * 5 + 3)])
def test_beyond_4g(dtype, n):
    X, Y, W, max_exp = 3, 3, 7, 123
    x = synth.gaussian_bf16(n, std=0.05, seed=21, device=DEV)
    if dtype == torch.float32:
        x = x.float() * 1.0009765625  # give the low mantissa bits something to round
    dt = O.F32 if dtype == torch.float32 else O.BF16
    G = (n + 7) // 8
    packed = exmy.encode(x, X, Y, max_exp)
    back = exmy.decode(packed, dtype, n, X, Y, max_exp)
    emu = exmy.emulate(x.clone(), X, Y, max_exp)
    torch.cuda.synchronize()
    assert packed.numel() == G * W
    for a, b in shards(n):
        host = synth.bits_numpy(x[a:b])
        want = O.encode(host, X, Y, max_exp, threads=THREADS)
        g0, g1 = a // 8, (b + 7) // 8
        wo, po = 0, 0
        for s in plane_sizes(W):
            got = packed[po + g0 * s : po + g1 * s].cpu().numpy()
            assert np.array_equal(got, want[wo : wo + (g1 - g0) * s]), (dtype, a, b, s)
            wo += (g1 - g0) * s
            po += G * s
        want_dec = O.decode(want, dt, b - a, X, Y, max_exp, threads=THREADS)
        got_dec = synth.bits_numpy(back[a:b])
        assert np.array_equal(got_dec.view(want_dec.dtype.str.replace("f", "u")), want_dec.view(want_dec.dtype.str.replace("f", "u"))), (dtype, a, b)
        want_emu = O.emulate(host, X, Y, max_exp, threads=THREADS)
        got_emu = synth.bits_numpy(emu[a:b])
        assert np.array_equal(got_emu.view(want_emu.dtype.str.replace("f", "u")), want_emu.view(want_emu.dtype.str.replace("f", "u"))), (dtype, a, b)
    # a property that holds everywhere: decode(encode(x)) == emulate(x) for finite x
    view = torch.int16 if dtype == torch.bfloat16 else torch.int32
    assert torch.equal(back.view(view), emu.view(view))
    del back, emu, packed
    # histogram of the whole tensor (fused with a second encode) against a host count
    hist = exmy.exponent_histogram(x)
    p2, hist2 = exmy.encode_with_histogram(x, X, Y, max_exp)
    torch.cuda.synchronize()
    shift = 7 if dtype == torch.bfloat16 else 23
    want = np.zeros(256, dtype=np.int64)
    step = 1 << 28
    for a in range(0, n, step):
        part = x[a : a + step]
        e = (part.view(view).to(torch.int32) >> shift) & 0xFF
        want += torch.bincount(e.cpu(), minlength=256).numpy()
    assert want.sum() == n
    assert np.array_equal(hist.cpu().numpy(), want)
    assert np.array_equal(hist2.cpu().numpy(), want)
    host = synth.bits_numpy(x[: 1 << 22])
    assert np.array_equal(O.exponent_histogram(host), np.bincount((host.view(np.uint32 if dtype == torch.float32 else np.uint16) >> shift) & 0xFF, minlength=256).astype(np.uint64))


def block_shards(n, block, span=1 << 20):
    """Shards that start on a block boundary: at the start, across element 2^32 and at the ragged end."""
    per = max(1, span // block)
    mid = ((1 << 32) // block - per // 2) * block
    last = max(0, ((n - 1) // block - per + 1)) * block
    out = [(0, per * block), (mid, mid + per * block), (last, n)]
    return [(a, min(b, n)) for a, b in out if 0 <= a < n]


@pytest.mark.parametrize("block", [64, 11008])
def test_block_forms_beyond_4g(block):
    X, Y, W = 3, 3, 7
    n = (1 << 32) + 11008 * 40 + 8 * 5 + 3
    x = synth.gaussian_bf16(n, std=0.05, seed=23, device=DEV)
    x[::4099] *= 37.0  # spread the block maxima over several binades
    G = (n + 7) // 8
    meta = exmy.block_max_exp(x, block, X)
    packed, meta2 = exmy.encode_blocks_auto(x, block, X, Y, 0)
    packed2 = exmy.encode_blocks(x, block, X, Y, meta)
    back = exmy.decode_blocks(packed, torch.bfloat16, n, block, X, Y, meta)
    scale = exmy.block_scale(x, block, X, Y)
    spacked = exmy.encode_scaled(x, block, X, Y, scale)
    sback = exmy.decode_scaled(spacked, torch.bfloat16, n, block, X, Y, scale)
    torch.cuda.synchronize()
    assert torch.equal(meta, meta2) and torch.equal(packed, packed2)
    del packed2, meta2

    def plane_slices(p, g0, g1):
        out, po = [], 0
        for s in plane_sizes(W):
            out.append(p[po + g0 * s : po + g1 * s].cpu().numpy())
            po += G * s
        return np.concatenate(out)

    for a, b in block_shards(n, block):
        host = synth.bits_numpy(x[a:b])
        b0, b1 = a // block, (b + block - 1) // block
        want_meta = O.block_max_exp(host, block, X)
        assert np.array_equal(meta[b0:b1].cpu().numpy(), want_meta), (block, a, b)
        want = O.encode_blocks(host, block, X, Y, want_meta, threads=THREADS)
        assert np.array_equal(plane_slices(packed, a // 8, (b + 7) // 8), want), (block, a, b)
        want_dec = O.decode_blocks(want, O.BF16, b - a, block, X, Y, want_meta, threads=THREADS)
        assert np.array_equal(synth.bits_numpy(back[a:b]), want_dec), (block, a, b)
        want_scale = O.block_scale(host, block, X, Y)
        assert np.array_equal(scale[b0:b1].cpu().numpy().view(np.uint32), want_scale.view(np.uint32)), (block, a, b)
        want_s = O.encode_scaled(host, block, X, Y, want_scale, threads=THREADS)
        assert np.array_equal(plane_slices(spacked, a // 8, (b + 7) // 8), want_s), (block, a, b)
        want_sdec = O.decode_scaled(want_s, O.BF16, b - a, block, X, Y, want_scale, threads=THREADS)
        assert np.array_equal(synth.bits_numpy(sback[a:b]), want_sdec), (block, a, b)
    # everywhere: emulate == decode(encode) for these finite inputs
    emu = exmy.emulate_blocks(x.clone(), block, X, Y, meta)
    torch.cuda.synchronize()
    assert torch.equal(emu.view(torch.int16), back.view(torch.int16))


@pytest.mark.parametrize("cols, rows", [
    (4096, (1 << 20) + 8 * 3 + 5),  # a workgroup tile per 512 columns of a row block
    (128, (1 << 25) + 8 * 3 + 5),   # narrow: 4 row blocks per workgroup tile
    (136, (1 << 25) + 8 * 3 + 5),   # narrow, rows that start inside cache lines: tiles in die-ranged order
])
def test_row_packing_beyond_4g(cols, rows):
    # rows * cols > 2^32, ragged last row block, more than 2^20 workgroup tiles
    X, Y, W = 3, 3, 7
    x = synth.gaussian_bf16(rows * cols, std=0.05, seed=24, device=DEV).view(rows, cols)
    meta = exmy.block_max_exp(x.view(-1), cols, X)
    packed = exmy.encode_rows(x, X, Y, 0, meta)
    back = exmy.decode_rows(packed, torch.bfloat16, rows, cols, X, Y, 0, meta)
    torch.cuda.synchronize()
    R = (rows + 7) // 8
    # row blocks: the middle shard straddles byte offset 2^32 of the source, the last one element 2^32 and the ragged end
    mid = (1 << 32) // (16 * cols)  # the row block that holds byte offset 2^32 of the source
    for r0, r1 in ((0, 16), (mid - 8, mid + 8), (R // 2 + 3, R // 2 + 19), (R - 16, R)):
        a, b = 8 * r0, min(rows, 8 * r1)
        host = synth.bits_numpy(x[a:b])
        m = meta[a:b].cpu().numpy()
        want = O.encode_rows(host, b - a, cols, X, Y, 0, m)
        got, po, wo = [], 0, 0
        for s in plane_sizes(W):
            got.append(packed[po + r0 * cols * s : po + r1 * cols * s].cpu().numpy())
            po += R * cols * s
        assert np.array_equal(np.concatenate(got), want), (r0, r1)
        want_dec = O.decode_rows(want, O.BF16, b - a, cols, X, Y, 0, m)
        assert np.array_equal(synth.bits_numpy(back[a:b]), want_dec), (r0, r1)
    # everywhere: values equal those of the flat per-block codec with block = one row
    flat = exmy.decode_blocks(exmy.encode_blocks(x.view(-1), cols, X, Y, meta), torch.bfloat16, rows * cols, cols, X, Y, meta)
    torch.cuda.synchronize()
    assert torch.equal(flat.view(torch.int16), back.view(-1).view(torch.int16))


def test_tiles_and_columns_beyond_4g():
    X, Y, W = 3, 3, 7
    cols, tr, tc = 4096, 128, 128
    rows = (1 << 20) + 128 + 40  # rows * cols > 2^32; the last tile row is ragged
    n = rows * cols
    x = synth.gaussian_bf16(n, std=0.05, seed=25, device=DEV).view(rows, cols)
    x[::1031, ::67] *= 41.0  # spread the tile maxima over several binades
    G = n // 8
    ntc = cols // tc

    def plane_slices(p, g0, g1):
        out, po = [], 0
        for s in plane_sizes(W):
            out.append(p[po + g0 * s : po + g1 * s].cpu().numpy())
            po += G * s
        return np.concatenate(out)

    meta = exmy.tile_max_exp(x, tr, tc, X)
    packed = exmy.encode_tiles(x, tr, tc, X, Y, meta)
    back = exmy.decode_tiles(packed, torch.bfloat16, rows, cols, tr, tc, X, Y, meta)
    col_meta = exmy.tile_max_exp(x, rows, 1, X)
    col_packed = exmy.encode_tiles(x, rows, 1, X, Y, col_meta)
    col_back = exmy.decode_tiles(col_packed, torch.bfloat16, rows, cols, rows, 1, X, Y, col_meta)
    torch.cuda.synchronize()
    # the column maxima against a reduction by the tensor library (no Inf / NaN in this input)
    top = x.abs().amax(dim=0).float()
    want_cols = ((top.view(torch.int32) >> 23) & 0xFF).clamp(1 << X, 254).to(torch.uint8)
    assert torch.equal(col_meta, want_cols)
    cm = col_meta.cpu().numpy()
    last = (rows // tr) * tr
    # row shards on tile-row boundaries: the start, across element 2^32 (row 2^20) and the ragged end
    for r0, r1 in ((0, 2 * tr), ((1 << 20) - tr, (1 << 20) + tr), (last - tr, rows)):
        host = synth.bits_numpy(x[r0:r1]).reshape(r1 - r0, cols)
        t0, t1 = r0 // tr, (r1 + tr - 1) // tr
        want_meta = O.tile_max_exp(host, tr, tc, X)
        assert np.array_equal(meta[t0 * ntc : t1 * ntc].cpu().numpy(), want_meta), (r0, r1)
        want = O.encode_tiles(host, tr, tc, X, Y, want_meta, threads=THREADS)
        g0, g1 = r0 * cols // 8, r1 * cols // 8
        assert np.array_equal(plane_slices(packed, g0, g1), want), (r0, r1)
        want_dec = O.decode_tiles(want, O.BF16, r1 - r0, cols, tr, tc, X, Y, want_meta, threads=THREADS)
        assert np.array_equal(synth.bits_numpy(back[r0:r1]), want_dec.reshape(-1)), (r0, r1)
        # whole columns: every row shard uses the same per-column metadata
        want = O.encode_tiles(host, r1 - r0, 1, X, Y, cm, threads=THREADS)
        assert np.array_equal(plane_slices(col_packed, g0, g1), want), (r0, r1)
        want_dec = O.decode_tiles(want, O.BF16, r1 - r0, cols, r1 - r0, 1, X, Y, cm, threads=THREADS)
        assert np.array_equal(synth.bits_numpy(col_back[r0:r1]), want_dec.reshape(-1)), (r0, r1)
    # everywhere: emulate == decode(encode) for these finite inputs
    emu = exmy.emulate_tiles(x.clone(), tr, tc, X, Y, meta)
    torch.cuda.synchronize()
    assert torch.equal(emu.view(torch.int16), back.view(torch.int16))
    del emu, back
    emu = exmy.emulate_tiles(x.clone(), rows, 1, X, Y, col_meta)
    torch.cuda.synchronize()
    assert torch.equal(emu.view(torch.int16), col_back.view(torch.int16))
