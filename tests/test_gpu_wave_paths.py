"""Kernels that decide per wavefront whether rare work is needed (an Inf / NaN somewhere in
the wavefront, one metadatum shared by all of its lanes): inputs built so that every side
of those decisions is taken, each compared with the CPU oracle, tolerance 0."""
import numpy as np
import pytest
import torch

import paper_2405_13938_amd as exmy
from oracle import exmy_oracle as O
from paper_2405_13938_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
ODT = {torch.float32: O.F32, torch.bfloat16: O.BF16}


def ubits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else a


def tbits(t):
    return ubits(synth.bits_numpy(t))


def with_specials(x, where):
    """x with Inf / NaN patterns (both signs, NaNs with payloads) written at the given indices."""
    x = x.clone()
    if x.dtype == torch.bfloat16:
        pats = torch.tensor([0x7F80, 0xFF80, 0x7FC0, 0xFFA5, 0x7F81, 0xFFFF], dtype=torch.int32).to(torch.int16)
        v = x.view(torch.int16)
    else:
        pats = torch.tensor([0x7F800000, -0x00800000, 0x7FC00000, -0x005A0001, 0x7F800001, -1], dtype=torch.int32)
        v = x.view(torch.int32)
    for k, i in enumerate(where):
        v[i] = pats[k % len(pats)]
    return x


def cases(dtype, n):
    """(name, tensor): no special at all; one in the low half and one in the high half of a
    dword, in the first and the last lane of a wavefront; one per 16-byte vector; only specials."""
    base = synth.gaussian_bf16(n, 1.0, seed=11).to(dtype)
    per = 8 if dtype == torch.bfloat16 else 4  # elements per lane
    out = [("finite", base)]
    out.append(("two", with_specials(base, [0, 63 * per + 1])))
    out.append(("far apart", with_specials(base, [n // 2 + 1, n - 2])))
    out.append(("every lane", with_specials(base, list(range(3, n, per)))))
    out.append(("all", with_specials(base, list(range(n)))))
    return out


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_emulate_with_and_without_specials(dtype):
    n = 4 * 4096 + 24
    for name, x in cases(dtype, n):
        host = synth.bits_numpy(x)
        xd = x.to(DEV)
        for X, Y, me in ((3, 3, 128), (2, 1, 126), (4, 3, 131)):
            got = exmy.emulate(xd.clone(), X, Y, me)
            torch.cuda.synchronize()
            assert np.array_equal(tbits(got), ubits(O.emulate(host, X, Y, me))), ("emulate", name, X, Y, dtype)
            for block in (16, 64, 4096):
                meta = O.block_max_exp(host, block, X)
                got = exmy.emulate_blocks(xd.clone(), block, X, Y, torch.from_numpy(meta).to(DEV))
                torch.cuda.synchronize()
                want = O.emulate_blocks(host, block, X, Y, meta)
                assert np.array_equal(tbits(got), ubits(want)), ("emulate_blocks", name, block, X, Y, dtype)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_column_blocks_with_and_without_specials(dtype):
    rows, cols = 96, 512
    for name, x in cases(dtype, rows * cols):
        x2 = x.reshape(rows, cols).contiguous()
        host = synth.bits_numpy(x2).reshape(rows, cols)
        meta = O.tile_max_exp(host, rows, 1, 3)
        got = exmy.emulate_tiles(x2.to(DEV), rows, 1, 3, 3, torch.from_numpy(meta).to(DEV))
        torch.cuda.synchronize()
        want = O.emulate_tiles(host, rows, 1, 3, 3, meta)
        assert np.array_equal(tbits(got), ubits(want).reshape(-1)), ("emulate_tiles", name, dtype)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_reserved_codes_with_and_without_specials(dtype):
    n = 4 * 4096 + 24
    for name, x in cases(dtype, n):
        host = synth.bits_numpy(x)
        xd = x.to(DEV)
        for X, Y, me, kind in ((3, 3, 130, exmy.binding.SPECIALS_IEEE), (4, 3, 131, exmy.binding.SPECIALS_NAN_ONLY), (2, 1, 128, exmy.binding.SPECIALS_IEEE)):
            want = O.encode_specials(host, X, Y, me, kind)
            got = exmy.encode_specials(xd, X, Y, me, kind)
            torch.cuda.synchronize()
            assert np.array_equal(got.cpu().numpy(), want), ("encode_specials", name, X, Y, dtype)
            back = exmy.decode_specials(torch.from_numpy(want).to(DEV), dtype, n, X, Y, me, kind)
            torch.cuda.synchronize()
            assert np.array_equal(tbits(back), ubits(O.decode_specials(want, ODT[dtype], n, X, Y, me, kind))), ("decode_specials", name, X, Y, dtype)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_block_metadata_shared_or_not(dtype):
    """Blocks whose metadata all agree (every wavefront derives its constants once), alternate
    from block to block, or differ in a single block."""
    n = 6 * 4096 + 40
    x = synth.gaussian_bf16(n, 1.0, seed=5).to(dtype)
    host = synth.bits_numpy(x)
    xd = x.to(DEV)
    X, Y = 3, 3
    for block in (16, 32, 64, 512, 4096):
        nb = (n + block - 1) // block
        metas = {
            "same": np.full(nb, 129, np.uint8),
            "alternating": np.where(np.arange(nb) % 2 == 0, 129, 126).astype(np.uint8),
            "one differs": np.full(nb, 129, np.uint8),
            "wide path in one": np.full(nb, 129, np.uint8),
        }
        metas["one differs"][nb // 3] = 124
        metas["wide path in one"][nb // 2] = 250  # needs the fp64 rounding
        for name, meta in metas.items():
            md = torch.from_numpy(meta).to(DEV)
            want = O.encode_blocks(host, block, X, Y, meta)
            got = exmy.encode_blocks(xd, block, X, Y, md)
            torch.cuda.synchronize()
            assert np.array_equal(got.cpu().numpy(), want), ("encode_blocks", name, block, dtype)
            got = exmy.emulate_blocks(xd.clone(), block, X, Y, md)
            torch.cuda.synchronize()
            assert np.array_equal(tbits(got), ubits(O.emulate_blocks(host, block, X, Y, meta))), ("emulate_blocks", name, block, dtype)
