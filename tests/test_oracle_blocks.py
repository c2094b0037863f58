"""Pins of the CPU oracle's per-block-metadata functions: the paper's printed
block-dependent outcomes, a numpy definition of the block maximum exponent, and
reduction to the (separately pinned) per-tensor functions block by block."""
import numpy as np
import pytest
import torch

from oracle import exmy_oracle as O
from paper_2405_13938_amd import synth

F32, BF16 = O.F32, O.BF16


def as_np(t):
    return synth.bits_numpy(t)


def test_block_outcomes_e2m1(golden):
    # Section 2.1: outcomes (a)-(d) for one input value, by its block's maximum
    rows = golden("e2m1_block_outcomes.txt")
    block = 16
    for dtype in (torch.float32, torch.bfloat16):
        vals = torch.zeros(len(rows) * block, dtype=torch.float32)
        for r, (v, bmax, _, _) in enumerate(rows):
            vals[r * block + 5] = float(v)
            vals[r * block + 11] = float(bmax)
        x = vals.to(dtype)
        me = O.block_max_exp(as_np(x), block, 2)
        me_after = O.block_max_exp_after_rounding(as_np(x), block, 2, 1)
        for r, row in enumerate(rows):
            if row[3] == "after":
                me[r] = me_after[r]
        out = O.emulate_blocks(as_np(x), block, 2, 1, me)
        out_t = torch.from_numpy(out.view(np.int16 if dtype == torch.bfloat16 else np.int32)).view(dtype).float()
        for r, (v, bmax, want, _) in enumerate(rows):
            got = out_t[r * block + 5].item()
            assert got == float(want), (dtype, v, bmax, got, want)


def test_staircase_one_step_per_binade():
    # Section 2.1: with e2m1 there is one step between consecutive powers of two
    g = torch.Generator().manual_seed(5)
    x = (torch.rand(1 << 14, generator=g) * 3.0 + 1.0).float()  # [1, 4): top two binades of blocks whose max is in [2, 4)
    x[::16] = 3.5  # every block's maximum exponent is that of 2^1
    me = O.block_max_exp(as_np(x), 16, 2)
    assert (me == 128).all()
    out = torch.from_numpy(O.emulate_blocks(as_np(x), 16, 2, 1, me).view(np.float32))
    assert sorted(set(out.tolist())) == [1.0, 1.5, 2.0, 3.0]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("block,X", [(8, 0), (16, 2), (32, 4), (40, 3), (4096, 5), (1 << 20, 7)])
def test_block_max_exp_definition(dtype, block, X):
    g = torch.Generator().manual_seed(100 + block + X)
    n = 3 * 4096 + 1234
    # exponents spread over the whole fp32 range, with zeros, denormals, Inf and NaN mixed in
    x = torch.randn(n, generator=g) * torch.exp2(torch.randint(-140, 128, (n,), generator=g).float())
    x[torch.rand(n, generator=g) < 0.05] = 0.0
    x[torch.rand(n, generator=g) < 0.02] = float("inf")
    x[torch.rand(n, generator=g) < 0.02] = float("nan")
    x[torch.rand(n, generator=g) < 0.02] = 1e-41
    x[block: 2 * block] = float("nan") if n >= 2 * block else x[block: 2 * block]  # a block with no finite value
    x = x.to(dtype)
    got = O.block_max_exp(as_np(x), block, X)
    # definition: floor(log2 |x|) + 127 of the largest finite magnitude, 0 below the normals
    v = x.double().numpy()
    v = np.where(np.isfinite(v), np.abs(v), 0.0)
    nb = (n + block - 1) // block
    lo, hi = (1, 253) if X == 0 else (1 << X, 254)
    want = np.empty(nb, dtype=np.uint8)
    for b in range(nb):
        m = v[b * block: (b + 1) * block].max()
        _, e = np.frexp(m)  # m = f * 2^e, f in [0.5, 1)
        biased = int(e) - 1 + 127 if m >= 2.0 ** -126 else 0
        want[b] = min(max(biased, lo), hi)
    assert np.array_equal(got, want)


def per_block_reference(x_np, dt, n, block, X, Y, meta):
    """Codes from the per-tensor oracle applied to each block with its own metadatum."""
    lo, hi = (1, 253) if X == 0 else (1 << X, 254)
    codes = np.empty(n, dtype=np.uint32)
    for b in range((n + block - 1) // block):
        s = slice(b * block, min(n, (b + 1) * block))
        codes[s] = O.to_codes(x_np[s], X, Y, int(min(max(int(meta[b]), lo), hi)))
    return codes


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("X,Y,block", [(2, 1, 16), (3, 3, 32), (1, 2, 64), (0, 3, 8), (4, 3, 24), (3, 2, 4096),
                                       (5, 2, 520), (2, 3, 512), (7, 0, 1024), (0, 0, 8), (4, 7, 128)])
def test_blocks_reduce_to_per_tensor_functions(dtype, X, Y, block):
    g = torch.Generator().manual_seed(1000 * X + 10 * Y + block)
    n = 5 * block + 8 * 3 + 5 if block <= 1024 else 2 * block + 77
    x = torch.randn(n, generator=g) * torch.exp2(torch.randint(-12, 6, (n,), generator=g).float())
    x[::97] = float("inf")
    x[::89] = float("-inf")
    x[::83] = float("nan")
    x = x.to(dtype)
    xn = as_np(x)
    dt = F32 if dtype == torch.float32 else BF16
    nb = (n + block - 1) // block
    for kind in ("before_rounding", "random_bytes"):
        if kind == "before_rounding":
            meta = O.block_max_exp(xn, block, X)
        else:  # any byte is accepted and read as the nearest valid metadatum
            meta = np.random.default_rng(block).integers(0, 256, nb).astype(np.uint8)
        codes = per_block_reference(xn, dt, n, block, X, Y, meta)
        packed = O.encode_blocks(xn, block, X, Y, meta)
        assert np.array_equal(packed, O.pack(codes, 1 + X + Y))
        # decode: per block through the per-tensor function
        dec = O.decode_blocks(packed, dt, n, block, X, Y, meta)
        lo, hi = (1, 253) if X == 0 else (1 << X, 254)
        for b in range(nb):
            s = slice(b * block, min(n, (b + 1) * block))
            want = O.from_codes(codes[s], dt, X, Y, int(min(max(int(meta[b]), lo), hi)))
            assert np.array_equal(dec[s].view(np.uint8), want.view(np.uint8))
        # emulate = decode(encode) away from Inf / NaN, which stay bit-identical
        emu = O.emulate_blocks(xn, block, X, Y, meta)
        fin = torch.isfinite(x.float()).numpy()
        u = np.uint32 if dtype == torch.float32 else np.uint16
        assert np.array_equal(emu.view(u)[fin], dec.view(u)[fin])
        assert np.array_equal(emu.view(u)[~fin], xn.view(u)[~fin])


def test_uniform_metadata_equals_per_tensor():
    x = synth.gaussian_bf16(40000, seed=9)
    xn = as_np(x)
    for X, Y, me in [(3, 3, 127), (2, 1, 129), (0, 4, 126)]:
        meta = np.full((xn.size + 63) // 64, me, dtype=np.uint8)
        assert np.array_equal(O.encode_blocks(xn, 64, X, Y, meta), O.encode(xn, X, Y, me))


def test_block_validation():
    x = as_np(torch.zeros(64))
    meta = np.zeros(8, dtype=np.uint8)
    with pytest.raises(Exception):
        O.block_max_exp(x, 12, 3)  # not a multiple of 8
    with pytest.raises(Exception):
        O.block_max_exp(x, 8, 8)  # X = 8 has no per-block metadata
    with pytest.raises(Exception):
        O.encode_blocks(x, 0, 3, 3, meta)
    with pytest.raises(Exception):
        O.encode_blocks(x, 8, 8, 3, meta)


@pytest.mark.parametrize("tdtype,Y", [(torch.bfloat16, 7), (torch.float16, 10), (torch.float8_e5m2, 2),
                                      (torch.float8_e4m3fn, 3), (torch.float8_e8m0fnu, 0)])
def test_after_rounding_matches_library_rounding(tdtype, Y):
    # rounding an fp32 value to Y mantissa bits is what the library conversion to a float type with
    # Y mantissa bits does, wherever the value is a normal of that type
    g = torch.Generator().manual_seed(Y)
    n, block = 1 << 15, 8
    x = torch.randn(n, generator=g) * torch.exp2(torch.randint(-5, 6, (n,), generator=g).float())
    x[::5] = (1.0 + torch.randint(0, 1 << Y, (x[::5].numel(),), generator=g).float() / (1 << Y) + 2.0 ** -(Y + 1)) * 2  # ties
    x[1::5] = 2.0 - 2.0 ** -(Y + 2)  # rounds up into the next binade
    m = x.abs().reshape(-1, block).max(dim=1).values
    rounded = m.to(tdtype).float()
    assert torch.isfinite(rounded).all()
    want = (rounded.view(torch.int32) >> 23) & 0xFF
    X = 5  # valid range [32, 254] holds every exponent met here
    got = O.block_max_exp_after_rounding(x.numpy(), block, X, Y)
    assert np.array_equal(got, want.numpy().astype(np.uint8))
    before = O.block_max_exp(x.numpy(), block, X)
    assert ((got == before) | (got == before + 1)).all() and (got != before).any()


def test_after_rounding_never_cuts_the_block_maximum():
    # Section 2.1: the scheme exists "to prevent excessive truncation of the largest value in the block"
    g = torch.Generator().manual_seed(3)
    for dtype in (torch.float32, torch.bfloat16):
        x = (torch.randn(1 << 14, generator=g) * torch.exp2(torch.randint(-20, 20, (1 << 14,), generator=g).float())).to(dtype)
        xn = as_np(x)
        for X, Y, block in ((2, 1, 16), (3, 2, 32), (1, 3, 64), (0, 3, 8), (4, 0, 128), (0, 1, 16)):
            me = O.block_max_exp_after_rounding(xn, block, X, Y)
            emu = O.emulate_blocks(xn, block, X, Y, me)
            e = torch.from_numpy(emu.view(np.int16 if dtype == torch.bfloat16 else np.int32)).view(dtype).double().abs()
            m = x.double().abs().reshape(-1, block).max(dim=1).values
            em = e.reshape(-1, block).max(dim=1).values
            # the emulated maximum is the grid point nearest to the true maximum: off by at most half a step
            # of the maximum's own binade, whose mantissa width is that of the format's top binade
            bits = (Y - 1 if Y else 0) if X == 0 else Y
            half_step = torch.exp2(torch.floor(torch.log2(m)) - bits - 1)
            assert ((em - m).abs() <= half_step).all(), (X, Y, block)
            # while "before rounding" does cut some maxima in the same data when the top mantissa is all ones
            if X >= 1 and Y >= 1:
                me0 = O.block_max_exp(xn, block, X)
                assert ((me == me0) | (me == me0 + 1)).all()


def test_after_rounding_special_blocks():
    x = np.zeros(64, dtype=np.float32)
    x[8:16] = np.inf
    x[16:24] = np.nan
    x[24] = 3.4028235e38   # rounds up past the largest finite float: clamps to 254
    x[32] = 1e-40          # below the normals: exponent 0, clamped up to the smallest valid metadatum
    x[40] = 1.9999999      # rounds to 2.0 with any Y < 23
    x[48] = 1.9999999
    got = O.block_max_exp_after_rounding(x, 8, 3, 3)
    assert got.tolist() == [8, 8, 8, 254, 8, 128, 128, 8]
    assert O.block_max_exp_after_rounding(x, 8, 3, 23).tolist() == [8, 8, 8, 254, 8, 127, 127, 8]
    assert O.block_max_exp(x, 8, 3).tolist() == [8, 8, 8, 254, 8, 127, 127, 8]
