"""Pins of the CPU oracle's float-scaling scheme (one fp32 scale per block, codes
of the max_exp = 127 format): the paper's 3.9 example for the three schemes, the
library's bf16 rounding, exact equivalence with the power-of-two metadata when
the scale is a power of two, and a brute-force nearest-value search."""
import numpy as np
import pytest
import torch

from oracle import exmy_oracle as O
from paper_2405_13938_amd import synth

F32, BF16 = O.F32, O.BF16


def as_np(t):
    return synth.bits_numpy(t)


def to_torch(a, dtype):
    return torch.from_numpy(a.view(np.int16 if dtype == torch.bfloat16 else np.int32)).view(dtype)


def test_three_schemes_on_3p9(golden):
    want = {k: float(v) for k, v in golden("e2m1_schemes_3p9.txt")}
    for dtype in (torch.float32, torch.bfloat16):
        x = torch.zeros(16)
        x[3], x[7], x[9] = 3.9, -1.2, 0.4
        x = x.to(dtype)
        xn = as_np(x)
        before = to_torch(O.emulate_blocks(xn, 16, 2, 1, O.block_max_exp(xn, 16, 2)), dtype)
        after = to_torch(O.emulate_blocks(xn, 16, 2, 1, O.block_max_exp_after_rounding(xn, 16, 2, 1)), dtype)
        scaled = to_torch(O.emulate_scaled(xn, 16, 2, 1, O.block_scale(xn, 16, 2, 1)), dtype)
        assert before[3].item() == want["before_rounding"]
        assert after[3].item() == want["after_rounding"]
        # "accurately": to the precision of the container (the printed 3.9 is not a bf16 value itself)
        tol = 2.0 ** -22 if dtype == torch.float32 else 2.0 ** -8
        assert abs(scaled[3].item() - want["float_scale"]) <= tol * 3.9 + abs(x[3].item() - 3.9)


def test_bf16_rounding_is_the_library_conversion():
    g = torch.Generator().manual_seed(1)
    bits = torch.randint(0, 2 ** 32, (200000,), generator=g, dtype=torch.int64)
    # ties, carries into the next binade, the overflow edge, denormals
    extra = [0x3F808000, 0x3F818000, 0x3F80FFFF, 0x3FFF8000, 0x7F7F8000, 0x7F7F7FFF, 0x00008000, 0x00018000,
             0x00000001, 0x007FFFFF, 0x00800000, 0x7F7FFFFF, 0x0, 0x80000000]
    bits = torch.cat([bits, torch.tensor(extra, dtype=torch.int64)])
    bits = torch.where(bits >= 2 ** 31, bits - 2 ** 32, bits).to(torch.int32)
    x = bits.view(torch.float32)
    keep = torch.isfinite(x)
    x = x[keep]
    want = x.to(torch.bfloat16).view(torch.int16).to(torch.int32) & 0xFFFF
    got = torch.tensor([O.round_to_bf16_bits(v) >> 16 for v in x.tolist()], dtype=torch.int32)
    assert torch.equal(got, want)


def test_bf16_scale_is_the_smallest_bf16_not_below_the_fp32_scale():
    """Section 2 "Metadata" offers a bfloat16 scaling factor.  Checked through the library's bf16 conversion:
    its round-to-nearest result, moved one bf16 up where it fell below the fp32 scale."""
    g = torch.Generator().manual_seed(9)
    n, block = 1 << 15, 16
    x = torch.randn(n, generator=g) * torch.exp2(torch.randint(-60, 60, (n,), generator=g).float())
    x[0:16] = 0.0
    x[16:32] = 3.4e38  # with e1m0 (largest value 1) the scale exceeds the largest finite bf16
    xn = as_np(x)
    for X, Y in ((1, 0), (2, 1), (3, 3), (0, 4), (5, 2)):
        s32 = O.block_scale(xn, block, X, Y)
        s16 = O.block_scale(xn, block, X, Y, bf16=True)
        assert s16.dtype == np.uint16
        near = torch.from_numpy(s32).bfloat16()
        bits = near.view(torch.int16).numpy().astype(np.int64) & 0xFFFF
        bits = bits + (near.float().numpy() < s32)            # positive values: the next bf16 is the next pattern
        bits = np.minimum(bits, 0x7F7F)                        # Inf is not a scale
        assert np.array_equal(s16.astype(np.int64), bits), (X, Y)
        wide = (s16.astype(np.uint32) << 16).view(np.float32)
        capped = s16 == 0x7F7F
        assert (wide[~capped] >= s32[~capped]).all() and s16[0] == 0x0080
        assert (((s16[~capped].astype(np.uint32) - 1) << 16).view(np.float32) < s32[~capped]).all()
        # the block maximum stays inside the format: its scaled value does not exceed the largest value by more
        # than the two roundings of the scaling
        m = torch.where(torch.isfinite(x), x.abs(), torch.zeros(())).reshape(-1, block).max(dim=1).values.numpy()
        a = m * (np.float32(1.0) / wide)
        assert (a[~capped] <= np.float32(vmax_of(X, Y)) * np.float32(1 + 2.0 ** -22)).all()
        # bf16 scales are used widened: same results as the fp32 array of those values
        assert np.array_equal(O.encode_scaled(xn, block, X, Y, s16), O.encode_scaled(xn, block, X, Y, wide))
        assert np.array_equal(O.emulate_scaled(xn, block, X, Y, s16).view(np.uint32), O.emulate_scaled(xn, block, X, Y, wide).view(np.uint32))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("X,Y", [(2, 1), (3, 3), (1, 2), (0, 3), (4, 3), (7, 0), (0, 1), (5, 7)])
def test_power_of_two_scale_equals_power_of_two_metadata(dtype, X, Y):
    # scaling by 2^k is exact, so codes and decoded values must equal those of max_exp = 127 + k
    x = synth.shuffled(synth.all_bf16_patterns(), 7).to(dtype)
    x = x[torch.isfinite(x.float()) & ((x.float().abs() > 1e-25) | (x.float() == 0)) & (x.float().abs() < 1e25)]
    x = x[: (x.numel() // 64) * 64]
    xn = as_np(x)
    block = 64
    nb = x.numel() // block
    lo, hi = (1, 253) if X == 0 else (1 << X, 254)
    k = np.random.default_rng(X * 10 + Y).integers(-20, 21, nb)
    k = np.clip(127 + k, max(lo, 107), min(hi, 147)) - 127
    scale = np.ldexp(np.float32(1.0), k).astype(np.float32)
    meta = (127 + k).astype(np.uint8)
    dt = F32 if dtype == torch.float32 else BF16
    packed = O.encode_scaled(xn, block, X, Y, scale)
    assert np.array_equal(packed, O.encode_blocks(xn, block, X, Y, meta))
    a = O.decode_scaled(packed, dt, x.numel(), block, X, Y, scale)
    b = O.decode_blocks(packed, dt, x.numel(), block, X, Y, meta)
    assert np.array_equal(a.view(np.uint8), b.view(np.uint8))
    assert np.array_equal(O.emulate_scaled(xn, block, X, Y, scale).view(np.uint8),
                          O.emulate_blocks(xn, block, X, Y, meta).view(np.uint8))


def vmax_of(X, Y):
    return max(O.code_value(X, Y, 127, c) for c in range(1 << (X + Y)))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_block_scale_definition_and_block_maximum_is_kept(dtype):
    g = torch.Generator().manual_seed(2)
    n, block = 1 << 14, 32
    x = torch.randn(n, generator=g) * torch.exp2(torch.randint(-30, 30, (n,), generator=g).float())
    x[torch.rand(n, generator=g) < 0.02] = float("inf")
    x[torch.rand(n, generator=g) < 0.02] = float("nan")
    x[0:32] = 0.0            # all-zero block
    x[32:64] = float("nan")  # no finite value
    x[64:96] = 1e-42         # so small that the scale would leave the normals
    x = x.to(dtype)
    xn = as_np(x)
    for X, Y in ((2, 1), (3, 3), (0, 3), (1, 2), (4, 3), (7, 0)):
        vmax = vmax_of(X, Y)
        s = O.block_scale(xn, block, X, Y)
        v = x.float()
        m = torch.where(torch.isfinite(v), v.abs(), torch.zeros(())).reshape(-1, block).max(dim=1).values.numpy()
        want = np.maximum(m.astype(np.float32) / np.float32(vmax), np.float32(2.0 ** -126))
        assert np.array_equal(s, want)
        assert s[0] == s[1] == s[2] == np.float32(2.0 ** -126)
        # Section 2.1: the scheme reproduces the block maximum (here: to 2 ulp of the container)
        emu = to_torch(O.emulate_scaled(xn, block, X, Y, s), dtype).double()
        em = torch.where(torch.isfinite(emu), emu.abs(), torch.zeros((), dtype=torch.double)).reshape(-1, block).max(dim=1).values.numpy()
        ulp = 2.0 ** -22 if dtype == torch.float32 else 2.0 ** -7
        ok = np.abs(em - m.astype(np.float64)) <= ulp * m
        assert ok[3:].all(), (X, Y)


@pytest.mark.parametrize("X,Y", [(2, 1), (3, 2), (1, 3), (0, 4), (4, 3)])
def test_scaled_codes_are_the_nearest_grid_points(X, Y):
    g = torch.Generator().manual_seed(X + 10 * Y)
    n, block = 1 << 13, 16
    x = (torch.randn(n, generator=g) * torch.exp2(torch.randint(-6, 6, (n,), generator=g).float())).float()
    xn = x.numpy()
    s = O.block_scale(xn, block, X, Y)
    packed = O.encode_scaled(xn, block, X, Y, s)
    codes = O.unpack(packed, n, 1 + X + Y)
    grid = np.array([O.code_value(X, Y, 127, c) for c in range(1 << (X + Y))])  # ascending magnitudes
    mag = codes & ((1 << (X + Y)) - 1)
    sign = codes >> (X + Y)
    assert np.array_equal(sign, (xn < 0).astype(codes.dtype) | (np.signbit(xn)).astype(codes.dtype))
    t = np.abs(xn.astype(np.float64)) / np.repeat(s.astype(np.float64), block)  # exact quotient, to fp64
    t = np.minimum(t, grid[-1])
    best = np.abs(grid[None, :] - t[:, None]).min(axis=1)
    got = np.abs(grid[mag] - t)
    # nearest, except that the fp32 rounding of the product may swap the two neighbours of a near-tie
    assert (got <= best + 4e-7 * np.maximum(t, grid[1])).all()
    # and the decoded value is the grid point times the scale, rounded once
    dec = O.decode_scaled(packed, F32, n, block, X, Y, s)
    want = (grid[mag].astype(np.float32) * np.repeat(s, block)).astype(np.float32) * np.where(sign == 1, -1.0, 1.0).astype(np.float32)
    assert np.array_equal(dec.view(np.uint32), want.view(np.uint32))


def test_bf16_results_are_the_fp32_results_rounded_by_the_library():
    g = torch.Generator().manual_seed(11)
    n, block = 1 << 14, 32
    x = (torch.randn(n, generator=g) * torch.exp2(torch.randint(-20, 20, (n,), generator=g).float())).bfloat16()
    xn = as_np(x)
    for X, Y in ((2, 1), (3, 3), (0, 4), (4, 3)):
        s = O.block_scale(xn, block, X, Y)
        s = (s * np.float32(1.2345)).astype(np.float32)  # not a power of two: products need rounding
        packed = O.encode_scaled(xn, block, X, Y, s)
        d32 = O.decode_scaled(packed, F32, n, block, X, Y, s)
        d16 = O.decode_scaled(packed, BF16, n, block, X, Y, s)
        want = torch.from_numpy(d32).bfloat16()
        assert np.array_equal(d16, want.view(torch.int16).numpy().view(np.uint16))
        assert (torch.from_numpy(d32) != want.float()).any()  # the rounding really happens


def test_scaled_validation():
    x = np.zeros(64, dtype=np.float32)
    s = np.ones(8, dtype=np.float32)
    for bad in ((8, 3), (0, 0), (9, 1), (-1, 2)):
        with pytest.raises(Exception):
            O.block_scale(x, 8, *bad)
        with pytest.raises(Exception):
            O.encode_scaled(x, 8, bad[0], bad[1], s)
    with pytest.raises(Exception):
        O.encode_scaled(x, 12, 3, 3, s)
    with pytest.raises(Exception):
        O.encode_scaled(x, 8, 3, 13, s)  # packed form stops at 16 bits
    O.emulate_scaled(x, 8, 3, 13, s)     # emulation does not
