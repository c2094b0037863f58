"""Pins of the CPU oracle's float-scaling scheme (one fp32 scale per block, codes
of the max_exp = 127 format): the paper's 3.9 example for the three schemes, the
library's bf16 rounding, exact equivalence with the power-of-two metadata when
the scale is a power of two, and a brute-force nearest-value search."""
import bisect
import math
from fractions import Fraction

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


def nearest_code_exact(grid, a, s):
    """Index of the grid point nearest the rational a / s, ties to the even index, by exact integer
    arithmetic (grid: ascending Fractions)."""
    t = Fraction(float(a)) / Fraction(float(s))
    if t >= grid[-1]:
        return len(grid) - 1
    hi = bisect.bisect_right(grid, t)      # grid[hi - 1] <= t < grid[hi]
    lo = hi - 1
    d_lo, d_hi = t - grid[lo], grid[hi] - t
    if d_lo != d_hi:
        return lo if d_lo < d_hi else hi
    return lo if lo % 2 == 0 else hi


def near_boundary_inputs(grid, rng, count):
    """(x, scale) pairs, one element per block, whose quotient lies within an fp32 rounding error of a rounding
    boundary of the grid (the midpoint of two neighbouring grid points), on either side of it or exactly on it:
    the inputs on which a quotient computed in fp32 (a division, or a multiplication by a reciprocal) picks the
    wrong neighbour."""
    xs, ss = [], []
    mids = [(grid[i] + grid[i + 1]) / 2 for i in range(len(grid) - 1)]
    while len(xs) < count:
        m = mids[int(rng.integers(len(mids)))]
        if rng.random() < 0.25:
            s = np.float32(np.ldexp(float(rng.integers(1, 1 << 8)), int(rng.integers(-20, 20))))  # few bits: m * s is an fp32
        else:
            s = np.float32(np.ldexp(1.0 + rng.random(), int(rng.integers(-40, 40))))
        x = np.float32(float(m * Fraction(float(s))))      # the fp32 nearest the boundary's preimage
        x = np.nextafter(x, np.float32(np.inf if rng.random() < 0.5 else 0), dtype=np.float32) if rng.random() < 0.5 else x
        xs.append(x if rng.random() < 0.5 else -x)
        ss.append(s)
    return np.array(xs, dtype=np.float32), np.array(ss, dtype=np.float32)


@pytest.mark.parametrize("X,Y", [(2, 1), (3, 2), (1, 3), (0, 4), (4, 3), (3, 0), (5, 10), (7, 1)])
def test_scaled_codes_are_the_nearest_grid_points(X, Y):
    """The code is that of the real quotient |x| / s: nearest grid point, ties to even, found here with exact
    rational arithmetic on random data and on inputs built to sit on or next to a rounding boundary."""
    g = torch.Generator().manual_seed(X + 10 * Y)
    n, block = 1 << 11, 16
    x = (torch.randn(n, generator=g) * torch.exp2(torch.randint(-6, 6, (n,), generator=g).float())).float()
    xn = x.numpy()
    s = O.block_scale(xn, block, X, Y)
    grid = [Fraction(O.code_value(X, Y, 127, c)) for c in range(1 << (X + Y))]  # ascending magnitudes
    assert all(p < q for p, q in zip(grid, grid[1:]))

    def check(xn, s, block):
        codes = O.unpack(O.encode_scaled(xn, block, X, Y, s), xn.size, 1 + X + Y)
        mag = codes & ((1 << (X + Y)) - 1)
        assert np.array_equal(codes >> (X + Y), np.signbit(xn).astype(codes.dtype))
        want = [nearest_code_exact(grid, abs(v), s[i // block]) for i, v in enumerate(xn.tolist())]
        if Y == 0:  # an exact tie goes to the even significand, which for Y = 0 is the next binade (the code above)
            ties = [i for i, v in enumerate(xn.tolist())
                    if mag[i] != want[i] and mag[i] == want[i] + 1
                    and Fraction(abs(v)) / Fraction(float(s[i // block])) == (grid[want[i]] + grid[mag[i]]) / 2]
            for i in ties:
                assert want[i] >= 1  # between two normals, not at the top of the subnormal range
                want[i] += 1
        assert np.array_equal(mag, np.array(want, dtype=mag.dtype))
        return mag

    check(xn, s, block)
    bx, bs = near_boundary_inputs(grid, np.random.default_rng(X * 100 + Y), 3000)
    pad = np.zeros((bx.size, 8), dtype=np.float32)
    pad[:, 0] = bx
    mag = check(pad.reshape(-1), bs, 8)
    # the built inputs really are decided by less than an fp32 rounding error: the fp32 quotient
    # |x| * fl(1 / s) rounded onto the grid differs from the exact result on some of them
    q32 = (np.abs(bx) * (np.float32(1.0) / bs)).astype(np.float32)
    naive = np.array([nearest_code_exact(grid, q, 1.0) for q in q32.tolist()])
    assert (naive != mag[::8]).any()


def nearest_in_container_exact(p, mant_bits, emin):
    """Fraction p >= 0 rounded to nearest, ties to even, onto the floating-point grid with `mant_bits` stored
    mantissa bits and smallest normal 2^emin (denormals below), as a Fraction; no overflow handling."""
    if p == 0:
        return p
    e = max(math.floor(math.log2(p)) if p >= 1 else -math.ceil(math.log2(1 / p)), emin)
    while Fraction(2) ** e > p and e > emin:
        e -= 1
    while Fraction(2) ** (e + 1) <= p:
        e += 1
    q = Fraction(2) ** (e - mant_bits)
    k = p / q
    lo = k.numerator // k.denominator
    r = k - lo
    if r > Fraction(1, 2) or (r == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    return lo * q


@pytest.mark.parametrize("dt,torch_dt,mant,emin", [(F32, torch.float32, 23, -126), (BF16, torch.bfloat16, 7, -126),
                                                 (O.F16, torch.float16, 10, -14)])
def test_scaled_decode_is_the_exact_product_rounded_once(dt, torch_dt, mant, emin):
    """Decoded value = grid value * scale as a real number, rounded once into the container.  For bf16 and fp16
    that is not the fp32 product rounded again: the test searches for products whose fp32 rounding lands exactly
    on a tie of the narrower type and checks that the result follows the real product there."""
    X, Y = (3, 3) if dt != O.F16 else (3, 5)
    rng = np.random.default_rng(5 + dt)
    ncodes = 1 << (X + Y)
    grid = np.array([O.code_value(X, Y, 127, c) for c in range(ncodes)])
    trials = 1 << 22
    c = rng.integers(1, ncodes, trials)
    lo_e, hi_e = (-20, 20) if dt != O.F16 else (-18, 8)   # fp16: results from deep denormals to near the top
    s = np.ldexp(1.0 + rng.random(trials), rng.integers(lo_e, hi_e, trials)).astype(np.float32)
    exact = grid[c] * s.astype(np.float64)                # exact: at most 7 + 24 bits
    p32 = exact.astype(np.float32)
    keep = np.zeros(trials, dtype=bool)
    keep[:4096] = True
    if dt != F32:
        # fp32 product inexact and exactly half-way between two values of the narrower type
        narrow = torch.from_numpy(p32).to(torch_dt).float().numpy().astype(np.float64)
        up = torch.nextafter(torch.from_numpy(p32).to(torch_dt), torch.tensor(float("inf"), dtype=torch_dt)).float().numpy().astype(np.float64)
        dn = torch.nextafter(torch.from_numpy(p32).to(torch_dt), torch.tensor(float("-inf"), dtype=torch_dt)).float().numpy().astype(np.float64)
        p = p32.astype(np.float64)
        tie = ((p - narrow == up - p) | (narrow - p == p - dn)) & (p != narrow)
        hazard = tie & (p != exact)
        assert hazard.sum() >= 8
        keep |= hazard
    c, s, exact = c[keep], s[keep], exact[keep]
    n = c.size // 8 * 8
    c, s, exact = c[:n], s[:n], exact[:n]
    sign = rng.integers(0, 2, n)
    codes = (c | (sign << (X + Y))).astype(np.uint32)
    packed = O.pack(codes, 1 + X + Y)
    got = O.decode_scaled(packed, dt, n, 8, X, Y, np.repeat(s.reshape(-1, 8)[:, :1], 8, axis=1).reshape(-1)[::8].copy())
    # one scale per block of 8: rebuild the products with the scale each element really got
    s_used = np.repeat(s[::8], 8)
    got = to_torch(got, torch_dt).double().numpy()
    want = np.array([float(nearest_in_container_exact(Fraction(float(grid[ci])) * Fraction(float(si)), mant, emin))
                     for ci, si in zip(c.tolist(), s_used.tolist())])
    want = np.where(sign == 1, -want, want)
    assert np.array_equal(got, want)
    if dt != F32:
        twice = torch.from_numpy((grid[c] * s_used.astype(np.float64)).astype(np.float32)).to(torch_dt).double().numpy()
        twice = np.where(sign == 1, -twice, twice)
        # the search is over (code, scale) pairs; after regrouping by block only the first of each 8 keeps its scale
        assert (np.abs(twice[::8]) != np.abs(got[::8])).any()  # rounding the fp32 product again would differ


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
