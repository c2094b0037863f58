"""Pins of the CPU oracle's number format against things other than itself:
values the paper prints (tests/golden/), library float8 / bfloat16 / float16
conversions, and a brute-force nearest-value search over textbook value sets."""
import math

import numpy as np
import pytest
import torch

from oracle import exmy_oracle as O
from paper_2405_13938_amd import synth

F32, BF16 = O.F32, O.BF16


def max_exp_for_bias(X, bias):
    # the top exponent code 2^X-1 stands for 2^(2^X-1-bias); biased by 127
    return (1 << X) - 1 - bias + 127


def textbook_values(X, Y, max_exp):
    """Non-negative value set, by magnitude code, in the usual float reading:
    bias b, normals 2^(E-b)(1+M/2^Y), subnormals 2^(1-b) M/2^Y."""
    b = (1 << X) - 1 + 127 - max_exp
    vals = []
    for c in range(1 << (X + Y)):
        E, M = c >> Y, c & ((1 << Y) - 1)
        if E == 0:
            vals.append(math.ldexp(M, 1 - b - Y))
        else:
            vals.append(math.ldexp((1 << Y) + M, E - b - Y))
    if X == 8:  # exponent code 255 is not used: clamp at the largest finite float
        top = (254 << Y) | ((1 << Y) - 1)
        vals = vals[: top + 1]
    return np.array(vals, dtype=np.float64)


def brute_force_codes(a, vals):
    """Index of the nearest member of the ascending array vals to each a >= 0,
    saturating at the top.  A tie goes to the neighbour that is an even multiple of
    the spacing at a (round-half-even on the significand): the even code when
    Y >= 1, and the next power of two when Y = 0 leaves a 1-digit significand."""
    a = np.asarray(a, dtype=np.float64)
    hi = np.searchsorted(vals, a, side="left")
    hi = np.clip(hi, 1, len(vals) - 1)
    lo = hi - 1
    two_a, s = 2.0 * a, vals[lo] + vals[hi]  # both exact in double
    q = vals[hi] - vals[lo]
    lo_odd = np.mod(vals[lo] / q, 2.0) == 1.0
    pick_hi = (two_a > s) | ((two_a == s) & lo_odd)
    c = np.where(pick_hi, hi, lo)
    c = np.where(a >= vals[-1], len(vals) - 1, c)
    return c.astype(np.uint32)


# ---------------------------------------------------------------- paper values


def test_table1_biases_and_ranges(golden):
    for name, X, Y, bias, lo, hi in golden("table1_formats.txt"):
        X, Y, bias = int(X), int(Y), int(bias)
        max_exp = max_exp_for_bias(X, bias)
        if X == 8:
            assert max_exp == 255, name  # bias 127 <=> identity exponent map
        smallest_normal = O.code_value(X, Y, max_exp, 1 << Y)
        assert smallest_normal == math.ldexp(1.0, 1 - bias), name
        if lo != "-":
            assert smallest_normal == math.ldexp(1.0, int(lo)), name
            # largest value lies in the binade 2^hi
            top = max(O.code_value(X, Y, max_exp, c) for c in range((1 << (X + Y)) - 8, 1 << (X + Y)))
            assert math.floor(math.log2(top)) == int(hi), name


def test_e3m3_bias_examples(golden):
    for X, Y, bias, lo, hi in golden("e3m3_bias_examples.txt"):
        X, Y, bias, lo, hi = map(int, (X, Y, bias, lo, hi))
        max_exp = max_exp_for_bias(X, bias)
        assert max_exp == hi + 127
        assert O.code_value(X, Y, max_exp, 1 << Y) == 2.0 ** lo
        assert O.code_value(X, Y, max_exp, ((1 << X) - 1) << Y) == 2.0 ** hi
        # largest subnormal sits one quantum under the smallest normal
        q = 2.0 ** (lo - Y)
        assert O.code_value(X, Y, max_exp, (1 << Y) - 1) == 2.0 ** lo - q


def test_integer_formats(golden):
    for name, X, Y, lo, hi in golden("integer_formats.txt"):
        X, Y, lo, hi = int(X), int(Y), int(lo), int(hi)
        # choose max_exp so that the quantum is 1: the largest value hi has biased exponent
        max_exp = 127 + int(math.floor(math.log2(hi)))
        vals = [O.code_value(X, Y, max_exp, c) for c in range(1 << (1 + X + Y))]
        assert sorted(set(vals)) == [float(v) for v in range(lo, hi + 1)], name
        half = 1 << (X + Y)
        assert vals[0] == 0.0 and vals[half] == 0.0 and math.copysign(1, vals[half]) == -1.0  # double zero
        assert [abs(v) for v in vals[half:]] == vals[:half]


def test_e1mY_equals_e0mY1_bit_for_bit():
    x = synth.f32_edge_sweep()
    xs = synth.bits_numpy(x)
    for Y in (0, 2, 5):
        for max_exp in (100, 127, 140):
            a = O.to_codes(xs, 1, Y, max_exp)
            b = O.to_codes(xs, 0, Y + 1, max_exp)
            assert np.array_equal(a, b)
            assert np.array_equal(O.emulate(xs, 1, Y, max_exp).view(np.uint32), O.emulate(xs, 0, Y + 1, max_exp).view(np.uint32))


def test_format_counts(golden):
    rows = dict(golden("format_counts.txt"))
    fmts = [(X, W - 1 - X) for W in range(1, 9) for X in range(0, W)]
    assert len(fmts) == int(rows["le_8"])
    assert len([f for f in fmts if 1 + f[0] + f[1] == 7]) == int(rows["7_only"])
    # every one of them is a format the oracle accepts (in an fp32 container)
    for X, Y in fmts:
        max_exp = 255 if X == 8 else 130
        assert O.check_format(F32, X, Y, max_exp) == 0, (X, Y)


def test_e2m1_rounding_example(golden):
    for X, Y, max_exp, x, want in golden("e2m1_rounding_example.txt"):
        got = O.emulate(np.array([float(x), -float(x)], dtype=np.float32), int(X), int(Y), int(max_exp))
        assert got[0] == np.float32(want) and got[1] == -np.float32(want)
    # one step between every two powers of two inside the normal range
    xs = np.linspace(1.0, 2.0, 1001, dtype=np.float32)
    assert sorted(set(O.emulate(xs, 2, 1, 129).tolist())) == [1.0, 1.5, 2.0]


def test_exponent_window(golden):
    for X, max_exp, lo, hi in golden("exponent_window.txt"):
        X, max_exp, lo, hi = map(int, (X, max_exp, lo, hi))
        Y = 0
        # exponent code E of 2^(e-127), for every biased exponent e
        xs = np.array([math.ldexp(1.0, e - 127) for e in range(1, 255)], dtype=np.float32)
        E = O.to_codes(xs, X, Y, max_exp) >> Y
        for e, code in zip(range(1, 255), E):
            if e > hi:
                assert code == (1 << X) - 1  # saturated
            elif e >= lo:
                assert code == e - lo + 1
            elif e == lo - 1:
                pass  # half of the smallest normal: a tie, rounds to even
            else:
                assert code == 0, e
        assert hi - lo + 1 == (1 << X) - 1


def test_ocp_small_format_value_sets():
    # OCP microscaling element formats the paper cites (fp4 e2m1, fp6 e2m3 / e3m2)
    e2m1 = sorted({abs(O.code_value(2, 1, max_exp_for_bias(2, 1), c)) for c in range(16)})
    assert e2m1 == [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    assert max(O.code_value(2, 3, max_exp_for_bias(2, 1), c) for c in range(64)) == 7.5
    assert max(O.code_value(3, 2, max_exp_for_bias(3, 3), c) for c in range(64)) == 28.0


# --------------------------------------------------------- library conversions


def _finite_sample(limit, n=200_000, seed=11):
    g = torch.Generator().manual_seed(seed)
    # log-uniform magnitudes down to well under every format's quantum, plus exact ties
    mag = torch.exp2(torch.rand(n, generator=g) * 40.0 - 30.0)
    x = mag * (torch.randint(0, 2, (n,), generator=g).float() * 2 - 1)
    x = torch.cat([x, torch.linspace(-limit, limit, 20001), torch.tensor([0.0, -0.0, limit, -limit])])
    return x[x.abs() <= limit].contiguous()


@pytest.mark.parametrize(
    "tdtype,X,Y,bias,limit",
    [
        (torch.float8_e4m3fn, 4, 3, 7, 448.0),
        (torch.float8_e5m2, 5, 2, 15, 57344.0),
        (torch.float16, 5, 10, 15, 65504.0),
    ],
)
def test_matches_library_float_formats(tdtype, X, Y, bias, limit):
    x = _finite_sample(limit)
    max_exp = max_exp_for_bias(X, bias)
    lib = x.to(tdtype)
    lib_bits = lib.view(torch.uint8 if lib.element_size() == 1 else torch.int16).numpy()
    lib_bits = lib_bits.view(np.uint8 if lib.element_size() == 1 else np.uint16).astype(np.uint32)
    codes = O.to_codes(x.numpy(), X, Y, max_exp)
    assert np.array_equal(codes, lib_bits)
    emu = O.emulate(x.numpy(), X, Y, max_exp)
    assert np.array_equal(emu.view(np.uint32), lib.float().numpy().view(np.uint32))
    # decode of the library's own bit patterns
    dec = O.from_codes(lib_bits, F32, X, Y, max_exp)
    assert np.array_equal(dec.view(np.uint32), lib.float().numpy().view(np.uint32))


def test_matches_fnuz_bias():
    # float8_e4m3fnuz has bias 8: same codes and values wherever it has a code (no -0 there)
    x = _finite_sample(240.0)
    max_exp = max_exp_for_bias(4, 8)
    lib = x.to(torch.float8_e4m3fnuz)
    emu = O.emulate(x.numpy(), 4, 3, max_exp)
    want = lib.float().numpy()
    assert np.array_equal(np.abs(emu), np.abs(want))
    nz = want != 0
    assert np.array_equal(emu[nz], want[nz])
    codes = O.to_codes(x.numpy(), 4, 3, max_exp)
    assert np.array_equal(codes[nz], lib.view(torch.uint8).numpy().astype(np.uint32)[nz])


def test_e8m7_is_fp32_to_bf16_rtne():
    # Section 2 "Rounding": the rule generalises the float32 -> bfloat16 RTNE conversion
    x = synth.f32_edge_sweep()
    x = x[torch.isfinite(x)]
    bf = x.to(torch.bfloat16)
    keep = torch.isfinite(bf)  # where the library conversion does not overflow to Inf
    x, bf = x[keep].contiguous(), bf[keep].contiguous()
    codes = O.to_codes(x.numpy(), 8, 7, 255)
    assert np.array_equal(codes, bf.view(torch.int16).numpy().view(np.uint16).astype(np.uint32))
    emu = O.emulate(x.numpy(), 8, 7, 255)
    assert np.array_equal(emu.view(np.uint32), bf.float().numpy().view(np.uint32))
    # values that would overflow to Inf in the library saturate at the largest finite bf16 here
    big = np.array([3.4e38, -3.4e38], dtype=np.float32)
    assert np.array_equal(O.to_codes(big, 8, 7, 255), np.array([0x7F7F, 0xFF7F], dtype=np.uint32))


def test_e8m0_ties_match_library_power_of_two_rounding():
    # with no mantissa bits a tie (1.5 * 2^e) goes up to the next power of two, as the
    # library's e8m0 conversion does
    e = torch.arange(-100, 100, dtype=torch.float32)
    x = torch.cat([torch.exp2(e) * m for m in (1.0, 1.25, 1.5, 1.75, 1.4999999, 1.5000001)]).contiguous()
    lib = x.to(torch.float8_e8m0fnu)
    emu = O.emulate(x.numpy(), 8, 0, 255)
    assert np.array_equal(emu, lib.float().numpy())
    assert np.array_equal(O.to_codes(x.numpy(), 8, 0, 255), lib.view(torch.uint8).numpy().astype(np.uint32))


def test_identity_formats():
    bf = synth.bits_numpy(synth.all_bf16_patterns())
    assert np.array_equal(O.emulate(bf, 8, 7, 255), bf)  # e8m7 in a bf16 container
    xs = synth.bits_numpy(synth.f32_edge_sweep())
    assert np.array_equal(O.emulate(xs, 8, 23, 255).view(np.uint32), xs.view(np.uint32))


# -------------------------------------------------------------- brute force


FORMATS_3_TO_9 = [(X, W - 1 - X) for W in range(3, 10) for X in range(0, min(W, 9))]


def _max_exps(X):
    if X == 8:
        return [255]
    if X == 0:
        return [1, 120, 253]
    return sorted({(1 << X) - 1, max(120, (1 << X) - 1), 254})


@pytest.mark.parametrize("X,Y", FORMATS_3_TO_9)
def test_nearest_value_bruteforce_all_bf16(X, Y):
    if Y > (8 if X == 0 else 7):
        pytest.skip("does not fit a bf16 container")
    bits = synth.bits_numpy(synth.all_bf16_patterns())
    f = (bits.astype(np.uint32) << 16).view(np.float32)
    finite = np.isfinite(f)
    a = np.abs(f[finite]).astype(np.float64)
    for max_exp in _max_exps(X):
        vals = textbook_values(X, Y, max_exp)
        want = brute_force_codes(a, vals) | ((bits[finite] >> 15).astype(np.uint32) << (X + Y))
        got = O.to_codes(bits, X, Y, max_exp)
        assert np.array_equal(got[finite], want), (X, Y, max_exp)
        # non-finite input: sign + largest code
        nf = ~finite
        assert np.array_equal(got[nf] & ((1 << (X + Y)) - 1), np.full(nf.sum(), len(vals) - 1, dtype=np.uint32))
        assert np.array_equal(got[nf] >> (X + Y), (bits[nf] >> 15).astype(np.uint32))


@pytest.mark.parametrize("X,Y", [(3, 3), (4, 2), (2, 3), (5, 0), (0, 6), (1, 5), (8, 0), (8, 7), (4, 11), (2, 13), (0, 15),
                                 (4, 14), (8, 10), (2, 19), (5, 16), (1, 21)])  # the last five: packed widths above 16
def test_nearest_value_bruteforce_fp32_sweep(X, Y):
    x = synth.f32_edge_sweep()
    xs = x.numpy()
    finite = np.isfinite(xs)
    a = np.abs(xs[finite]).astype(np.float64)
    sign = (xs.view(np.uint32)[finite] >> 31).astype(np.uint32)
    for max_exp in _max_exps(X):
        vals = textbook_values(X, Y, max_exp)
        want = brute_force_codes(a, vals) | (sign << (X + Y))
        got = O.to_codes(xs, X, Y, max_exp)[finite]
        assert np.array_equal(got, want), (X, Y, max_exp)


@pytest.mark.parametrize("X,Y", FORMATS_3_TO_9)
def test_every_code_point(X, Y):
    """All code points of every format at widths 3..9: decode is the textbook value,
    strictly monotone in the magnitude code, +-0 distinct, and encode(decode(c)) == c."""
    W = 1 + X + Y
    for max_exp in _max_exps(X):
        vals = textbook_values(X, Y, max_exp)
        codes = np.arange(1 << W, dtype=np.uint32)
        dec = O.from_codes(codes, F32, X, Y, max_exp)
        mag = codes & ((1 << (X + Y)) - 1)
        top = len(vals) - 1
        want = vals[np.minimum(mag, top)] * np.where(codes >> (X + Y), -1.0, 1.0)
        assert np.array_equal(dec.astype(np.float64), want)
        assert np.array_equal(np.signbit(dec), (codes >> (X + Y)).astype(bool))
        assert np.all(np.diff(vals) > 0)
        back = O.to_codes(dec, X, Y, max_exp)
        assert np.array_equal(back, np.where(mag > top, (codes & ~np.uint32((1 << (X + Y)) - 1)) | top, codes))
        if Y <= (8 if X == 0 else 7):  # also through a bf16 container
            dec16 = O.from_codes(codes, BF16, X, Y, max_exp)
            assert np.array_equal((dec16.astype(np.uint32) << 16), dec.view(np.uint32))


@pytest.mark.parametrize("X,Y", [(8, 10), (5, 11), (4, 14), (7, 16), (3, 20), (8, 22), (6, 23), (0, 23), (1, 23)])
def test_sampled_code_points_of_wide_formats(X, Y):
    """Formats wider than 16 bits (fp32 container only): decode is the textbook formula on sampled codes,
    encode(decode(c)) == c, and codes survive the packed form."""
    W = 1 + X + Y
    rng = np.random.default_rng(W)
    mags = np.unique(np.concatenate([rng.integers(0, 1 << (X + Y), 20000), np.arange(0, 300),
                                     (1 << (X + Y)) - 1 - np.arange(0, 300)])).astype(np.uint32)
    codes = np.concatenate([mags, mags | np.uint32(1 << (X + Y))])
    for max_exp in _max_exps(X):
        b = (1 << X) - 1 + 127 - max_exp
        E, M = (mags >> Y).astype(np.int64), (mags & ((1 << Y) - 1)).astype(np.int64)
        vals = np.where(E == 0, np.ldexp(M.astype(np.float64), 1 - b - Y),
                        np.ldexp(((1 << Y) + M).astype(np.float64), (E - b - Y).astype(np.int64)))
        if X == 8:
            vals = np.minimum(vals, np.ldexp(2.0 - 2.0 ** -Y, 127))
        dec = O.from_codes(codes, F32, X, Y, max_exp)
        assert np.array_equal(dec.astype(np.float64), np.concatenate([vals, -vals]))
        back = O.to_codes(dec, X, Y, max_exp)
        keep = np.concatenate([E, E]) < 255 if X == 8 else np.ones(codes.size, dtype=bool)
        assert np.array_equal(back[keep], codes[keep])
        if W <= 31:
            assert np.array_equal(O.unpack(O.pack(codes, W), codes.size, W), codes)


def test_sum_of_code_points():
    assert sum(W * (1 << W) for W in range(3, 10)) == 8184
    assert len(FORMATS_3_TO_9) == 42


# ---------------------------------------------------------------- emulation


def test_emulate_properties():
    x = synth.f32_edge_sweep()
    xs = x.numpy()
    nonfinite = ~np.isfinite(xs)
    for X, Y, max_exp in [(3, 3, 129), (2, 1, 127), (4, 3, 135), (0, 4, 126), (5, 2, 254), (8, 3, 255), (3, 23, 140)]:
        e = O.emulate(xs, X, Y, max_exp)
        # NaN / Inf bit-identical (Section 2.1)
        assert np.array_equal(e.view(np.uint32)[nonfinite], xs.view(np.uint32)[nonfinite])
        # idempotent, sign kept (also for values flushed to zero)
        assert np.array_equal(O.emulate(e, X, Y, max_exp).view(np.uint32), e.view(np.uint32))
        assert np.array_equal(np.signbit(e), np.signbit(xs))
        if 1 + X + Y <= 31:
            fin = ~nonfinite
            d = O.from_codes(O.to_codes(xs, X, Y, max_exp), F32, X, Y, max_exp)
            assert np.array_equal(d.view(np.uint32)[fin], e.view(np.uint32)[fin])


def test_format_validation():
    assert O.check_format(BF16, 3, 3, 130) == 0
    assert O.check_format(BF16, 0, 8, 130) == 0  # X = 0 needs only Y significant bits
    assert O.check_format(BF16, 1, 8, 130) != 0
    assert O.check_format(BF16, 0, 9, 130) != 0
    assert O.check_format(F32, 9, 0, 130) != 0
    assert O.check_format(F32, 4, 12, 130) == 0  # W = 17 = 16 + 1 packs
    assert O.check_format(F32, 8, 22, 255) == 0  # W = 31 = 16 + 8 + 4 + 2 + 1
    assert O.check_format(F32, 8, 23, 255) == 0  # W = 32: one 32-bit segment, the widest packed form
    assert O.check_format(F32, 8, 23, 255, packed=False) == 0
    assert O.check_format(F32, 8, 3, 254) != 0 and O.check_format(F32, 8, 3, 255) == 0
    assert O.check_format(F32, 3, 3, 6) != 0 and O.check_format(F32, 3, 3, 7) == 0
    assert O.check_format(F32, 3, 3, 255) != 0
    assert O.check_format(F32, 0, 3, 254) != 0 and O.check_format(F32, 0, 3, 253) == 0
    assert O.check_format(F32, 0, 3, 0) == 0
    # e0m8 in bf16: the quantum 2^(max_exp - 134) must be a bf16 value
    assert O.check_format(BF16, 0, 8, 0) != 0 and O.check_format(BF16, 0, 8, 1) == 0


def test_histogram_and_max_exp_choice():
    x, _ = synth.cfg1(n=4096)
    xs = x.numpy()
    h = O.exponent_histogram(xs)
    want = np.bincount((xs.view(np.uint32) >> 23) & 0xFF, minlength=256)
    assert np.array_equal(h, want.astype(np.uint64))
    assert h.sum() == xs.size
    bf = synth.bits_numpy(synth.gaussian_bf16(5000))
    assert np.array_equal(O.exponent_histogram(bf), np.bincount((bf >> 7) & 0xFF, minlength=256).astype(np.uint64))
    # coverage rule: smallest exponent with at least that share of finite elements at or below it
    hist = np.zeros(256, dtype=np.uint64)
    hist[100], hist[120], hist[130], hist[255] = 10, 80, 10, 1000
    assert O.max_exp_from_histogram(hist, 0.05) == 100
    assert O.max_exp_from_histogram(hist, 0.5) == 120
    assert O.max_exp_from_histogram(hist, 0.9) == 120
    assert O.max_exp_from_histogram(hist, 0.91) == 130
    assert O.max_exp_from_histogram(hist, 1.0) == 130
    assert O.max_exp_from_histogram(np.zeros(256, dtype=np.uint64), 0.5) == -1
