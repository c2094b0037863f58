"""Pins of the CPU oracle's fp16 container (Section 2.1: fp16 emulates X <= 5,
Y <= 10): its half <-> float conversions against the library's, its results
against the fp32 container's on the same values, and its validity rules."""
import numpy as np
import pytest
import torch

from oracle import exmy_oracle as O
from paper_2405_13938_amd import synth

F32, BF16, F16 = O.F32, O.BF16, O.F16


def f16_range(X, Y):
    """max_exp values for which every value of eXmY is an fp16 value."""
    lo = (101 + Y + (1 << X)) if X >= 1 else (102 + Y)
    return max(lo, (1 << X) - 1 if X >= 1 else 0), 142


def test_container_limits_of_the_paper():
    # Section 2.1: fp16 holds X <= 5 and Y <= 10 (bf16: X <= 8, Y <= 7; fp32: X <= 8, Y <= 23)
    for X in range(0, 9):
        for Y in range(0, 13):
            lo, hi = f16_range(X, Y)
            fits = X <= 5 and Y <= (10 if X >= 1 else 11)
            any_ok = any(O.check_format(F16, X, Y, me, False) == 0 for me in range(0, 256))
            assert any_ok == (fits and lo <= hi), (X, Y)
            if fits and lo <= hi:
                assert O.check_format(F16, X, Y, lo, False) == 0 and O.check_format(F16, X, Y, hi, False) == 0
                assert O.check_format(F16, X, Y, hi + 1, False) != 0
                if lo > 0:
                    assert O.check_format(F16, X, Y, lo - 1, False) != 0
    assert O.check_format(F16, 5, 9, 142) == 0      # 31 binades do not fit next to fp16's 30 ...
    assert O.check_format(F16, 5, 10, 142) != 0     # ... with 10 mantissa bits the quantum 2^-25 is no half
    assert O.check_format(F16, 4, 10, 130) == 0


@pytest.mark.parametrize("X,Y", [(3, 3), (2, 1), (4, 3), (5, 2), (1, 7), (0, 4), (4, 10), (5, 9), (0, 11), (1, 10)])
def test_every_f16_pattern_matches_the_fp32_container(X, Y):
    x = synth.all_f16_patterns()
    xn = synth.bits_numpy(x)
    x32 = x.float().numpy()  # the library's exact half -> float conversion
    fin = np.isfinite(x32)
    lo, hi = f16_range(X, Y)
    for me in sorted({lo, (lo + hi) // 2, hi}):
        # codes: same as from the fp32 container (pins the oracle's half -> float reading)
        c16 = O.to_codes(xn, X, Y, me)
        c32 = O.to_codes(x32, X, Y, me)
        assert np.array_equal(c16, c32), (X, Y, me)
        # values: the fp32 container's, converted by the library (exactly: they are fp16 values)
        d32 = O.from_codes(c32, F32, X, Y, me)
        d16 = O.from_codes(c16, F16, X, Y, me)
        assert np.array_equal(torch.from_numpy(d32).half().float().numpy(), d32)
        assert np.array_equal(d16.view(np.uint16), torch.from_numpy(d32).half().numpy().view(np.uint16))
        # emulate: decode(encode) on finite input, Inf / NaN bit-identical
        e = O.emulate(xn, X, Y, me)
        assert np.array_equal(e.view(np.uint16)[fin], d16.view(np.uint16)[fin])
        assert np.array_equal(e.view(np.uint16)[~fin], xn.view(np.uint16)[~fin])
        # packed form
        p = O.encode(xn, X, Y, me)
        assert np.array_equal(p, O.pack(c16, 1 + X + Y))
        assert np.array_equal(O.decode(p, F16, xn.size, X, Y, me).view(np.uint16), d16.view(np.uint16))


def test_e4m3_and_e5m2_grids_inside_fp16():
    # e4m3 at the OCP bias 7: every finite float8_e4m3 value is an fp16 value.  e5m2's 31 finite binades
    # need max_exp = 142 in fp16 (bias 16); its grid equals float8_e5m2's over that type's normal range.
    for tdtype, X, Y, me, lo, hi in ((torch.float8_e4m3fn, 4, 3, 135, 0.0, 240.0),
                                     (torch.float8_e5m2, 5, 2, 142, 2.0 ** -14, 57344.0)):
        assert O.check_format(F16, X, Y, me) == 0
        g = torch.Generator().manual_seed(X)
        x = (torch.randn(200000, generator=g) * torch.exp2(torch.randint(-12, 14, (200000,), generator=g).float())).half()
        a = x.float().abs()
        x = x[(a <= hi) & (a >= lo)]
        want = x.to(tdtype).half()  # library rounding to the float8 grid (in range: no NaN codes involved)
        got = O.emulate(synth.bits_numpy(x), X, Y, me)
        assert np.array_equal(got.view(np.uint16), want.numpy().view(np.uint16))
    assert O.check_format(F16, 5, 2, 143) != 0  # bias 15 would put 1.75 * 2^16 in the top binade


def test_f16_histogram_bins_by_value_exponent():
    x = synth.all_f16_patterns()
    h = O.exponent_histogram(synth.bits_numpy(x))
    v = x.float()
    want = torch.bincount(((v.view(torch.int32) >> 23) & 0xFF).long(), minlength=256).numpy()
    assert np.array_equal(h, want.astype(np.uint64))
    assert h[0] == 2 and h[255] == 2 * 1024 and h.sum() == 65536


def test_half_rounding_is_the_library_conversion():
    g = torch.Generator().manual_seed(2)
    bits = torch.randint(0, 2 ** 32, (200000,), generator=g, dtype=torch.int64)
    extra = [0x477FE000, 0x477FEFFF, 0x477FF000, 0x47800000, 0x33000000, 0x33000001, 0x32FFFFFF, 0x38800000, 0x387FC000,
             0x387FE000, 0x3F801000, 0x3F803000, 0x3F802FFF, 0x0, 0x80000000, 0x00000001]
    bits = torch.cat([bits, torch.tensor(extra, dtype=torch.int64)])
    bits = torch.where(bits >= 2 ** 31, bits - 2 ** 32, bits).to(torch.int32)
    x = bits.view(torch.float32)
    x = x[torch.isfinite(x)]
    want = x.half().float().view(torch.int32)
    got = torch.tensor([O.round_to_half_float_bits(v) for v in x.tolist()], dtype=torch.int64)
    got = torch.where(got >= 2 ** 31, got - 2 ** 32, got).to(torch.int32)
    assert torch.equal(got, want)


def block_range(X, Y):
    lo, hi = f16_range(X, Y)
    return max(lo, 1 if X == 0 else (1 << X)), hi


@pytest.mark.parametrize("X,Y", [(3, 3), (2, 1), (4, 3), (5, 2), (1, 7), (0, 4), (4, 10), (0, 11)])
def test_block_forms_match_the_fp32_container_on_the_same_values(X, Y):
    # with metadata inside the fp16 range, codes and values are those of the fp32 container (pinned
    # elsewhere); metadata outside is read as the nearest value of the (narrower) fp16 range
    x = synth.shuffled(synth.all_f16_patterns(), 40 + X)
    x = x[: (x.numel() // 64) * 64]
    xn = synth.bits_numpy(x)
    x32 = x.float().numpy()
    fin = np.isfinite(x32)
    lo, hi = block_range(X, Y)
    for block in (32, 64):
        nb = x.numel() // block
        before = O.block_max_exp(xn, block, X)
        assert np.array_equal(before, np.minimum(O.block_max_exp(x32, block, X), 142))
        after = O.block_max_exp_after_rounding(xn, block, X, Y)
        assert np.array_equal(after, np.clip(O.block_max_exp_after_rounding(x32, block, X, Y), lo, hi))
        for meta in (before, after, np.random.default_rng(X + Y).integers(0, 256, nb).astype(np.uint8)):
            eff = np.clip(meta, lo, hi).astype(np.uint8)
            p16 = O.encode_blocks(xn, block, X, Y, meta)
            assert np.array_equal(p16, O.encode_blocks(x32, block, X, Y, eff))
            d16 = O.decode_blocks(p16, F16, x.numel(), block, X, Y, meta)
            d32 = O.decode_blocks(p16, F32, x.numel(), block, X, Y, eff)
            assert np.array_equal(d16.astype(np.float32), d32)
            e16 = O.emulate_blocks(xn, block, X, Y, meta)
            assert np.array_equal(e16.view(np.uint16)[fin], d16.view(np.uint16)[fin])
            assert np.array_equal(e16.view(np.uint16)[~fin], xn.view(np.uint16)[~fin])
    # packing along rows with per-row metadata: the flat block codec's codes, permuted
    rows, cols = 40, 64
    m = O.block_max_exp(xn[: rows * cols], cols, X)
    pr = O.encode_rows(xn[: rows * cols], rows, cols, X, Y, max_exp_rows=m)
    assert np.array_equal(pr, O.encode_rows(x32[: rows * cols], rows, cols, X, Y, max_exp_rows=np.clip(m, lo, hi).astype(np.uint8)))
    dr = O.decode_rows(pr, F16, rows, cols, X, Y, max_exp_rows=m)
    assert np.array_equal(dr.astype(np.float32), O.decode_rows(pr, F32, rows, cols, X, Y, max_exp_rows=np.clip(m, lo, hi).astype(np.uint8)))


@pytest.mark.parametrize("X,Y", [(3, 3), (2, 1), (4, 3), (1, 7), (0, 4), (4, 10)])
def test_float_scaling_in_fp16_is_the_fp32_result_rounded_by_the_library(X, Y):
    g = torch.Generator().manual_seed(X * 7 + Y)
    n, block = 1 << 14, 32
    x = (torch.randn(n, generator=g) * torch.exp2(torch.randint(-12, 10, (n,), generator=g).float())).half()
    x[::101] = float("inf")
    x[5::103] = float("nan")
    x[64:96] = 65504.0
    xn = synth.bits_numpy(x)
    x32 = x.float().numpy()
    s = O.block_scale(xn, block, X, Y)
    assert np.array_equal(s.view(np.uint32), O.block_scale(x32, block, X, Y).view(np.uint32))
    p = O.encode_scaled(xn, block, X, Y, s)
    assert np.array_equal(p, O.encode_scaled(x32, block, X, Y, s))
    d32 = torch.from_numpy(O.decode_scaled(p, F32, n, block, X, Y, s))
    d16 = O.decode_scaled(p, F16, n, block, X, Y, s)
    assert np.array_equal(d16.view(np.uint16), d32.half().numpy().view(np.uint16))
    e16 = O.emulate_scaled(xn, block, X, Y, s)
    fin = np.isfinite(x32)
    assert np.array_equal(e16.view(np.uint16)[fin], d16.view(np.uint16)[fin])
    assert np.array_equal(e16.view(np.uint16)[~fin], xn.view(np.uint16)[~fin])
    # the block maximum is kept (Section 2.1), to an ulp of the container
    m = torch.where(torch.isfinite(x.float()), x.float().abs(), torch.zeros(())).reshape(-1, block).max(dim=1).values
    em = torch.where(torch.isfinite(torch.from_numpy(e16.astype(np.float32))), torch.from_numpy(e16.astype(np.float32)).abs(),
                     torch.zeros(())).reshape(-1, block).max(dim=1).values
    assert ((em - m).abs() <= m * 2.0 ** -10).all()


@pytest.mark.parametrize("Y,max_exp", [(3, 129), (7, 133), (8, 127), (10, 141), (4, 110)])
def test_twos_complement_in_fp16(Y, max_exp):
    x = synth.all_f16_patterns()
    xn = synth.bits_numpy(x)
    x32 = x.float().numpy()
    fin = np.isfinite(x32)
    c16 = O.to_codes_int(xn, Y, max_exp)
    assert np.array_equal(c16, O.to_codes_int(x32, Y, max_exp))
    d16 = O.from_codes_int(c16, F16, Y, max_exp)
    assert np.array_equal(d16.astype(np.float32), O.from_codes_int(c16, F32, Y, max_exp))
    e16 = O.emulate_int(xn, Y, max_exp)
    assert np.array_equal(e16.view(np.uint16)[fin], d16.view(np.uint16)[fin])
    assert np.array_equal(e16.view(np.uint16)[~fin], xn.view(np.uint16)[~fin])
    assert np.array_equal(O.decode_int(O.encode_int(xn, Y, max_exp), F16, xn.size, Y, max_exp).view(np.uint16), d16.view(np.uint16))


def test_fp16_limits_of_the_other_forms():
    x = np.zeros(64, dtype=np.float16)
    m = np.full(8, 130, dtype=np.uint8)
    with pytest.raises(Exception):
        O.encode_blocks(x, 8, 5, 10, m)   # no max_exp keeps e5m10 inside fp16
    with pytest.raises(Exception):
        O.encode_blocks(x, 8, 6, 2, m)    # X <= 5
    with pytest.raises(Exception):
        O.block_scale(x, 8, 5, 2)         # max_exp = 127 is below e5m2's fp16 range
    O.block_scale(x, 8, 4, 10)
    with pytest.raises(Exception):
        O.encode_int(x, 7, 142)           # -2^16 is not a half
    O.encode_int(x, 7, 141)
    with pytest.raises(Exception):
        O.encode_int(x, 7, 108)           # quantum 2^-25
    O.encode_int(x, 7, 109)
