"""Pins of the CPU oracle's reserved NaN / Inf code points (Section 5 of the paper leaves their encoding
open; the oracle offers the two conventions of the float types in use).  Each convention is pinned against
the library's own float types that follow it: float8_e5m2, float16 and bfloat16 (IEEE style), float8_e4m3fn
(NaN only), over every bf16 / fp16 bit pattern and fp32 tie sweeps.  Saturation of finite overflow is the
paper's policy (Section 2.1) and differs from the library's overflow to Inf / NaN: it is checked apart."""
import numpy as np
import pytest
import torch

from oracle import exmy_oracle as O
from paper_2405_13938_amd import synth

IEEE, NAN_ONLY = O.IEEE, O.NAN_ONLY


def fp32_sweep(seed=0):
    """Every bf16 pattern as fp32, plus neighbours and exact ties of 2- and 3-bit mantissa grids."""
    base = synth.all_bf16_patterns().float()
    g = torch.Generator().manual_seed(seed)
    jitter = base * (1 + (torch.rand(base.numel(), generator=g) - 0.5) * 2 ** -6)
    mid = (base.view(torch.int32) + 0x4000).view(torch.float32)  # halfway patterns between bf16 neighbours
    return torch.cat([base, jitter, mid])


CASES = [  # X, Y, max_exp, specials, library dtype, its integer view, largest finite value
    (5, 2, 143, IEEE, torch.float8_e5m2, torch.uint8, 57344.0),
    (4, 3, 135, NAN_ONLY, torch.float8_e4m3fn, torch.uint8, 448.0),
    (5, 10, 143, IEEE, torch.float16, torch.int16, 65504.0),
    (8, 7, 255, IEEE, torch.bfloat16, torch.int16, 3.3895313892515355e38),
]


@pytest.mark.parametrize("X,Y,max_exp,specials,ldt,view,top", CASES)
def test_codes_are_the_library_types_bit_patterns(X, Y, max_exp, specials, ldt, view, top):
    x = fp32_sweep(X + Y)
    if ldt == torch.float16:
        x = torch.cat([x, synth.all_f16_patterns().float()])
    n = x.numel() - x.numel() % 8
    x = x[:n]
    W = 1 + X + Y
    codes = O.unpack(O.encode_specials(x.numpy(), X, Y, max_exp, specials), n, W)
    lib = x.to(ldt).view(view).to(torch.int64).numpy() & ((1 << W) - 1)
    a = x.abs()
    # where the library does not overflow: finite values that round to at most the largest finite one, Inf with an
    # Inf code, NaN
    fits = x.to(ldt).float().abs() <= top
    if specials == IEEE:
        fits |= torch.isinf(x)
    fits = fits.numpy()
    assert np.array_equal(codes[fits], lib[fits].astype(np.uint32))
    # NaN: the all-ones magnitude code under the NaN's own sign (the 8-bit library types give the same pattern;
    # the 16-bit ones keep a payload, which the format does not promise)
    nan = torch.isnan(x).numpy()
    sign = (x.view(torch.int32).numpy()[nan] < 0).astype(np.uint32) << (W - 1)
    assert np.array_equal(codes[nan], ((1 << (W - 1)) - 1) | sign)
    if W == 8:
        assert np.array_equal(codes[nan], lib[nan].astype(np.uint32))
    fits |= nan
    # the rest overflowed in the library; here it saturates to the largest finite value under its sign
    over = ~fits
    assert over.any()
    top_code = int(torch.tensor([top]).to(ldt).view(view).to(torch.int64)[0]) & ((1 << W) - 1)
    sign = (x.view(torch.int32).numpy()[over] < 0).astype(np.uint32) << (W - 1)
    assert np.array_equal(codes[over], top_code | sign)
    assert (a[torch.from_numpy(over)] > top).all()


@pytest.mark.parametrize("X,Y,max_exp,specials,ldt,view,top", CASES)
def test_every_code_decodes_as_the_library_type(X, Y, max_exp, specials, ldt, view, top):
    W = 1 + X + Y
    codes = np.arange(1 << W, dtype=np.uint32)
    got = O.decode_specials(O.pack(codes, W), O.F32, codes.size, X, Y, max_exp, specials).view(np.uint32)
    lib = torch.from_numpy(codes.astype(np.int64)).to(torch.int16 if W == 16 else torch.uint8).view(ldt).float()
    want = lib.view(torch.int32).numpy().view(np.uint32)
    nan = np.isnan(lib.numpy())
    assert np.array_equal(got[~nan], want[~nan])
    # NaN codes: quiet NaN under the code's sign
    assert np.array_equal(got[nan], ((codes[nan] >> (W - 1)) << 31) | 0x7FC00000)
    assert nan.sum() == (2 if specials == NAN_ONLY else 2 * ((1 << Y) - 1))


def test_emulate_keeps_specials_and_saturates():
    x = fp32_sweep(3)
    for X, Y, max_exp, specials, ldt, view, top in CASES[:3]:
        emu = torch.from_numpy(O.emulate_specials(x.numpy(), X, Y, max_exp, specials))
        lib = x.to(ldt).float()
        fin = torch.isfinite(x)
        inside = fin & (lib.abs() <= top)
        assert torch.equal(emu[inside].view(torch.int32), lib[inside].view(torch.int32))
        over = fin & ~inside
        assert torch.equal(emu[over], torch.sign(x[over]) * top)
        assert torch.equal(emu[~fin].view(torch.int32), x[~fin].view(torch.int32))  # bit-identical
        # emulate == decode(encode) on finite input
        n = x.numel() - x.numel() % 8
        dec = O.decode_specials(O.encode_specials(x[:n].numpy(), X, Y, max_exp, specials), O.F32, n, X, Y, max_exp, specials)
        f = fin[:n].numpy()
        assert np.array_equal(dec.view(np.uint32)[f], emu[:n].numpy().view(np.uint32)[f])


def test_other_formats_lose_exactly_the_reserved_codes():
    """For any format the finite codes decode as in the plain format, and encode agrees with the plain format
    wherever the plain code is still finite."""
    x = synth.bits_numpy(synth.shuffled(synth.all_bf16_patterns(), 11))
    for X, Y, me in ((2, 1, 128), (3, 3, 130), (4, 2, 131), (1, 3, 127), (3, 0, 129)):
        W = 1 + X + Y
        plain = O.unpack(O.encode(x, X, Y, me), x.size, W)
        mag = plain & ((1 << (X + Y)) - 1)
        fin = ((x & 0x7F80) != 0x7F80)
        for specials, cfin in ((IEEE, (((1 << X) - 1) << Y) - 1), (NAN_ONLY, (1 << (X + Y)) - 2)):
            got = O.unpack(O.encode_specials(x, X, Y, me, specials), x.size, W)
            same = fin & (mag <= cfin)
            assert np.array_equal(got[same], plain[same])
            sat = fin & (mag > cfin)
            assert np.array_equal(got[sat] & ((1 << (X + Y)) - 1), np.full(sat.sum(), cfin))
            codes = np.arange(1 << W, dtype=np.uint32)
            d1 = O.decode_specials(O.pack(codes, W), O.BF16, codes.size, X, Y, me, specials)
            d0 = O.decode(O.pack(codes, W), O.BF16, codes.size, X, Y, me)
            keep = (codes & ((1 << (X + Y)) - 1)) <= cfin
            assert np.array_equal(d1[keep], d0[keep])


def test_specials_validation():
    x = np.zeros(8, dtype=np.float32)
    for bad in (lambda: O.encode_specials(x, 3, 3, 130, 0), lambda: O.encode_specials(x, 3, 3, 130, 3),
                lambda: O.encode_specials(x, 0, 3, 130, IEEE), lambda: O.encode_specials(x, 8, 7, 255, NAN_ONLY),
                lambda: O.encode_specials(x, 4, 12, 130, IEEE), lambda: O.encode_specials(x, 3, 3, 6, IEEE)):
        with pytest.raises(Exception):
            bad()
    assert O.encode_specials(x, 0, 3, 130, NAN_ONLY).size == 4
    assert O.emulate_specials(x, 4, 12, 130, IEEE).size == 8  # emulation has no width limit
