"""Reserved NaN / Inf code points on the GPU, against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

import paper_2405_13938_amd as exmy
from oracle import exmy_oracle as O
from paper_2405_13938_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ODT = {torch.float32: O.F32, torch.bfloat16: O.BF16, torch.float16: O.F16}
IEEE, NAN_ONLY = exmy.binding.SPECIALS_IEEE, exmy.binding.SPECIALS_NAN_ONLY


def ubits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else (a.view(np.uint16) if a.dtype == np.float16 else a)


def tbits(t):
    return ubits(synth.bits_numpy(t))


def check(x, X, Y, me, specials, codes=None):
    n = x.numel()
    host = synth.bits_numpy(x)
    label = (X, Y, me, specials, n, x.dtype)
    if 1 + X + Y <= 16:
        want = O.encode_specials(host, X, Y, me, specials)
        got = exmy.encode_specials(x, X, Y, me, specials)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), want), ("encode", label)
        # decode every kind of code, not only those that encode produces
        blob = want if codes is None else O.pack(codes, 1 + X + Y)
        m = n if codes is None else codes.size
        back = exmy.decode_specials(torch.from_numpy(blob).to(DEV), x.dtype, m, X, Y, me, specials)
        torch.cuda.synchronize()
        assert np.array_equal(tbits(back), ubits(O.decode_specials(blob, ODT[x.dtype], m, X, Y, me, specials))), ("decode", label)
    emu = exmy.emulate_specials(x.clone(), X, Y, me, specials)
    torch.cuda.synchronize()
    assert np.array_equal(tbits(emu), ubits(O.emulate_specials(host, X, Y, me, specials))), ("emulate", label)


def formats(dtype, W):
    P = {torch.float32: 23, torch.bfloat16: 7, torch.float16: 10}[dtype]
    xmax = 5 if dtype == torch.float16 else 8
    return [(X, W - 1 - X) for X in range(0, min(W - 1, xmax) + 1) if W - 1 - X <= (P if X >= 1 else P + 1)]


@pytest.mark.parametrize("W", range(2, 17))
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32, torch.float16])
def test_every_width(W, dtype):
    if dtype == torch.float16:
        x = synth.shuffled(synth.all_f16_patterns(), W).to(DEV)
    else:
        x = synth.shuffled(synth.all_bf16_patterns(), W).to(dtype).to(DEV)
        if dtype == torch.float32:
            x = torch.cat([x, (x.view(torch.int32) + 0x4000).view(torch.float32), x * 1.0009765625]).contiguous()
    x = x[: x.numel() - 3]  # ragged
    rng = np.random.default_rng(W)
    codes = np.concatenate([np.arange(min(1 << W, 70000)), rng.integers(0, 1 << W, 5003)]).astype(np.uint32)
    for X, Y in formats(dtype, W):
        for specials in (IEEE, NAN_ONLY):
            if (specials == IEEE and X < 1) or (specials == NAN_ONLY and (X == 8 or X + Y < 1)):
                continue
            for me in ([255] if X == 8 else [127, 131, 142, (1 << X) - 1 if X else 1, 254 if X else 253]):
                if O.check_format(ODT[dtype], X, Y, me) != 0:
                    continue
                check(x, X, Y, me, specials, codes)


def test_the_library_float_types():
    x = synth.cfg1(n=(1 << 20) + 5, seed=3)[0].to(DEV) * 100.0
    n = x.numel()
    for X, Y, me, specials, ldt in ((5, 2, 143, IEEE, torch.float8_e5m2), (4, 3, 135, NAN_ONLY, torch.float8_e4m3fn)):
        check(x, X, Y, me, specials)
        # one plane of 8 bits: the packed form is the array of codes, comparable with the library's conversion
        got = exmy.encode_specials(x, X, Y, me, specials)[:n]
        top = {torch.float8_e5m2: 57344.0, torch.float8_e4m3fn: 448.0}[ldt]
        lib = x.to(ldt)
        fits = (lib.float().abs() <= top) | torch.isnan(x) | (torch.isinf(x) if specials == IEEE else torch.zeros_like(x, dtype=torch.bool))
        assert torch.equal(got[fits], lib.view(torch.uint8)[fits])
    xb = x.bfloat16()
    assert torch.equal(exmy.encode_specials(xb, 8, 7, 255, IEEE)[: 2 * n].view(torch.int16)[~torch.isnan(xb)], xb.view(torch.int16)[~torch.isnan(xb)])


@pytest.mark.parametrize("n", [0, 1, 7, 8, 9, 2049, 100003])
def test_lengths(n):
    for dtype in (torch.bfloat16, torch.float32):
        x = synth.cfg1(n=max(n, 16), seed=n)[0][:n].to(dtype).contiguous().to(DEV)
        for X, Y, specials in ((3, 3, IEEE), (2, 1, NAN_ONLY), (4, 2, IEEE)):
            check(x, X, Y, 130, specials)


def test_wide_emulate_and_errors():
    x = synth.cfg1(n=40003, seed=9)[0].to(DEV)
    for X, Y, me in ((5, 18, 140), (8, 23, 255), (3, 22, 130)):
        check(x, X, Y, me, IEEE)
    check(x, 0, 24, 100, NAN_ONLY)
    with pytest.raises(exmy.ExmyError):
        exmy.encode_specials(x, 0, 3, 130, IEEE)
    with pytest.raises(exmy.ExmyError):
        exmy.encode_specials(x, 3, 3, 130, 0)
    with pytest.raises(exmy.ExmyError):
        exmy.encode_specials(x, 4, 12, 130, IEEE)
