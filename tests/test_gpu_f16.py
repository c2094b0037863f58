"""Parity of the fp16 container (through the C ABI) with the CPU oracle, tolerance 0."""
import numpy as np
import pytest
import torch

import paper_2405_13938_amd as exmy
from oracle import exmy_oracle as O
from paper_2405_13938_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
THREADS = min(O.default_threads(), 16)


def hbits(t):
    return synth.bits_numpy(t).view(np.uint16)


def f16_formats(W):
    return [(X, W - 1 - X) for X in range(0, min(W - 1, 5) + 1) if W - 1 - X <= (10 if X >= 1 else 11)]


def f16_max_exps(X, Y):
    lo = (101 + Y + (1 << X)) if X >= 1 else (102 + Y)
    if lo > 142:
        return []
    return sorted({lo, (lo + 142) // 2, 142})


def check_all(x_dev, X, Y, max_exp, host):
    n = x_dev.numel()
    label = "fp16 e%dm%d max_exp=%d n=%d" % (X, Y, max_exp, n)
    want_packed = O.encode(host, X, Y, max_exp, threads=THREADS)
    got = exmy.encode(x_dev, X, Y, max_exp)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), want_packed), "encode " + label
    dec = exmy.decode(torch.from_numpy(want_packed).to(DEV), torch.float16, n, X, Y, max_exp)
    torch.cuda.synchronize()
    want = O.decode(want_packed, O.F16, n, X, Y, max_exp, threads=THREADS)
    assert np.array_equal(hbits(dec), want.view(np.uint16)), "decode " + label
    emu = exmy.emulate(x_dev.clone(), X, Y, max_exp)
    torch.cuda.synchronize()
    assert np.array_equal(hbits(emu), O.emulate(host, X, Y, max_exp, threads=THREADS).view(np.uint16)), "emulate " + label


@pytest.mark.parametrize("W", range(1, 17))
def test_every_f16_pattern_every_format(W):
    x = torch.cat([synth.all_f16_patterns(), synth.all_f16_patterns()[31000:31005]]).to(DEV)
    host = synth.bits_numpy(x)
    for X, Y in f16_formats(W):
        for me in f16_max_exps(X, Y):
            check_all(x, X, Y, me, host)


def test_every_code_point_decodes():
    for W in range(1, 17):
        codes = np.arange(1 << W, dtype=np.uint32)
        codes = np.concatenate([codes, codes[: (3 if W > 2 else 1)]])
        pd = torch.from_numpy(O.pack(codes, W)).to(DEV)
        for X, Y in f16_formats(W):
            for me in f16_max_exps(X, Y):
                got = exmy.decode(pd, torch.float16, codes.size, X, Y, me)
                torch.cuda.synchronize()
                assert np.array_equal(hbits(got), O.from_codes(codes, O.F16, X, Y, me).view(np.uint16)), (W, X, Y, me)


def test_histogram_batch_and_ragged_lengths():
    g = torch.Generator().manual_seed(6)
    xs = []
    for n in (1, 7, 8, 9, 1023, 4096 + 5, 33 * 1024 + 1, (1 << 20) + 3):
        x = (torch.randn(n, generator=g) * torch.exp2(torch.randint(-14, 6, (n,), generator=g).float())).half()
        x[::97] = float("inf")
        x[::89] = float("nan")
        xs.append(x.to(DEV))
    outs = exmy.encode_batch(xs, 3, 3, [130] * len(xs))
    torch.cuda.synchronize()
    for x, o in zip(xs, outs):
        host = synth.bits_numpy(x)
        assert np.array_equal(o.cpu().numpy(), O.encode(host, 3, 3, 130))
        h = exmy.exponent_histogram(x)
        p, h2 = exmy.encode_with_histogram(x, 3, 3, 130)
        torch.cuda.synchronize()
        want_h = O.exponent_histogram(host)
        assert np.array_equal(h.cpu().numpy().astype(np.uint64), want_h)
        assert np.array_equal(h2.cpu().numpy().astype(np.uint64), want_h)
        assert torch.equal(p, o)
        check_all(x, 4, 3, 135, host)
    decs = exmy.decode_batch(outs, torch.float16, [x.numel() for x in xs], 3, 3, [130] * len(xs))
    torch.cuda.synchronize()
    for x, o, d in zip(xs, outs, decs):
        assert np.array_equal(hbits(d), O.decode(o.cpu().numpy(), O.F16, x.numel(), 3, 3, 130).view(np.uint16))
