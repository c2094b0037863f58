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
