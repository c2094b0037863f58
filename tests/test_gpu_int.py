"""Parity of the two's complement entry points (through the C ABI) with the CPU
oracle, tolerance 0."""
import numpy as np
import pytest
import torch

import paper_2405_13938_amd as exmy
from oracle import exmy_oracle as O
from paper_2405_13938_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def ubits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else a


def tbits(t):
    return ubits(synth.bits_numpy(t))


def max_exps(Y, dtype):
    P = 23 if dtype == torch.float32 else 7
    lo = 1 if Y == P + 1 else 0
    return sorted({lo, 60, 126 + Y if 126 + Y <= 253 else 253, min(253, 230 + Y)})


def check_int(x_dev, Y, max_exp, host=None, packed=True):
    n = x_dev.numel()
    if host is None:
        host = synth.bits_numpy(x_dev)
    dt = O.F32 if x_dev.dtype == torch.float32 else O.BF16
    label = "int%d max_exp=%d n=%d %s" % (Y + 1, max_exp, n, x_dev.dtype)
    if packed:
        want = O.encode_int(host, Y, max_exp)
        got = exmy.encode_int(x_dev, Y, max_exp)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), want), "encode_int " + label
        dec = exmy.decode_int(torch.from_numpy(want).to(DEV), x_dev.dtype, n, Y, max_exp)
        torch.cuda.synchronize()
        assert np.array_equal(tbits(dec), ubits(O.decode_int(want, dt, n, Y, max_exp))), "decode_int " + label
    emu = exmy.emulate_int(x_dev.clone(), Y, max_exp)
    torch.cuda.synchronize()
    assert np.array_equal(tbits(emu), ubits(O.emulate_int(host, Y, max_exp))), "emulate_int " + label


@pytest.mark.parametrize("Y", range(1, 9))
def test_every_bf16_pattern(Y):
    x = torch.cat([synth.all_bf16_patterns(), synth.all_bf16_patterns()[777:782]]).to(DEV)
    host = synth.bits_numpy(x)
    for me in max_exps(Y, torch.bfloat16):
        check_int(x, Y, me, host)


@pytest.mark.parametrize("Y", range(1, 22))
def test_fp32_sweep(Y):
    x = synth.f32_edge_sweep(seed=Y)
    x = torch.cat([x, x[:3]]).to(DEV)
    host = synth.bits_numpy(x)
    for me in max_exps(Y, torch.float32):
        check_int(x, Y, me, host, packed=Y <= 15)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_every_code_point_decodes(dtype):
    for Y in range(1, 9 if dtype == torch.bfloat16 else 16):
        W = 1 + Y
        codes = np.arange(1 << W, dtype=np.uint32)
        codes = np.concatenate([codes, codes[:3]])
        pd = torch.from_numpy(O.pack(codes, W)).to(DEV)
        for me in max_exps(Y, dtype):
            got = exmy.decode_int(pd, dtype, codes.size, Y, me)
            torch.cuda.synchronize()
            want = O.from_codes_int(codes, O.F32 if dtype == torch.float32 else O.BF16, Y, me)
            assert np.array_equal(tbits(got), ubits(want)), (Y, me)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_ragged_lengths_and_int8_example(dtype):
    g = torch.Generator().manual_seed(3)
    for n in (0, 1, 5, 8, 9, 1023, 1024, 1025, 2048 + 3, 33 * 1024 + 7, (1 << 20) + 11):
        x = (torch.randn(n, generator=g) * 40).to(dtype).to(DEV)
        check_int(x, 7, 133)  # int8 with a quantum of 1
        check_int(x, 3, 131)  # int4 with a quantum of 4
    x = (torch.randn(1 << 16, generator=g) * 60).float().to(DEV)
    codes = exmy.encode_int(x, 7, 133)  # W = 8: the packed form of 8-bit codes is the bytes themselves
    assert torch.equal(codes.view(torch.int8), torch.round(x).clamp(-128, 127).to(torch.int8))
