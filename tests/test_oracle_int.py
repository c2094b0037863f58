"""Pins of the CPU oracle's two's complement reading of the X = 0 formats: the
paper's int4 range, the library's rounded / clamped integer conversions, and the
sign-magnitude functions wherever the two readings must agree."""
import numpy as np
import pytest
import torch

from oracle import exmy_oracle as O
from paper_2405_13938_amd import synth

F32, BF16 = O.F32, O.BF16


def unit_quantum_max_exp(Y):
    # quantum 2^(max_exp + 1 - 127 - Y) = 1
    return 126 + Y


def test_e0m3_is_int4(golden):
    (Y, lo, hi, count), = [[int(v) for v in row] for row in golden("e0m3_as_int4.txt")]
    me = unit_quantum_max_exp(Y)
    vals = O.from_codes_int(np.arange(1 << (Y + 1), dtype=np.uint32), F32, Y, me)
    assert vals.min() == lo and vals.max() == hi and np.unique(vals).size == count
    assert sorted(vals.tolist()) == list(range(lo, hi + 1))
    # codes are the two's complement bit patterns of the integers
    for k in range(lo, hi + 1):
        assert O.to_codes_int(np.array([k], dtype=np.float32), Y, me)[0] == k & 0xF
    # the sign-magnitude reading of the same bits has one value fewer and a double zero
    sm = O.from_codes(np.arange(16, dtype=np.uint32), F32, 0, Y, me)
    assert np.unique(sm).size == 15 and sm.min() == -7 and sm.max() == 7


@pytest.mark.parametrize("Y,tdtype", [(7, torch.int8), (15, torch.int16)])
def test_matches_library_integer_conversion(Y, tdtype):
    g = torch.Generator().manual_seed(Y)
    x = torch.randn(200000, generator=g) * (1 << Y) * 0.6
    x[:2000] = torch.randint(-(1 << Y) - 3, (1 << Y) + 3, (2000,), generator=g).float() + 0.5  # ties and the clamp edges
    x[2000:2004] = torch.tensor([float("inf"), float("-inf"), -0.0, 0.4999])
    want = torch.round(x).clamp(-(1 << Y), (1 << Y) - 1).to(tdtype)  # round-half-even, saturating
    codes = O.to_codes_int(x.numpy(), Y, unit_quantum_max_exp(Y))
    assert np.array_equal(codes, want.to(torch.int64).numpy() & ((2 << Y) - 1))
    back = O.from_codes_int(codes, F32, Y, unit_quantum_max_exp(Y))
    assert np.array_equal(back, want.float().numpy())


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("Y,max_exp", [(1, 126), (3, 129), (4, 120), (7, 133), (8, 127), (12, 140), (15, 100)])
def test_agrees_with_sign_magnitude_inside_the_common_range(dtype, Y, max_exp):
    if dtype == torch.bfloat16 and Y > 8:
        pytest.skip("does not fit a bf16 container")
    x = (synth.f32_edge_sweep(seed=Y) if dtype == torch.float32 else synth.all_bf16_patterns())
    xn = synth.bits_numpy(x)
    dt = F32 if dtype == torch.float32 else BF16
    a = O.emulate(xn, 0, Y, max_exp)
    b = O.emulate_int(xn, Y, max_exp)
    xf = x.float().numpy().astype(np.float64)
    q = 2.0 ** (max_exp + 1 - 127 - Y)
    fa = torch.from_numpy(a.view(np.int16 if dtype == torch.bfloat16 else np.int32)).view(dtype).float().numpy()
    fb = torch.from_numpy(b.view(np.int16 if dtype == torch.bfloat16 else np.int32)).view(dtype).float().numpy()
    fin = np.isfinite(xf)
    # same value wherever the sign-magnitude result is not the negative end of its range ...
    same = fin & ~(xf <= -((1 << Y) - 0.5) * q)
    assert np.array_equal(fa[same], fb[same])  # (-0 == +0 here)
    # ... and one step further down on the negative side
    low = fin & (xf <= -((1 << Y) - 0.5) * q)
    assert (fb[low] == -(1 << Y) * q).all() and (fa[low] == -((1 << Y) - 1) * q).all()
    # zero results are +0 in the two's complement reading
    ub = b.view(np.uint32 if dtype == torch.float32 else np.uint16)
    assert (ub[fin & (fb == 0)] == 0).all()
    # Inf / NaN kept bit-identical by emulation
    ux = xn.view(np.uint32 if dtype == torch.float32 else np.uint16)
    assert np.array_equal(ub[~fin], ux[~fin])
    # packed form = codes through the flat packer; decode(encode) = emulate on finite input
    codes = O.to_codes_int(xn, Y, max_exp)
    packed = O.encode_int(xn, Y, max_exp)
    assert np.array_equal(packed, O.pack(codes, 1 + Y))
    dec = O.decode_int(packed, dt, xn.size, Y, max_exp)
    ud = dec.view(np.uint32 if dtype == torch.float32 else np.uint16)
    assert np.array_equal(ud[fin], ub[fin])
    # Inf / NaN encode to the end of the range on the side of their sign
    neg = (ux >> (31 if dtype == torch.float32 else 15)).astype(bool)
    assert (codes[~fin & neg] == 1 << Y).all() and (codes[~fin & ~neg] == (1 << Y) - 1).all()


def test_int_validation():
    x = np.zeros(8, dtype=np.float32)
    with pytest.raises(Exception):
        O.encode_int(x, 0, 127)      # no magnitude bit
    with pytest.raises(Exception):
        O.encode_int(x, 16, 127)     # 17 bits: above the packed limit of this form
    with pytest.raises(Exception):
        O.encode_int(x, 3, 254)      # max_exp range of X = 0
    O.emulate_int(x, 20, 127)
