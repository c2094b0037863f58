"""Pins of the CPU oracle's record arrangement (the plane words of a group one after another, W bytes per
group).  Not a layout of the paper: it holds the words of Section 2.2.2 / Fig. 2 in another order, so it
is pinned against the planar form (pinned in test_oracle_pack.py) through a numpy reshape, plus
walking-one bit positions."""
import numpy as np
import pytest
import torch

from oracle import exmy_oracle as O
from paper_2405_13938_amd import synth


def plane_sizes(W):
    return [s for s in (16, 8, 4, 2, 1) if W & s]


def records_from_planar(blob, n, W):
    G = (n + 7) // 8
    parts, off = [], 0
    for s in plane_sizes(W):
        parts.append(blob[off : off + G * s].reshape(G, s))
        off += G * s
    return np.concatenate(parts, axis=1).reshape(-1) if G else blob


@pytest.mark.parametrize("W", range(1, 17))
def test_records_are_the_planar_words_regrouped(W):
    for dtype in (torch.bfloat16, torch.float32):
        x = synth.bits_numpy(synth.shuffled(synth.all_bf16_patterns(), W).to(dtype)[: 4096 + 13])
        for X in range(0, min(W - 1, 8) + 1):
            Y = W - 1 - X
            if Y > (7 if X else 8) and dtype == torch.bfloat16:
                continue
            me = 255 if X == 8 else (130 if X else 128)
            for n in (0, 5, 8, 4096 + 13):
                planar = O.encode(x[:n], X, Y, me)
                rec = O.encode_records(x[:n], X, Y, me)
                assert rec.size == planar.size == ((n + 7) // 8) * W
                assert np.array_equal(rec, records_from_planar(planar, n, W)), (W, X, Y, n)
                dt = O.F32 if dtype == torch.float32 else O.BF16
                a, b = O.decode_records(rec, dt, n, X, Y, me), O.decode(planar, dt, n, X, Y, me)
                assert np.array_equal(a.view(np.uint32 if dt == O.F32 else np.uint16), b.view(np.uint32 if dt == O.F32 else np.uint16))


@pytest.mark.parametrize("X,Y", [(3, 3), (2, 1), (4, 3), (0, 4), (5, 7)])
def test_walking_one_positions(X, Y):
    """A single element with a single code bit set lands in exactly one bit of the blob: record g, the word of
    the segment that owns the bit (widest segment = lowest bits, first in the record), bit s*j + (b - lo)."""
    W = 1 + X + Y
    me = 130
    G = 3
    for g in range(G):
        for j in range(8):
            for b in range(W):
                code = 1 << b
                sign, mag = code >> (X + Y), code & ((1 << (X + Y)) - 1)
                v = O.code_value(X, Y, me, mag)
                x = np.zeros(8 * G, dtype=np.float32)
                x[8 * g + j] = -v if sign else v
                if sign and v == 0:
                    x[8 * g + j] = -0.0
                blob = O.encode_records(x, X, Y, me)
                bits = np.flatnonzero(np.unpackbits(blob, bitorder="little"))
                assert bits.size == 1, (g, j, b)
                lo, off = 0, 0
                for s in plane_sizes(W):
                    if lo <= b < lo + s:
                        want = 8 * (g * W + off) + s * j + (b - lo)
                    lo += s
                    off += s
                assert bits[0] == want, (g, j, b)


def test_seven_bit_record_by_hand():
    # e3m3, codes 0x7F 0x00 0x15 0x2A 0x40 0x31 0x0F 0x70: int32 word of the low nibbles, int16 word of bits 4-5,
    # int8 word of bit 6, 7 bytes in a row
    codes = [0x7F, 0x00, 0x15, 0x2A, 0x40, 0x31, 0x0F, 0x70]
    x = np.array([(-1.0 if c >> 6 else 1.0) * O.code_value(3, 3, 130, c & 0x3F) for c in codes], dtype=np.float32)
    x[4] = -0.0  # code 0x40: sign alone
    low = sum((c & 0xF) << (4 * j) for j, c in enumerate(codes))
    mid = sum(((c >> 4) & 3) << (2 * j) for j, c in enumerate(codes))
    top = sum(((c >> 6) & 1) << j for j, c in enumerate(codes))
    want = list(low.to_bytes(4, "little")) + list(mid.to_bytes(2, "little")) + [top]
    assert O.encode_records(x, 3, 3, 130).tolist() == want


def test_shards_are_contiguous_byte_ranges():
    x = synth.bits_numpy(synth.gaussian_bf16(4096, seed=3))
    whole = O.encode_records(x, 3, 3, 125)
    for a, b in ((0, 64), (64, 1024), (1000, 4096)):
        assert np.array_equal(O.encode_records(x[a:b], 3, 3, 125), whole[a // 8 * 7 : (b + 7) // 8 * 7])


def test_records_validation():
    x = np.zeros(8, dtype=np.float32)
    with pytest.raises(Exception):
        O.encode_records(x, 4, 12, 130)  # 17 bits
    with pytest.raises(Exception):
        O.encode_records(x, 3, 3, 6)
