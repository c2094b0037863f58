"""Pins of the oracle's bit packing (power-of-2 decomposition, Section 2.2.2 and
Fig. 2).  Sizes and the structural properties are the paper's; the exact bit
positions inside a plane word are this repository's reading (parity unpinned by
the paper) and are fixed here by walking-one patterns."""
import numpy as np
import pytest

from oracle import exmy_oracle as O
from paper_2405_13938_amd import synth


def plane_sizes(W):
    return [s for s in (32, 16, 8, 4, 2, 1) if W & s]


def test_paper_plane_sizes(golden):
    for row in golden("packing_sizes.txt"):
        W, sizes = int(row[0]), [int(v) for v in row[1:]]
        assert plane_sizes(W) == sizes
        assert sum(sizes) * 8 == 8 * W  # perfect compression: 8 W-bit elements in 8W bits
        codes = np.zeros(8, dtype=np.uint32)
        assert O.pack(codes, W).size == W


@pytest.mark.parametrize("W", range(1, 33))
def test_roundtrip_and_size(W):
    rng = np.random.default_rng(W)
    for n in (0, 1, 7, 8, 9, 64, 1000, 4099):
        codes = rng.integers(0, 1 << W, size=n, dtype=np.uint64).astype(np.uint32)
        p = O.pack(codes, W)
        assert p.size == ((n + 7) // 8) * W == O.packed_bytes(n, 0, W - 1)
        assert np.array_equal(O.unpack(p, n, W), codes)
        assert np.array_equal(O.pack(codes, W, threads=3), p)


@pytest.mark.parametrize("W", [3, 5, 6, 7, 9, 12, 16, 17, 23, 31, 32])
def test_walking_one_bit_positions(W):
    """Code bit b of element j lands in exactly one bit of the blob: plane of the segment
    that owns b (widest plane owns the lowest bits), group word g, bit s*j + (b - lo)."""
    G = 3
    n = 8 * G
    sizes = plane_sizes(W)
    for g in range(G):
        for j in range(8):
            for b in range(W):
                codes = np.zeros(n, dtype=np.uint32)
                codes[8 * g + j] = 1 << b
                blob = O.pack(codes, W)
                bits = np.flatnonzero(np.unpackbits(blob, bitorder="little"))
                assert bits.size == 1
                lo, off = 0, 0
                for s in sizes:
                    if lo <= b < lo + s:
                        want = 8 * (off + g * s) + s * j + (b - lo)
                    lo += s
                    off += G * s
                assert bits[0] == want, (g, j, b)


def test_seven_bit_planes_by_hand():
    # 8 seven-bit codes -> one int32 (low nibbles), one int16 (bits 4-5), one int8 (bit 6)
    codes = np.array([0x7F, 0x00, 0x15, 0x2A, 0x40, 0x31, 0x0F, 0x70], dtype=np.uint32)
    blob = O.pack(codes, 7)
    w32 = sum(int(c & 0xF) << (4 * j) for j, c in enumerate(codes))
    w16 = sum(int((c >> 4) & 3) << (2 * j) for j, c in enumerate(codes))
    w8 = sum(int((c >> 6) & 1) << j for j, c in enumerate(codes))
    assert blob.tobytes() == w32.to_bytes(4, "little") + w16.to_bytes(2, "little") + w8.to_bytes(1, "little")


def test_wide_planes_are_plain_arrays():
    rng = np.random.default_rng(0)
    c8 = rng.integers(0, 256, size=64, dtype=np.uint32)
    assert np.array_equal(O.pack(c8, 8), c8.astype(np.uint8))
    c16 = rng.integers(0, 65536, size=64, dtype=np.uint32)
    assert np.array_equal(O.pack(c16, 16).view(np.uint16), c16.astype(np.uint16))
    c9 = rng.integers(0, 512, size=64, dtype=np.uint32)
    blob = O.pack(c9, 9)
    assert np.array_equal(blob[:64], (c9 & 0xFF).astype(np.uint8))
    assert np.array_equal(np.unpackbits(blob[64:], bitorder="little"), (c9 >> 8).astype(np.uint8))


@pytest.mark.parametrize("W", [5, 6, 7, 9])
def test_shard_then_pack_equals_pack_then_shard(W):
    """Section 2.2.2: the array can be sharded before or after packing."""
    rng = np.random.default_rng(W)
    n = 8 * 96
    codes = rng.integers(0, 1 << W, size=n, dtype=np.uint32)
    whole = O.pack(codes, W)
    G = n // 8
    for a, b in [(0, 8), (8, 64), (64, 96), (0, 96)]:  # shard bounds in groups
        shard = O.pack(codes[8 * a : 8 * b], W)
        off_w, off_s = 0, 0
        for s in plane_sizes(W):
            assert np.array_equal(shard[off_s : off_s + (b - a) * s], whole[off_w + a * s : off_w + b * s])
            off_w += G * s
            off_s += (b - a) * s


def test_packing_independent_of_format_split():
    """Section 2.2.2: the 7-bit layout is the same whether the codes are e4m2 or e3m3:
    encode == pack(to_codes) for every split, and pack only sees the W-bit integers."""
    x, _ = synth.cfg1(n=4096)
    xs = x.numpy()
    for X, Y in [(4, 2), (3, 3), (0, 6), (6, 0)]:
        codes = O.to_codes(xs, X, Y, 129)
        assert np.array_equal(O.encode(xs, X, Y, 129), O.pack(codes, 7))
        assert np.array_equal(O.decode(O.pack(codes, 7), O.F32, xs.size, X, Y, 129), O.from_codes(codes, O.F32, X, Y, 129))


def test_ragged_tail_is_zero_padded():
    codes = np.full(13, 0x7F, dtype=np.uint32)
    padded = np.concatenate([codes, np.zeros(3, dtype=np.uint32)])
    assert np.array_equal(O.pack(codes, 7), O.pack(padded, 7))
    x = np.linspace(-3, 3, 13, dtype=np.float32)
    p = O.encode(x, 3, 3, 128)
    assert p.size == 14
    assert np.array_equal(O.decode(p, O.F32, 13, 3, 3, 128), O.emulate(x, 3, 3, 128))


def test_threads_do_not_change_results():
    x = synth.cfg3(n=100_003).numpy()
    a = O.encode(x, 4, 2, 125, threads=1)
    assert np.array_equal(a, O.encode(x, 4, 2, 125, threads=5))
    assert np.array_equal(O.decode(a, O.F32, x.size, 4, 2, 125, threads=1), O.decode(a, O.F32, x.size, 4, 2, 125, threads=5))
    assert np.array_equal(O.emulate(x, 4, 2, 125, threads=1), O.emulate(x, 4, 2, 125, threads=5))


def test_e8m23_packs_to_the_float_itself():
    """W = 32 is e8m23 alone, the fp32 layout (Table 1 lists e8mY as fp32 / bf16 with fewer mantissa bits):
    one 32-bit segment, so the blob is the array of codes, and a finite float's code is its own bit pattern
    (max_exp 255: identity exponent map, denormals are the format's subnormals).  Inf / NaN clamp to the
    largest finite code under their sign."""
    rng = np.random.default_rng(5)
    bits = rng.integers(0, 1 << 32, size=4099, dtype=np.uint64).astype(np.uint32)
    bits[:8] = [0, 0x80000000, 1, 0x807FFFFF, 0x7F7FFFFF, 0xFF7FFFFF, 0x00800000, 0x3F800000]
    finite = (bits & 0x7F800000) != 0x7F800000
    blob = O.encode(bits.view(np.float32), 8, 23, 255)
    assert blob.size == ((bits.size + 7) // 8) * 32
    codes = blob.view(np.uint32)[: bits.size]
    assert np.array_equal(codes[finite], bits[finite])
    assert np.array_equal(codes[~finite], (bits[~finite] & 0x80000000) | 0x7F7FFFFF)
    assert not blob.view(np.uint32)[bits.size :].any()  # zero codes pad the last group
    back = O.decode(blob, O.F32, bits.size, 8, 23, 255).view(np.uint32)
    assert np.array_equal(back, codes)
    # a code with exponent field 255 is not a value: it decodes to the largest finite value
    odd = np.array([0x7F800000, 0xFFC00001, 0x7FFFFFFF, 0x3F800000] * 2, dtype=np.uint32)
    assert O.decode(odd.view(np.uint8), O.F32, 8, 8, 23, 255).view(np.uint32).tolist() == [0x7F7FFFFF, 0xFF7FFFFF, 0x7F7FFFFF, 0x3F800000] * 2
    with pytest.raises(Exception):
        O.encode(bits.view(np.float32), 8, 23, 254)
