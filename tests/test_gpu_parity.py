"""Parity of the HIP path (through the C ABI) with the CPU oracle, tolerance 0:
packed bytes, decoded and emulated bit patterns, histogram counts."""
import numpy as np
import pytest
import torch

import paper_2405_13938_amd as exmy
from oracle import exmy_oracle as O
from paper_2405_13938_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
THREADS = min(O.default_threads(), 16)


def odt(t):
    return O.F32 if t.dtype == torch.float32 else O.BF16


def ubits(a):
    """numpy array of floats or bit patterns -> unsigned bit patterns."""
    return a.view(np.uint32) if a.dtype == np.float32 else a


def tbits(t):
    return ubits(synth.bits_numpy(t))


def max_exp_of(host_bits, dt, X):
    """Per-tensor max exponent before rounding, clamped into the range valid for X."""
    hist = O.exponent_histogram(host_bits)
    m = O.max_exp_from_histogram(hist, 1.0)
    return clamp_max_exp(m, X)


def clamp_max_exp(m, X):
    if X == 8:
        return 255
    if X == 0:
        return min(max(m, 1), 253)
    return min(max(m, (1 << X) - 1), 254)


def check_all(x_dev, X, Y, max_exp, host=None, what=("encode", "decode", "emulate")):
    """Run the three operations on the GPU tensor x_dev and compare with the oracle."""
    n = x_dev.numel()
    if host is None:
        host = synth.bits_numpy(x_dev)
    dt = odt(x_dev)
    label = "e%dm%d max_exp=%d n=%d %s" % (X, Y, max_exp, n, x_dev.dtype)
    if 1 + X + Y <= 32 and Y <= 23 and ("encode" in what or "decode" in what):
        want_packed = O.encode(host, X, Y, max_exp, threads=THREADS)
        if "encode" in what:
            got = exmy.encode(x_dev.reshape(-1), X, Y, max_exp)
            torch.cuda.synchronize()
            assert np.array_equal(got.cpu().numpy(), want_packed), "encode " + label
        if "decode" in what:
            pd = torch.from_numpy(want_packed).to(DEV)
            got = exmy.decode(pd, x_dev.dtype, n, X, Y, max_exp)
            torch.cuda.synchronize()
            want = O.decode(want_packed, dt, n, X, Y, max_exp, threads=THREADS)
            assert np.array_equal(tbits(got), ubits(want)), "decode " + label
    if "emulate" in what:
        got = exmy.emulate(x_dev.clone().reshape(-1), X, Y, max_exp)
        torch.cuda.synchronize()
        want = O.emulate(host, X, Y, max_exp, threads=THREADS)
        assert np.array_equal(tbits(got), ubits(want)), "emulate " + label


def formats_of_width(W, dtype):
    P = 23 if dtype == torch.float32 else 7
    out = []
    for X in range(0, min(W - 1, 8) + 1):
        Y = W - 1 - X
        if Y <= (P if X >= 1 else P + 1):
            out.append((X, Y))
    return out


def some_max_exps(X):
    if X == 8:
        return [255]
    if X == 0:
        return [1, 126, 253]
    return sorted({(1 << X) - 1, max(125, (1 << X) - 1), 254})


# ------------------------------------------------------------ exhaustive inputs


@pytest.mark.parametrize("W", range(1, 17))
def test_every_bf16_pattern_every_format(W):
    """All 65536 bf16 bit patterns (every exponent, NaNs, Infs, denormals, +-0) plus a
    ragged tail, for every format of the width that a bf16 container holds."""
    x = torch.cat([synth.all_bf16_patterns(), synth.all_bf16_patterns()[12345:12350]]).to(DEV)
    host = synth.bits_numpy(x)
    for X, Y in formats_of_width(W, torch.bfloat16):
        for max_exp in some_max_exps(X):
            check_all(x, X, Y, max_exp, host)


@pytest.mark.parametrize("W", range(1, 32))
def test_fp32_edge_sweep_every_format(W):
    """fp32 patterns at and around every rounding tie of every exponent, plus random bits."""
    x = synth.f32_edge_sweep()
    x = torch.cat([x, x[:3]]).to(DEV)
    host = synth.bits_numpy(x)
    for X, Y in formats_of_width(W, torch.float32):
        for max_exp in some_max_exps(X):
            check_all(x, X, Y, max_exp, host)


@pytest.mark.parametrize("W", range(17, 32))
def test_sampled_code_points_of_wide_formats_decode(W):
    """Formats wider than 16 bits: sampled codes (both ends of the code space included) through the packed form."""
    rng = np.random.default_rng(W)
    mags = np.unique(np.concatenate([rng.integers(0, 1 << (W - 1), 100000), np.arange(0, 2000),
                                     (1 << (W - 1)) - 1 - np.arange(0, 2000)])).astype(np.uint32)
    codes = np.concatenate([mags, mags | np.uint32(1 << (W - 1))])[:-3]  # ragged
    n = codes.size
    pd = torch.from_numpy(O.pack(codes, W)).to(DEV)
    for X, Y in formats_of_width(W, torch.float32):
        if Y > 23:
            continue  # e0m24 has no packed form
        for max_exp in some_max_exps(X):
            got = exmy.decode(pd, torch.float32, n, X, Y, max_exp)
            torch.cuda.synchronize()
            assert np.array_equal(tbits(got), ubits(O.from_codes(codes, O.F32, X, Y, max_exp))), (W, X, Y, max_exp)


def test_e8m23_is_the_array_of_codes():
    """W = 32: finite elements are their own codes; Inf / NaN and codes with exponent field 255 clamp."""
    for n in (0, 3, 8, 4099, (1 << 20) + 5):
        x, _ = synth.cfg1(n=max(n, 16), seed=n)
        x = x[:n].contiguous().to(DEV)
        host = synth.bits_numpy(x)
        packed = exmy.encode(x, 8, 23, 255)
        torch.cuda.synchronize()
        assert np.array_equal(packed.cpu().numpy(), O.encode(host, 8, 23, 255, threads=THREADS)), n
        rng = np.random.default_rng(n)
        codes = rng.integers(0, 1 << 32, size=(n + 7) // 8 * 8, dtype=np.uint64).astype(np.uint32)
        got = exmy.decode(torch.from_numpy(codes.view(np.uint8)).to(DEV), torch.float32, n, 8, 23, 255)
        torch.cuda.synchronize()
        assert np.array_equal(tbits(got), ubits(O.decode(codes.view(np.uint8), O.F32, n, 8, 23, 255, threads=THREADS))), n


def test_wide_formats_batch_and_histogram():
    xs = [synth.cfg1(n=(1 << 18) + 8 * k + k, seed=k)[0].to(DEV) for k in range(5)]
    for X, Y in ((8, 10), (5, 14), (4, 23), (8, 22), (8, 23)):
        me = 255 if X == 8 else 131
        outs = exmy.encode_batch(xs, X, Y, [me] * 5)
        torch.cuda.synchronize()
        for x, o in zip(xs, outs):
            assert np.array_equal(o.cpu().numpy(), O.encode(synth.bits_numpy(x), X, Y, me, threads=THREADS))
        decs = exmy.decode_batch(outs, torch.float32, [x.numel() for x in xs], X, Y, [me] * 5)
        torch.cuda.synchronize()
        for x, o, d in zip(xs, outs, decs):
            assert np.array_equal(tbits(d), ubits(O.decode(o.cpu().numpy(), O.F32, x.numel(), X, Y, me, threads=THREADS)))
        p, h = exmy.encode_with_histogram(xs[0], X, Y, me)
        torch.cuda.synchronize()
        assert torch.equal(p, outs[0])
        assert np.array_equal(h.cpu().numpy().astype(np.uint64), O.exponent_histogram(synth.bits_numpy(xs[0])))


def test_emulate_wider_than_packable():
    x = synth.f32_edge_sweep().to(DEV)
    host = synth.bits_numpy(x)
    for X, Y, max_exp in [(8, 10, 255), (8, 23, 255), (5, 10, 143), (4, 21, 130), (3, 22, 140), (2, 23, 128), (0, 24, 100)]:
        check_all(x, X, Y, max_exp, host, what=("emulate",))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_every_code_point_decodes(dtype):
    """Every code of every packable format, through the packed form."""
    for W in range(1, 17):
        codes = np.arange(1 << W, dtype=np.uint32)
        codes = np.concatenate([codes, codes[: (3 if W > 2 else 1)]])  # ragged
        n = codes.size
        blob = O.pack(codes, W)
        pd = torch.from_numpy(blob).to(DEV)
        for X, Y in formats_of_width(W, dtype):
            for max_exp in some_max_exps(X):
                got = exmy.decode(pd, dtype, n, X, Y, max_exp)
                torch.cuda.synchronize()
                want = O.from_codes(codes, O.F32 if dtype == torch.float32 else O.BF16, X, Y, max_exp)
                assert np.array_equal(tbits(got), ubits(want)), (W, X, Y, max_exp)


# ------------------------------------------------------------------ edge sizes


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_small_and_ragged_sizes(dtype):
    base, _ = synth.cfg1(n=70000)
    base = base.to(dtype)
    for n in (1, 2, 7, 8, 9, 15, 16, 17, 63, 64, 65, 2047, 2048, 2049, 8191, 8193, 16385, 65536 + 7):
        x = base[:n].contiguous().to(DEV)
        check_all(x, 3, 3, 129)
        check_all(x, 4, 0, 129)
    # n = 0: nothing happens, nothing fails
    empty = torch.empty(0, dtype=dtype, device=DEV)
    assert exmy.encode(empty, 3, 3, 129).numel() == 0
    assert exmy.decode(torch.empty(0, dtype=torch.uint8, device=DEV), dtype, 0, 3, 3, 129).numel() == 0
    exmy.emulate(empty, 3, 3, 129)
    assert int(exmy.exponent_histogram(empty).sum()) == 0


def test_outputs_do_not_spill():
    """Bytes after the packed blob and elements after the decoded tensor are left alone."""
    n = 8 * 1000 + 3
    x = synth.gaussian_bf16(n).to(DEV)
    nb = exmy.packed_bytes(n, 3, 3)
    buf = torch.full((nb + 64,), 0xAB, dtype=torch.uint8, device=DEV)
    exmy.encode(x, 3, 3, 122, out=buf[:nb])
    out = torch.full((n + 32,), 7.0, dtype=torch.bfloat16, device=DEV)
    exmy.decode(buf[:nb], torch.bfloat16, n, 3, 3, 122, out=out[:n])
    torch.cuda.synchronize()
    assert bool((buf[nb:] == 0xAB).all()) and bool((out[n:] == 7.0).all())


def test_errors_raise():
    x = torch.zeros(64, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(exmy.ExmyError):
        exmy.encode(x, 3, 8, 130)  # bf16 cannot hold 8 mantissa bits
    with pytest.raises(exmy.ExmyError):
        exmy.encode(x, 3, 3, 3)  # max_exp below 2^X - 1
    with pytest.raises(exmy.ExmyError):
        exmy.emulate(x[1:33], 3, 3, 130)  # 2-byte offset: not 16-byte aligned
    with pytest.raises(ValueError):
        exmy.encode(torch.zeros(8, 8, device=DEV).t(), 3, 3, 130)  # not contiguous


# --------------------------------------------------------------- configurations


def test_cfg1_fp32_with_specials():
    x, pos = synth.cfg1()
    host = synth.bits_numpy(x)
    # max exponent of the N(0,1) body: the injected FLT_MAX / Inf / NaN must saturate
    body = np.ones(host.size, dtype=bool)
    body[pos.numpy()] = False
    max_exp = clamp_max_exp(int(((host.view(np.uint32)[body] >> 23) & 0xFF).max()), 3)
    xd = x.to(DEV)
    check_all(xd, 3, 3, max_exp, host)
    assert exmy.packed_bytes(x.numel(), 3, 3) == 917504
    # the specials, one by one
    packed = exmy.encode(xd, 3, 3, max_exp)
    back = exmy.decode(packed, torch.float32, x.numel(), 3, 3, max_exp).cpu()
    top = O.code_value(3, 3, max_exp, 0x3F)
    sp = back[pos]
    vals = synth.special_values_f32()
    for v, got in zip(vals, sp.tolist()):
        if (v & 0x7FFFFFFF) >= 0x7F7FFFFF:  # NaN, Inf, FLT_MAX -> largest normal, sign kept
            assert abs(got) == top and (got < 0) == bool(v >> 31)
        elif (v & 0x7FFFFFFF) <= 0x00800000:  # zeros, denormals, FLT_MIN -> signed zero
            assert got == 0.0 and np.signbit(np.float32(got)) == bool(v >> 31)


@pytest.mark.parametrize("W", [3, 5, 6, 7, 9])
def test_cfg2_bf16_weights_all_formats(W):
    x = synth.cfg2(device=DEV)
    host = synth.bits_numpy(x)
    for X, Y in formats_of_width(W, torch.bfloat16):
        check_all(x, X, Y, max_exp_of(host, O.BF16, X), host)


def test_cfg3_fp32_lognormal_full_size():
    x = synth.cfg3(device=DEV)
    host = synth.bits_numpy(x)
    hist = O.exponent_histogram(host)
    for X, Y in ((4, 2), (2, 3)):
        # metadata from the tensor maximum, then from 99.9 % coverage so that the normal,
        # subnormal, flush and saturate outcomes all occur in bulk
        for cov in (1.0, 0.999):
            max_exp = clamp_max_exp(O.max_exp_from_histogram(hist, cov), X)
            check_all(x, X, Y, max_exp, host, what=("encode", "decode"))


def test_cfg4_bf16_activations_with_histogram():
    x = synth.cfg4(device=DEV)
    host = synth.bits_numpy(x)
    want_hist = O.exponent_histogram(host)
    hist = exmy.exponent_histogram(x)
    torch.cuda.synchronize()
    assert np.array_equal(hist.cpu().numpy().view(np.uint64), want_hist)
    max_exp0 = exmy.max_exp_from_histogram(hist, 0.99)
    assert max_exp0 == O.max_exp_from_histogram(want_hist, 0.99)
    for X, Y in ((5, 0), (4, 3)):
        max_exp = clamp_max_exp(max_exp0, X)
        want_packed = O.encode(host, X, Y, max_exp, threads=THREADS)
        packed, h2 = exmy.encode_with_histogram(x.reshape(-1), X, Y, max_exp)
        torch.cuda.synchronize()
        assert np.array_equal(packed.cpu().numpy(), want_packed)
        assert np.array_equal(h2.cpu().numpy().view(np.uint64), want_hist)
        # accumulation: a second pass doubles every count
        exmy.exponent_histogram(x, h2)
        torch.cuda.synchronize()
        assert np.array_equal(h2.cpu().numpy().view(np.uint64), 2 * want_hist)
        got = exmy.decode(packed, torch.bfloat16, x.numel(), X, Y, max_exp)
        torch.cuda.synchronize()
        want = O.decode(want_packed, O.BF16, x.numel(), X, Y, max_exp, threads=THREADS)
        assert np.array_equal(tbits(got), want)
        # saturation is on: outliers decode to the largest normal
        top = O.code_value(X, Y, max_exp, (1 << (X + Y)) - 1)
        assert float(got.float().abs().max()) == top < 1e4


def test_batch_equals_single_calls():
    """exmy_encode_batch / exmy_decode_batch: mixed sizes (several launches, sizes far apart,
    ragged and empty tensors), per-tensor max_exp, more tensors than one launch holds."""
    X, Y = 3, 3
    rng = np.random.default_rng(9)
    sizes = [4096, 4096, 1 << 20, (1 << 20) + 8, 3 * (1 << 18), 5, 0, 1 << 16, 12345, 1 << 20] + [4096 + 8 * i for i in range(70)]
    for dtype in (torch.bfloat16, torch.float32):
        srcs, max_exps = [], []
        for k, n in enumerate(sizes):
            x = (synth.gaussian_bf16(max(n, 1), std=0.02 * (1 + k % 5), seed=100 + k)[:n]).to(dtype).to(DEV)
            srcs.append(x)
            max_exps.append(int(rng.integers(118, 126)))
        outs = exmy.encode_batch(srcs, X, Y, max_exps)
        torch.cuda.synchronize()
        for x, m, o in zip(srcs, max_exps, outs):
            want = O.encode(synth.bits_numpy(x), X, Y, m) if x.numel() else np.zeros(0, dtype=np.uint8)
            assert np.array_equal(o.cpu().numpy(), want), (dtype, x.numel(), m)
        back = exmy.decode_batch(outs, dtype, [x.numel() for x in srcs], X, Y, max_exps)
        torch.cuda.synchronize()
        for x, m, o, b in zip(srcs, max_exps, outs, back):
            if x.numel():
                want = O.decode(o.cpu().numpy(), odt(x), x.numel(), X, Y, m)
                assert np.array_equal(tbits(b), ubits(want)), (dtype, x.numel(), m)
    # any invalid tensor: nothing is launched
    good = torch.zeros(64, dtype=torch.bfloat16, device=DEV)
    out0 = torch.full((exmy.packed_bytes(64, X, Y),), 0xCD, dtype=torch.uint8, device=DEV)
    out1 = out0.clone()
    with pytest.raises(exmy.ExmyError):
        exmy.encode_batch([good, good], X, Y, [120, 3], outs=[out0, out1])
    torch.cuda.synchronize()
    assert bool((out0 == 0xCD).all()) and bool((out1 == 0xCD).all())


def test_cfg5_checkpoint_batched():
    """The whole checkpoint through exmy_encode_batch / exmy_decode_batch: equal to the
    per-tensor calls everywhere (GPU compare over all 6.5 G elements) and to the oracle on
    layer 0 and on a shard of every tensor."""
    X, Y = 3, 3
    flat, table = synth.cfg5(device=DEV)
    srcs = [flat[off : off + sz] for _, off, sz in table]
    max_exps = [clamp_max_exp(int(t.abs().max().view(torch.int16).item() >> 7), X) for t in srcs]
    total = sum(exmy.packed_bytes(t.numel(), X, Y) for t in srcs)
    buf = torch.empty(total, dtype=torch.uint8, device=DEV)
    packs, poff = [], 0
    for t in srcs:
        nb = exmy.packed_bytes(t.numel(), X, Y)
        packs.append(buf[poff : poff + nb])
        poff += nb
    exmy.encode_batch(srcs, X, Y, max_exps, outs=packs)
    out = torch.empty_like(flat)
    outs = [out[off : off + sz] for _, off, sz in table]
    exmy.decode_batch(packs, torch.bfloat16, [t.numel() for t in srcs], X, Y, max_exps, outs=outs)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    for i, (t, m, p, o) in enumerate(zip(srcs, max_exps, packs, outs)):
        if i < 9 or t.numel() <= (1 << 20):
            a, b = 0, t.numel()
        else:
            a = int(rng.integers(0, (t.numel() - (1 << 19)) // 8)) * 8
            b = a + (1 << 19)
        want = O.encode(synth.bits_numpy(t[a:b]), X, Y, m, threads=THREADS)
        G, g, wo, po = t.numel() // 8, (b - a) // 8, 0, 0
        for s in (4, 2, 1):
            assert np.array_equal(p[po + (a // 8) * s : po + (b // 8) * s].cpu().numpy(), want[wo : wo + g * s]), (i, s)
            wo += g * s
            po += G * s
        assert np.array_equal(tbits(o[a:b]), O.decode(want, O.BF16, b - a, X, Y, m, threads=THREADS)), i
    # against the single-tensor entry points, every byte
    for t, m, p, o in zip(srcs[:27] + srcs[-27:], max_exps[:27] + max_exps[-27:], packs[:27] + packs[-27:], outs[:27] + outs[-27:]):
        single = exmy.encode(t, X, Y, m)
        assert torch.equal(single, p)
        assert torch.equal(exmy.decode(single, torch.bfloat16, t.numel(), X, Y, m).view(torch.int16), o.view(torch.int16))


def test_cfg5_checkpoint_stream_of_calls():
    """288 tensors encoded by 288 calls into one buffer at running offsets, then decoded.  The oracle encodes
    and decodes every tensor whole (all 6.5 G elements; about half a minute of host time) and every packed
    byte and decoded bit pattern is compared.  A few tensors are also checked shard-wise: the oracle's codes of
    an 8-aligned range of elements must be the slice of each plane that the range owns (Section 2.2.2:
    sharding before or after packing gives the same bytes)."""
    X, Y, W = 3, 3, 7
    flat, table = synth.cfg5(device=DEV)
    assert len(table) == 288 and flat.numel() == 6476267520
    total_packed = sum(exmy.packed_bytes(sz, X, Y) for _, _, sz in table)
    assert total_packed == 5666734080
    buf = torch.empty(total_packed, dtype=torch.uint8, device=DEV)
    out = torch.empty_like(flat)
    # per-tensor metadata: max exponent before rounding (Gaussian weights never reach 2^0)
    metas, poff = [], 0
    for name, off, sz in table:
        t = flat[off : off + sz]
        max_exp = clamp_max_exp(int(t.abs().max().view(torch.int16).item() >> 7), X)
        metas.append((off, sz, poff, max_exp))
        poff += exmy.packed_bytes(sz, X, Y)
    for off, sz, poff, max_exp in metas:
        nb = exmy.packed_bytes(sz, X, Y)
        assert poff % 16 == 0
        exmy.encode(flat[off : off + sz], X, Y, max_exp, out=buf[poff : poff + nb])
    for off, sz, poff, max_exp in metas:
        nb = exmy.packed_bytes(sz, X, Y)
        exmy.decode(buf[poff : poff + nb], torch.bfloat16, sz, X, Y, max_exp, out=out[off : off + sz])
    torch.cuda.synchronize()
    rng = np.random.default_rng(4)
    for i, (off, sz, poff, max_exp) in enumerate(metas):
        nb = exmy.packed_bytes(sz, X, Y)
        host = synth.bits_numpy(flat[off : off + sz])
        want = O.encode(host, X, Y, max_exp, threads=THREADS)
        assert np.array_equal(buf[poff : poff + nb].cpu().numpy(), want), i
        want_dec = O.decode(want, O.BF16, sz, X, Y, max_exp, threads=THREADS)
        assert np.array_equal(tbits(out[off : off + sz]), want_dec), i
        if i % 37 == 0 and sz > (1 << 20):
            G = sz // 8
            a = int(rng.integers(0, (sz - (1 << 20)) // 8)) * 8
            b = a + (1 << 20)
            shard = O.encode(host[a:b], X, Y, max_exp, threads=THREADS)
            g = (b - a) // 8
            wo, po = 0, 0
            for s_ in (4, 2, 1):
                assert np.array_equal(want[po + (a // 8) * s_ : po + (b // 8) * s_], shard[wo : wo + g * s_]), (i, s_)
                wo += g * s_
                po += G * s_
        if i % 36 == 0:
            print("cfg5: tensors 0..%d match the oracle whole" % i, flush=True)
    # a property that holds at any size: decode(encode(x)) == emulate(x), checked on the GPU
    # over the first two and the last layer, tensor by tensor
    for off, sz, poff, max_exp in metas[:18] + metas[-9:]:
        emu = exmy.emulate(flat[off : off + sz].clone(), X, Y, max_exp)
        assert torch.equal(emu.view(torch.int16), out[off : off + sz].view(torch.int16))
