"""Parity of the per-block-metadata entry points (through the C ABI) with the CPU
oracle, tolerance 0: metadata bytes, packed bytes, decoded and emulated bit patterns."""
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
    return a.view(np.uint32) if a.dtype == np.float32 else a


def tbits(t):
    return ubits(synth.bits_numpy(t))


def formats_of_width(W, dtype):
    P = 23 if dtype == torch.float32 else 7
    return [(X, W - 1 - X) for X in range(0, min(W - 1, 7) + 1) if W - 1 - X <= (P if X >= 1 else P + 1)]


def metadata(kind, host, block, X, seed=0):
    nb = (host.size + block - 1) // block
    if kind == "before_rounding":
        return O.block_max_exp(host, block, X)
    rng = np.random.default_rng(seed + block)
    if kind == "any_byte":  # out-of-range bytes, and ones that need the fp64 rounding path, included
        return rng.integers(0, 256, nb).astype(np.uint8)
    if kind == "near_before_rounding":  # the block maximum, moved by up to two binades either way
        m = O.block_max_exp(host, block, X).astype(np.int64) + rng.integers(-2, 3, nb)
        return np.clip(m, 0, 255).astype(np.uint8)
    raise ValueError(kind)


def check_blocks(x_dev, block, X, Y, kind, host=None, what=("max", "encode", "decode", "emulate"), seed=0):
    x_dev = x_dev.reshape(-1)
    n = x_dev.numel()
    if host is None:
        host = synth.bits_numpy(x_dev)
    dt = odt(x_dev)
    label = "e%dm%d block=%d n=%d %s %s" % (X, Y, block, n, x_dev.dtype, kind)
    if "max" in what:
        got = exmy.block_max_exp(x_dev, block, X)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), O.block_max_exp(host, block, X)), "block_max_exp " + label
    meta = metadata(kind, host, block, X, seed)
    meta_dev = torch.from_numpy(meta).to(DEV)
    if 1 + X + Y <= 16 and ("encode" in what or "decode" in what):
        want_packed = O.encode_blocks(host, block, X, Y, meta, threads=THREADS)
        if "encode" in what:
            got = exmy.encode_blocks(x_dev, block, X, Y, meta_dev)
            torch.cuda.synchronize()
            assert np.array_equal(got.cpu().numpy(), want_packed), "encode_blocks " + label
        if "decode" in what:
            pd = torch.from_numpy(want_packed).to(DEV)
            got = exmy.decode_blocks(pd, x_dev.dtype, n, block, X, Y, meta_dev)
            torch.cuda.synchronize()
            want = O.decode_blocks(want_packed, dt, n, block, X, Y, meta, threads=THREADS)
            assert np.array_equal(tbits(got), ubits(want)), "decode_blocks " + label
    if "emulate" in what:
        got = exmy.emulate_blocks(x_dev.clone(), block, X, Y, meta_dev)
        torch.cuda.synchronize()
        want = O.emulate_blocks(host, block, X, Y, meta, threads=THREADS)
        assert np.array_equal(tbits(got), ubits(want)), "emulate_blocks " + label


SMALL_BLOCKS = [8, 16, 32, 64, 128, 256, 512]  # looked up per lane inside flat tiles
ROW_BLOCKS = [24, 520, 1024, 4096, 11008]      # workgroups of their own


@pytest.mark.parametrize("W", range(1, 17))
def test_every_bf16_pattern_every_width(W):
    # all 65536 bf16 bit patterns (shuffled, so every block mixes binades), every (X, Y) of the width,
    # one small and one row block size per format, metadata of every kind
    x = synth.shuffled(synth.all_bf16_patterns(), W).to(DEV)
    host = synth.bits_numpy(x)
    for i, (X, Y) in enumerate(formats_of_width(W, torch.bfloat16)):
        sb = SMALL_BLOCKS[(W + i) % len(SMALL_BLOCKS)]
        rb = ROW_BLOCKS[(W + i) % len(ROW_BLOCKS)]
        check_blocks(x, sb, X, Y, "any_byte", host, seed=i)
        check_blocks(x, rb, X, Y, "any_byte", host, seed=i)
        check_blocks(x, sb, X, Y, "before_rounding", host, what=("encode", "decode", "emulate"))
        check_blocks(x, rb, X, Y, "near_before_rounding", host, what=("encode", "decode", "emulate"))


@pytest.mark.parametrize("W", range(1, 17))
def test_fp32_sweep_every_width(W):
    x = synth.shuffled(synth.f32_edge_sweep(seed=W), W).to(DEV)
    host = synth.bits_numpy(x)
    for i, (X, Y) in enumerate(formats_of_width(W, torch.float32)):
        sb = SMALL_BLOCKS[(W + i + 3) % len(SMALL_BLOCKS)]
        rb = ROW_BLOCKS[(W + i + 2) % len(ROW_BLOCKS)]
        check_blocks(x, sb, X, Y, "any_byte", host, seed=i)
        check_blocks(x, rb, X, Y, "any_byte", host, seed=i)
        check_blocks(x, rb, X, Y, "before_rounding", host, what=("encode", "decode", "emulate"))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_emulate_only_formats(dtype):
    # wider than the packed form allows, fp64 rounding path for the whole format (Y > 21) included
    x = synth.shuffled(synth.f32_edge_sweep(seed=3) if dtype == torch.float32 else synth.all_bf16_patterns(), 3).to(DEV)
    host = synth.bits_numpy(x)
    fmts = [(7, 7), (5, 7), (0, 8)] if dtype == torch.bfloat16 else [(7, 23), (2, 22), (4, 21), (0, 24), (7, 12), (3, 20)]
    for X, Y in fmts:
        for block in (32, 512, 1000, 4096):
            for kind in ("any_byte", "before_rounding"):
                check_blocks(x, block, X, Y, kind, host, what=("emulate",))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("block", [8, 32, 512, 24, 4096])
def test_every_block_size_at_ragged_lengths(dtype, block):
    # lengths around multiples of the block, of the group of 8 and of the kernels' tiles
    g = torch.Generator().manual_seed(block)
    lengths = sorted({1, 3, 7, 8, 9, 15, 17, block - 1, block, block + 1, block + 8, 2 * block + 5, 3 * block - 3,
                      1023, 1025, 2047, 2048 + 4, 4096 + 12, 5 * 4096 + 8 * 7 + 3, 33 * 1024 + 1})
    for n in lengths:
        x = (torch.randn(n, generator=g) * torch.exp2(torch.randint(-10, 10, (n,), generator=g).float())).to(dtype).to(DEV)
        for X, Y in ((3, 3), (2, 1), (0, 4)):
            check_blocks(x, block, X, Y, "near_before_rounding", seed=n)


def test_no_finite_value_in_a_block_and_empty_input():
    x = torch.randn(4096).to(torch.bfloat16)
    x[64:128] = float("nan")
    x[128:192] = float("inf")
    x[192:256] = 0.0
    x[256:320] = 1e-40  # below the normals of the container (flushes to 0 in bf16; kept tiny in fp32)
    for dtype in (torch.bfloat16, torch.float32):
        xd = x.to(dtype).to(DEV)
        for block in (64, 1024):
            check_blocks(xd, block, 3, 2, "before_rounding")
        empty = torch.empty(0, dtype=dtype, device=DEV)
        meta = torch.empty(0, dtype=torch.uint8, device=DEV)
        assert exmy.block_max_exp(empty, 32, 3).numel() == 0
        assert exmy.encode_blocks(empty, 32, 3, 3, meta).numel() == 0
        assert exmy.decode_blocks(torch.empty(0, dtype=torch.uint8, device=DEV), dtype, 0, 32, 3, 3, meta).numel() == 0
        assert exmy.emulate_blocks(empty, 32, 3, 3, meta).numel() == 0


@pytest.mark.parametrize("block", [64, 4096, 11008])
def test_weight_matrix_rows_and_sub_rows(block):
    # Section 4.1: one metadatum per row of the weight matrix, or per sub-row block
    x = synth.gaussian_bf16(1024 * 11008 if block == 11008 else 4096 * 4096, seed=block).to(DEV)
    host = synth.bits_numpy(x)
    for X, Y in ((3, 2), (2, 1), (1, 2)):
        check_blocks(x, block, X, Y, "before_rounding", host)


def test_many_short_rows():
    # 70000 rows of 1024 elements, each less than a tile of some kernels
    x = synth.gaussian_bf16(70000 * 1024 + 100, seed=17).to(DEV)
    check_blocks(x, 1024, 3, 3, "before_rounding")


def test_uniform_metadata_equals_per_tensor_entry_points():
    x = synth.gaussian_bf16(1 << 20, seed=4).to(DEV)
    for block in (32, 4096):
        meta = torch.full((exmy.block_count(x.numel(), block),), 127, dtype=torch.uint8, device=DEV)
        a = exmy.encode_blocks(x, block, 3, 3, meta)
        b = exmy.encode(x, 3, 3, 127)
        assert torch.equal(a, b)
        assert torch.equal(exmy.decode_blocks(a, torch.bfloat16, x.numel(), block, 3, 3, meta).view(torch.int16),
                           exmy.decode(b, torch.bfloat16, x.numel(), 3, 3, 127).view(torch.int16))
        assert torch.equal(exmy.emulate_blocks(x.clone(), block, 3, 3, meta).view(torch.int16),
                           exmy.emulate(x.clone(), 3, 3, 127).view(torch.int16))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_max_exp_after_rounding(dtype):
    # every rounding position, blocks of every launch form, maxima at ties and at carries into the next binade
    x = synth.shuffled(synth.f32_edge_sweep(seed=11) if dtype == torch.float32 else synth.all_bf16_patterns(), 11).to(DEV)
    host = synth.bits_numpy(x)
    P = 23 if dtype == torch.float32 else 7
    for X in (0, 1, 3, 7):
        for Y in sorted({0, 1, 2, 3, P - 1, P, P + 1 if X == 0 else P}):
            for block in (8, 64, 512, 24, 1024, 4096, 40000):
                got = exmy.block_max_exp_after_rounding(x, block, X, Y)
                torch.cuda.synchronize()
                want = O.block_max_exp_after_rounding(host, block, X, Y)
                assert np.array_equal(got.cpu().numpy(), want), (dtype, X, Y, block)


@pytest.mark.parametrize("scheme", [exmy.binding.BEFORE_ROUNDING, exmy.binding.AFTER_ROUNDING])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_encode_blocks_auto(scheme, dtype):
    # every launch form: blocks inside flat tiles, a wavefront-sized or a full workgroup per block with few or
    # many groups per lane, and the two-launch fallback (odd small blocks, very long blocks); ragged ends
    g = torch.Generator().manual_seed(21 + scheme)
    n = 300 * 1024 + 13
    x = (torch.randn(n, generator=g) * torch.exp2(torch.randint(-10, 10, (n,), generator=g).float()))
    x[::1001] = float("inf")
    x[5::1003] = float("nan")
    x[4096:8192] = 0.0
    x = x.to(dtype).to(DEV)
    host = synth.bits_numpy(x)
    fmts = [(2, 1), (3, 3), (1, 2), (0, 4), (4, 3), (5, 2), (7, 0), (4, 7)]
    blocks = [8, 16, 32, 64, 128, 256, 512, 24, 520, 1024, 2048, 2056, 4096, 8192, 11008, 16384, 22016, 32768, 40000, 65536, 1 << 18]
    for i, block in enumerate(blocks):
        X, Y = fmts[i % len(fmts)]
        for nn in (n, n - n % block if n >= block else n, 7, block + 3):
            xd, hd = x[:nn], host[:nn]
            packed, meta = exmy.encode_blocks_auto(xd, block, X, Y, scheme)
            torch.cuda.synchronize()
            want_meta = (O.block_max_exp_after_rounding(hd, block, X, Y) if scheme else O.block_max_exp(hd, block, X))
            assert np.array_equal(meta.cpu().numpy(), want_meta), (block, X, Y, nn)
            want = O.encode_blocks(hd, block, X, Y, want_meta, threads=THREADS)
            assert np.array_equal(packed.cpu().numpy(), want), (block, X, Y, nn)


@pytest.mark.parametrize("W", range(1, 17))
def test_encode_blocks_auto_every_width(W):
    x = synth.shuffled(synth.all_bf16_patterns(), 500 + W).to(DEV)
    host = synth.bits_numpy(x)
    x32 = synth.shuffled(synth.f32_edge_sweep(seed=W), 600 + W).to(DEV)
    host32 = synth.bits_numpy(x32)
    for i, (X, Y) in enumerate(formats_of_width(W, torch.bfloat16)):
        for block in ([16, 1024, 4096, 11008][(W + i) % 4], [512, 520, 8192, 32768][(W + i) % 4]):
            scheme = (W + i) % 2
            packed, meta = exmy.encode_blocks_auto(x, block, X, Y, scheme)
            torch.cuda.synchronize()
            want_meta = (O.block_max_exp_after_rounding(host, block, X, Y) if scheme else O.block_max_exp(host, block, X))
            assert np.array_equal(meta.cpu().numpy(), want_meta), (block, X, Y)
            assert np.array_equal(packed.cpu().numpy(), O.encode_blocks(host, block, X, Y, want_meta, threads=THREADS))
    for i, (X, Y) in enumerate(formats_of_width(W, torch.float32)):
        block = [32, 1024, 4096, 16384][(W + i) % 4]
        scheme = (W + i + 1) % 2
        packed, meta = exmy.encode_blocks_auto(x32, block, X, Y, scheme)
        torch.cuda.synchronize()
        want_meta = (O.block_max_exp_after_rounding(host32, block, X, Y) if scheme else O.block_max_exp(host32, block, X))
        assert np.array_equal(meta.cpu().numpy(), want_meta), (block, X, Y)
        assert np.array_equal(packed.cpu().numpy(), O.encode_blocks(host32, block, X, Y, want_meta, threads=THREADS))


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("block", [8, 32, 512, 1024, 4096])
def test_one_pass_partial_last_tile_runs_as_a_partial_tile(dtype, block):
    """Regression test of the tile bookkeeping of the one-pass metadata + codes kernels: a compiler-made select
    on a stale condition code once let the partial last workgroup tile run as a whole one.  Lengths end a few
    groups into a tile, a few groups short of one, and on a tile boundary, for every tile size in use (64 to
    1024 groups); outputs sit in guard bytes, so that a tile running past its end is seen as well."""
    g = torch.Generator().manual_seed(block)
    base = 6 * 8192
    x_all = (torch.randn(base + 8200, generator=g) * torch.exp2(torch.randint(-8, 8, (base + 8200,), generator=g).float())).to(dtype).to(DEV)
    h_all = synth.bits_numpy(x_all)
    X, Y = 3, 3
    for tile_groups in (64, 128, 256, 512, 1024):
        for extra in (8, 8 * 3 + 5, 8 * (tile_groups - 1), 8 * (tile_groups - 1) + 7, 8 * tile_groups, 8 * tile_groups + 1):
            n = base + extra
            xd, hd = x_all[:n], h_all[:n]
            nbytes, nmeta = exmy.packed_bytes(n, X, Y), exmy.block_count(n, block)
            pbuf = torch.full((nbytes + 256,), 0x5A, dtype=torch.uint8, device=DEV)
            mbuf = torch.full((nmeta + 256,), 0x5A, dtype=torch.uint8, device=DEV)
            exmy.encode_blocks_auto(xd, block, X, Y, 0, max_exps=mbuf[:nmeta], out=pbuf[:nbytes])
            torch.cuda.synchronize()
            want_meta = O.block_max_exp(hd, block, X)
            want = O.encode_blocks(hd, block, X, Y, want_meta, threads=THREADS)
            p, m = pbuf.cpu().numpy(), mbuf.cpu().numpy()
            assert np.array_equal(m[:nmeta], want_meta), (block, n)
            assert np.array_equal(p[:nbytes], want), (block, n)
            assert (p[nbytes:] == 0x5A).all() and (m[nmeta:] == 0x5A).all(), (block, n)
