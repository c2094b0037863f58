"""Seeded random sweep over entry points, formats, metadata and lengths (whole tiles, partial tiles, ragged
groups, sub-views at 16-byte offsets), each case checked bit for bit against the CPU oracle."""
import numpy as np
import pytest
import torch

import paper_2405_13938_amd as exmy
from oracle import exmy_oracle as O
from paper_2405_13938_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ODT = {torch.float32: O.F32, torch.bfloat16: O.BF16, torch.float16: O.F16}
P = {torch.float32: 23, torch.bfloat16: 7, torch.float16: 10}


def ubits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else (a.view(np.uint16) if a.dtype == np.float16 else a)


def tbits(t):
    return ubits(synth.bits_numpy(t))


def same(got, want):
    return np.array_equal(tbits(got), ubits(np.asarray(want)).reshape(-1))


def pick_format(rng, dtype, max_w=16, min_x=0):
    while True:
        X = int(rng.integers(min_x, (5 if dtype == torch.float16 else 7) + 1))
        Y = int(rng.integers(0, min(P[dtype] + (1 if X == 0 else 0), max_w - 1 - X) + 1))
        if 1 <= 1 + X + Y <= max_w and (X, Y) != (0, 0):
            return X, Y


def pick_max_exp(rng, dtype, X, Y):
    for _ in range(100):
        me = int(rng.integers(max((1 << X) - 1, 1), 254 if X else 253)) if dtype != torch.float16 else int(rng.integers(100, 143))
        if O.check_format(ODT[dtype], X, Y, me) == 0:
            return me
    return None


def make_input(rng, dtype, n, pad):
    """n elements at an offset of `pad` 16-byte pieces inside a larger buffer (a view, as callers pass them)."""
    per = 16 // torch.empty(0, dtype=dtype).element_size()
    g = torch.Generator().manual_seed(int(rng.integers(1 << 30)))
    x = torch.randn(n + pad * per, generator=g) * torch.exp2(torch.randint(-14, 14, (n + pad * per,), generator=g).float())
    x[torch.rand(x.numel(), generator=g) < 0.01] = float("inf")
    x[torch.rand(x.numel(), generator=g) < 0.01] = float("nan")
    x[torch.rand(x.numel(), generator=g) < 0.02] = 0.0
    if dtype == torch.float16:
        x = x.clamp(-6e4, 6e4)
    return x.to(dtype).to(DEV)[pad * per :]


LENGTHS = [1, 5, 8, 64, 1000, 1024, 2048, 2056, 4093, 8192, 16384, 16392, 40003, 65536, 131077]


@pytest.mark.parametrize("seed", range(12))
def test_random_cases(seed):
    rng = np.random.default_rng(1000 + seed)
    for case in range(80):
        dtype = [torch.bfloat16, torch.float32, torch.float16][int(rng.integers(3))]
        n = int(rng.choice(LENGTHS)) + int(rng.integers(0, 2)) * int(rng.integers(0, 300))
        x = make_input(rng, dtype, n, int(rng.integers(0, 4)))
        host = synth.bits_numpy(x)
        kind = ["flat", "blocks", "auto", "scaled", "records", "specials", "int", "tiles", "rows"][int(rng.integers(9))]
        tag = (seed, case, kind, str(dtype), n)
        if kind in ("flat", "records"):
            X, Y = pick_format(rng, dtype)
            me = pick_max_exp(rng, dtype, X, Y)
            if me is None:
                continue
            enc, dec = (exmy.encode, exmy.decode) if kind == "flat" else (exmy.encode_records, exmy.decode_records)
            oenc, odec = (O.encode, O.decode) if kind == "flat" else (O.encode_records, O.decode_records)
            want = oenc(host, X, Y, me)
            assert np.array_equal(enc(x, X, Y, me).cpu().numpy(), want), tag + (X, Y, me)
            assert same(dec(torch.from_numpy(want).to(DEV), dtype, n, X, Y, me), odec(want, ODT[dtype], n, X, Y, me)), tag + (X, Y, me)
            assert same(exmy.emulate(x.clone(), X, Y, me), O.emulate(host, X, Y, me)), tag + (X, Y, me)
        elif kind in ("blocks", "auto", "scaled"):
            X, Y = pick_format(rng, dtype)
            if kind == "scaled" and O.check_format(ODT[dtype], X, Y, 127) != 0:
                continue
            if dtype == torch.float16 and pick_max_exp(rng, dtype, X, Y) is None:
                continue
            block = int(rng.choice([8, 16, 32, 64, 128, 24, 520, 1024, 2048, 4096, 5504, 8192, 11008, 22016, 32768, 44032, 65536]))
            if kind == "scaled":
                s = O.block_scale(host, block, X, Y, bf16=bool(rng.integers(2)))
                sd = torch.from_numpy(s.view(np.int16)).view(torch.bfloat16).to(DEV) if s.dtype == np.uint16 else torch.from_numpy(s).to(DEV)
                got_s = exmy.block_scale(x, block, X, Y, scale_dtype=sd.dtype)
                assert torch.equal(got_s.view(torch.int16 if s.dtype == np.uint16 else torch.int32), sd.view(torch.int16 if s.dtype == np.uint16 else torch.int32)), tag
                want = O.encode_scaled(host, block, X, Y, s)
                assert np.array_equal(exmy.encode_scaled(x, block, X, Y, sd).cpu().numpy(), want), tag + (X, Y, block)
                assert same(exmy.decode_scaled(torch.from_numpy(want).to(DEV), dtype, n, block, X, Y, sd), O.decode_scaled(want, ODT[dtype], n, block, X, Y, s)), tag + (X, Y, block)
                assert same(exmy.emulate_scaled(x.clone(), block, X, Y, sd), O.emulate_scaled(host, block, X, Y, s)), tag + (X, Y, block)
                continue
            scheme = int(rng.integers(2))
            meta = O.block_max_exp_after_rounding(host, block, X, Y) if scheme else O.block_max_exp(host, block, X)
            if kind == "auto":
                packed, got_meta = exmy.encode_blocks_auto(x, block, X, Y, scheme)
                want_meta = meta
                if dtype == torch.float16 and not scheme:  # the one-pass call writes bytes valid for (X, Y)
                    lo = 102 + Y if X == 0 else 101 + Y + (1 << X)
                    want_meta = np.clip(meta, lo, 142).astype(np.uint8)
                assert np.array_equal(got_meta.cpu().numpy(), want_meta), tag + (X, Y, block, scheme)
                assert np.array_equal(packed.cpu().numpy(), O.encode_blocks(host, block, X, Y, want_meta)), tag + (X, Y, block, scheme)
                continue
            got_meta = exmy.block_max_exp_after_rounding(x, block, X, Y) if scheme else exmy.block_max_exp(x, block, X)
            assert np.array_equal(got_meta.cpu().numpy(), meta), tag + (X, Y, block, scheme)
            meta = (meta.astype(np.int32) + rng.integers(-2, 3, meta.size)).clip(0, 255).astype(np.uint8)
            md = torch.from_numpy(meta).to(DEV)
            want = O.encode_blocks(host, block, X, Y, meta)
            assert np.array_equal(exmy.encode_blocks(x, block, X, Y, md).cpu().numpy(), want), tag + (X, Y, block)
            assert same(exmy.decode_blocks(torch.from_numpy(want).to(DEV), dtype, n, block, X, Y, md), O.decode_blocks(want, ODT[dtype], n, block, X, Y, meta)), tag + (X, Y, block)
            assert same(exmy.emulate_blocks(x.clone(), block, X, Y, md), O.emulate_blocks(host, block, X, Y, meta)), tag + (X, Y, block)
        elif kind == "specials":
            sp = int(rng.integers(1, 3))
            X, Y = pick_format(rng, dtype, min_x=1 if sp == 1 else 0)
            me = pick_max_exp(rng, dtype, X, Y)
            if me is None:
                continue
            want = O.encode_specials(host, X, Y, me, sp)
            assert np.array_equal(exmy.encode_specials(x, X, Y, me, sp).cpu().numpy(), want), tag + (X, Y, me, sp)
            codes = rng.integers(0, 1 << (1 + X + Y), size=(n + 7) // 8 * 8).astype(np.uint32)
            blob = O.pack(codes, 1 + X + Y)
            assert same(exmy.decode_specials(torch.from_numpy(blob).to(DEV), dtype, n, X, Y, me, sp), O.decode_specials(blob, ODT[dtype], n, X, Y, me, sp)), tag + (X, Y, me, sp)
            assert same(exmy.emulate_specials(x.clone(), X, Y, me, sp), O.emulate_specials(host, X, Y, me, sp)), tag + (X, Y, me, sp)
        elif kind == "int":
            Y = int(rng.integers(1, min(P[dtype] + 1, 15) + 1))
            me = None
            for _ in range(50):
                c = int(rng.integers(90, 160))
                try:
                    O.encode_int(host[:8] if n >= 8 else host, Y, c)
                    me = c
                    break
                except Exception:
                    pass
            if me is None:
                continue
            want = O.encode_int(host, Y, me)
            assert np.array_equal(exmy.encode_int(x, Y, me).cpu().numpy(), want), tag + (Y, me)
            assert same(exmy.decode_int(torch.from_numpy(want).to(DEV), dtype, n, Y, me), O.decode_int(want, ODT[dtype], n, Y, me)), tag + (Y, me)
            assert same(exmy.emulate_int(x.clone(), Y, me), O.emulate_int(host, Y, me)), tag + (Y, me)
        else:  # matrices
            cols = 8 * int(rng.choice([1, 2, 3, 16, 17, 32, 33, 64, 65, 129, 172, 513]))
            if n < cols:
                cols = 8
            if n < cols:
                continue
            rows = n // cols
            m = x[: rows * cols].view(rows, cols)
            hm = host[: rows * cols].reshape(rows, cols)
            X, Y = pick_format(rng, dtype)
            if dtype == torch.float16 and pick_max_exp(rng, dtype, X, Y) is None:
                continue
            if kind == "tiles":
                tr = int(rng.choice([1, 2, 5, 8, 32, 100, 1 << 20]))
                tc = int(rng.choice([1, 8, 16, 24, 64, 1 << 20]))
                scheme = int(rng.integers(2))
                meta = O.tile_max_exp(hm, tr, tc, X, Y, bool(scheme))
                assert np.array_equal(exmy.tile_max_exp(m, tr, tc, X, Y, scheme).cpu().numpy(), meta), tag + (X, Y, rows, cols, tr, tc, scheme)
                meta = (meta.astype(np.int32) + rng.integers(-2, 3, meta.size)).clip(0, 255).astype(np.uint8)
                md = torch.from_numpy(meta).to(DEV)
                want = O.encode_tiles(hm, tr, tc, X, Y, meta)
                assert np.array_equal(exmy.encode_tiles(m, tr, tc, X, Y, md).cpu().numpy(), want), tag + (X, Y, rows, cols, tr, tc)
                assert same(exmy.decode_tiles(torch.from_numpy(want).to(DEV), dtype, rows, cols, tr, tc, X, Y, md), O.decode_tiles(want, ODT[dtype], rows, cols, tr, tc, X, Y, meta)), tag + (X, Y, rows, cols, tr, tc)
                assert same(exmy.emulate_tiles(m.clone(), tr, tc, X, Y, md), O.emulate_tiles(hm, tr, tc, X, Y, meta)), tag + (X, Y, rows, cols, tr, tc)
            else:
                per_row = bool(rng.integers(2))
                me = pick_max_exp(rng, dtype, X, Y)
                if me is None:
                    continue
                meta = O.block_max_exp(hm.reshape(-1), cols, X) if per_row else None
                md = torch.from_numpy(meta).to(DEV) if per_row else None
                want = O.encode_rows(hm.reshape(-1), rows, cols, X, Y, me, meta)
                assert np.array_equal(exmy.encode_rows(m, X, Y, me, md).cpu().numpy(), want), tag + (X, Y, rows, cols, per_row)
                assert same(exmy.decode_rows(torch.from_numpy(want).to(DEV), dtype, rows, cols, X, Y, me, md), O.decode_rows(want, ODT[dtype], rows, cols, X, Y, me, meta)), tag + (X, Y, rows, cols, per_row)
    torch.cuda.synchronize()
