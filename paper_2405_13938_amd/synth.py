"""Seeded synthetic inputs shaped like the workloads of the eXmY codec.

This module only makes input tensors.  It holds none of the codec's arithmetic
and is the one piece of code that both the HIP path's callers and the CPU
oracle's tests use, so that both sides see the same bits.

Each generator draws from ``torch.Generator(device).manual_seed(seed)`` on the
device asked for; the bits are whatever that device's generator gives, and
whoever needs them elsewhere copies them (nothing here promises that CPU and
GPU draws agree).  The paper's own tensors (one PaLM-2 layer, Section 3.1) are
not public; Gaussian weights reproduce the exponent histogram it describes
(counts doubling per binade on the left, a peak, a sharp drop) and stand in.
"""
import math

import torch

# Workload shapes (elements) of the five configurations.
CFG1_N = 1 << 20
CFG2_SHAPE = (8192, 8192)
CFG3_N = 1 << 28
CFG4_SHAPE = (16384, 14336)
CFG5_LAYERS = 32
CFG5_HIDDEN, CFG5_FFN = 4096, 11008

_CHUNK = 1 << 24


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _randn_into(out_flat, gen, transform):
    """Fill ``out_flat`` chunk by chunk with ``transform(chunk_len)`` draws."""
    n = out_flat.numel()
    for a in range(0, n, _CHUNK):
        b = min(n, a + _CHUNK)
        out_flat[a:b] = transform(b - a, gen).to(out_flat.dtype)
    return out_flat


def special_values_f32():
    """The 16 injected fp32 bit patterns of configuration 1."""
    return [
        0x7FC00000,  # quiet NaN
        0x7F800001,  # NaN with only a payload bit (signalling)
        0xFFC12345,  # negative NaN
        0x7F800000,  # +Inf
        0xFF800000,  # -Inf
        0x00000000,  # +0
        0x80000000,  # -0
        0x00000001,  # +min denormal
        0x80000001,  # -min denormal
        0x007FFFFF,  # +max denormal
        0x807FFFFF,  # -max denormal
        0x00800000,  # +FLT_MIN
        0x80800000,  # -FLT_MIN
        0x7F7FFFFF,  # +FLT_MAX
        0xFF7FFFFF,  # -FLT_MAX
        0x3F800000,  # 1.0
    ]


def cfg1(n=CFG1_N, seed=0, device="cpu"):
    """fp32 N(0,1) with 16 special values at seeded positions.

    Returns (tensor, positions of the specials)."""
    g = _gen(seed, device)
    x = torch.empty(n, dtype=torch.float32, device=device)
    _randn_into(x, g, lambda m, gg: torch.randn(m, generator=gg, device=device))
    k = min(16, n)
    pos = torch.randperm(n, generator=g, device=device)[:k]
    vals = torch.tensor(special_values_f32()[:k], dtype=torch.int64, device=device)
    vals = torch.where(vals >= 2 ** 31, vals - 2 ** 32, vals).to(torch.int32)
    x.view(torch.int32)[pos] = vals
    return x, pos


def gaussian_bf16(n, std=0.02, seed=1, device="cpu"):
    """bf16 N(0, std^2): weight-like (configurations 2 and 5)."""
    g = _gen(seed, device)
    x = torch.empty(n, dtype=torch.bfloat16, device=device)
    return _randn_into(x, g, lambda m, gg: torch.randn(m, generator=gg, device=device) * std)


def cfg2(shape=CFG2_SHAPE, seed=1, device="cpu"):
    return gaussian_bf16(shape[0] * shape[1], 0.02, seed, device).view(shape)


def cfg3(n=CFG3_N, seed=2, device="cpu"):
    """fp32 with log-normal magnitudes: log2|x| ~ N(-6, 3^2), random signs."""
    g = _gen(seed, device)
    x = torch.empty(n, dtype=torch.float32, device=device)

    def draw(m, gg):
        z = torch.randn(m, generator=gg, device=device) * 3.0 - 6.0
        s = torch.randint(0, 2, (m,), generator=gg, device=device).to(torch.float32) * 2.0 - 1.0
        return torch.exp2(z) * s

    return _randn_into(x, g, draw)


def cfg4(shape=CFG4_SHAPE, seed=3, device="cpu", outlier_frac=1e-3, outlier=1e4):
    """bf16 activation-like: 0.5 * Student-t(nu=3), a fraction set to +-1e4."""
    g = _gen(seed, device)
    n = shape[0] * shape[1]
    x = torch.empty(n, dtype=torch.bfloat16, device=device)

    def draw(m, gg):
        z = torch.randn(m, generator=gg, device=device)
        chi2 = torch.randn(3, m, generator=gg, device=device).square().sum(0)
        t = 0.5 * z / torch.sqrt(chi2 / 3.0)
        u = torch.rand(m, generator=gg, device=device)
        sgn = torch.randint(0, 2, (m,), generator=gg, device=device).to(torch.float32) * 2.0 - 1.0
        return torch.where(u < outlier_frac, sgn * outlier, t)

    return _randn_into(x, g, draw).view(shape)


def cfg5_shapes(layers=CFG5_LAYERS, hidden=CFG5_HIDDEN, ffn=CFG5_FFN):
    """Tensor shapes of a 7B-class decoder checkpoint, layer by layer."""
    per_layer = [
        ("q", (hidden, hidden)),
        ("k", (hidden, hidden)),
        ("v", (hidden, hidden)),
        ("o", (hidden, hidden)),
        ("gate", (hidden, ffn)),
        ("up", (hidden, ffn)),
        ("down", (ffn, hidden)),
        ("norm1", (hidden,)),
        ("norm2", (hidden,)),
    ]
    return [("layer%d.%s" % (l, name), shape) for l in range(layers) for name, shape in per_layer]


def cfg5(layers=CFG5_LAYERS, hidden=CFG5_HIDDEN, ffn=CFG5_FFN, seed=4, device="cpu"):
    """One flat bf16 N(0, 0.02^2) buffer holding every tensor back to back.

    Returns (flat tensor, [(name, offset_in_elements, numel)])."""
    shapes = cfg5_shapes(layers, hidden, ffn)
    sizes = [math.prod(s) for _, s in shapes]
    flat = gaussian_bf16(sum(sizes), 0.02, seed, device)
    table, off = [], 0
    for (name, _), sz in zip(shapes, sizes):
        table.append((name, off, sz))
        off += sz
    return flat, table


def all_bf16_patterns(device="cpu"):
    """Every one of the 65536 bf16 bit patterns, in order."""
    return torch.arange(0, 65536, dtype=torch.int32, device=device).to(torch.int16).view(torch.bfloat16)


def all_f16_patterns(device="cpu"):
    """Every one of the 65536 fp16 bit patterns, in order."""
    return torch.arange(0, 65536, dtype=torch.int32, device=device).to(torch.int16).view(torch.float16)


def f32_edge_sweep(device="cpu", seed=7, n_random=1 << 16):
    """fp32 bit patterns that stress rounding: every exponent with mantissas at
    and around each tie position, plus random bit patterns."""
    g = _gen(seed, device)
    exps = torch.arange(0, 256, dtype=torch.int64, device=device)
    mants = [0, 1, 2, 3, 0x7FFFFF, 0x7FFFFE, 0x400000, 0x400001, 0x3FFFFF]
    for y in range(0, 23):
        half = 1 << (22 - y)
        for k in (0, 1, 3, (1 << y) - 1 if y else 0):
            base = (k << (23 - y)) & 0x7FFFFF
            for d in (-1, 0, 1):
                mants.append((base + half + d) & 0x7FFFFF)
    m = torch.tensor(sorted(set(mants)), dtype=torch.int64, device=device)
    bits = (exps[:, None] << 23 | m[None, :]).reshape(-1)
    bits = torch.cat([bits, bits | (1 << 31)])
    rnd = torch.randint(0, 2 ** 32, (n_random,), generator=g, device=device, dtype=torch.int64)
    bits = torch.cat([bits, rnd])
    bits = torch.where(bits >= 2 ** 31, bits - 2 ** 32, bits).to(torch.int32)
    return bits.view(torch.float32)


def shuffled(t, seed):
    """The elements of ``t`` (flattened) in a seeded random order, so that
    neighbouring elements (one metadata block) mix magnitudes."""
    t = t.reshape(-1)
    perm = torch.randperm(t.numel(), generator=_gen(seed, "cpu")).to(t.device)
    return t[perm]


def bits_numpy(t):
    """Host numpy view of a tensor's bits in the form the oracle takes:
    float32 for fp32 tensors, uint16 bit patterns for bf16 tensors, float16 for fp16 tensors."""
    t = t.detach().reshape(-1).cpu().contiguous()
    if t.dtype == torch.float32:
        return t.numpy()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view("uint16")
    if t.dtype == torch.float16:
        return t.numpy()
    raise TypeError(t.dtype)
