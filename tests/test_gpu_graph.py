"""The entry points allocate nothing and clear nothing, so a stream that is being captured
into a HIP graph can take them: every replay must equal the eager result on the data then
in the buffers."""
import numpy as np
import pytest
import torch

import paper_2405_13938_amd as exmy
from oracle import exmy_oracle as O
from paper_2405_13938_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def test_codec_calls_inside_a_captured_graph():
    X, Y, me, block = 3, 3, 125, 64
    sizes = [4096, 12345, 1 << 16, (1 << 18) + 7]
    xs = [synth.gaussian_bf16(n, seed=70 + i).to(DEV) for i, n in enumerate(sizes)]
    packs = [torch.empty(exmy.packed_bytes(n, X, Y), dtype=torch.uint8, device=DEV) for n in sizes]
    outs = [torch.empty_like(x) for x in xs]
    enc = exmy.Batch(xs, packs, [me] * len(xs), X, Y, decode=False)
    dec = exmy.Batch(outs, packs, [me] * len(xs), X, Y, decode=True)
    big = xs[-1]
    meta = torch.empty(exmy.block_count(big.numel(), block), dtype=torch.uint8, device=DEV)
    bpack = torch.empty(exmy.packed_bytes(big.numel(), X, Y), dtype=torch.uint8, device=DEV)
    bout = torch.empty_like(big)
    emu = torch.empty_like(big)
    mat = xs[2].view(256, 256)  # blocks that are parts of columns: the metadata is cleared and then folded into
    tmeta = torch.empty(exmy.tile_count(256, 256, 64, 1), dtype=torch.uint8, device=DEV)
    tpack = torch.empty(exmy.packed_bytes(mat.numel(), X, Y), dtype=torch.uint8, device=DEV)
    tout = torch.empty_like(mat)

    def work():
        enc.run()
        dec.run()
        exmy.encode_blocks_auto(big, block, X, Y, 0, meta, out=bpack)
        exmy.decode_blocks(bpack, torch.bfloat16, big.numel(), block, X, Y, meta, out=bout)
        emu.copy_(big)
        exmy.emulate(emu, X, Y, me)
        exmy.tile_max_exp(mat, 64, 1, X, out=tmeta)
        exmy.encode_tiles(mat, 64, 1, X, Y, tmeta, out=tpack)
        exmy.decode_tiles(tpack, torch.bfloat16, 256, 256, 64, 1, X, Y, tmeta, out=tout)

    work()  # eager once: loads the kernels outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            work()
    torch.cuda.synchronize()

    for replay in range(3):
        # new contents in the same buffers, eager work of our own in between
        for i, x in enumerate(xs):
            x.copy_(synth.gaussian_bf16(x.numel(), std=0.02 * (replay + 1), seed=100 * replay + i).to(DEV))
        for t in packs + outs + [bpack, bout, emu, meta, tpack, tout]:
            t.zero_()
        tmeta.fill_(255)  # stale maxima must not survive the replay
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for x, p, o in zip(xs, packs, outs):
            host = synth.bits_numpy(x)
            want = O.encode(host, X, Y, me)
            assert np.array_equal(p.cpu().numpy(), want), replay
            assert np.array_equal(synth.bits_numpy(o), O.decode(want, O.BF16, x.numel(), X, Y, me)), replay
        host = synth.bits_numpy(big)
        want_meta = O.block_max_exp(host, block, X)
        assert np.array_equal(meta.cpu().numpy(), want_meta), replay
        want = O.encode_blocks(host, block, X, Y, want_meta)
        assert np.array_equal(bpack.cpu().numpy(), want), replay
        assert np.array_equal(synth.bits_numpy(bout), O.decode_blocks(want, O.BF16, big.numel(), block, X, Y, want_meta)), replay
        assert np.array_equal(synth.bits_numpy(emu), O.emulate(host, X, Y, me)), replay
        host = synth.bits_numpy(mat).reshape(256, 256)
        want_meta = O.tile_max_exp(host, 64, 1, X)
        assert np.array_equal(tmeta.cpu().numpy(), want_meta), replay
        want = O.encode_tiles(host, 64, 1, X, Y, want_meta)
        assert np.array_equal(tpack.cpu().numpy(), want), replay
        assert np.array_equal(synth.bits_numpy(tout), O.decode_tiles(want, O.BF16, 256, 256, 64, 1, X, Y, want_meta).reshape(-1)), replay
