"""MI355X (gfx950) eXmY tensor codec: encode / decode / emulate behind a C ABI.

``binding`` wraps the shared library; ``synth`` makes seeded synthetic inputs.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    BF16,
    F16,
    F32,
    Batch,
    ExmyError,
    block_count,
    block_max_exp,
    block_max_exp_after_rounding,
    block_scale,
    decode,
    decode_batch,
    decode_blocks,
    decode_int,
    decode_rows,
    decode_scaled,
    emulate,
    emulate_blocks,
    emulate_int,
    emulate_scaled,
    encode,
    encode_batch,
    encode_blocks,
    encode_blocks_auto,
    encode_int,
    encode_rows,
    encode_scaled,
    encode_with_histogram,
    exponent_histogram,
    max_exp_from_histogram,
    packed_bytes,
    packed_bytes_rows,
)
