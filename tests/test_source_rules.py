"""Rules that the HIP sources must keep, checked on their text (no GPU needed).

16-byte buffer stores: a `raw_buffer_store_b128` whose scalar-offset operand was a register was seen to store a
wrong third dword on gfx950 when a VALU write to its data registers followed at once (found by the parity tests
of the encoder: sporadic mismatches in elements 4-5 of a group, gone when the offset moved into the per-lane
operand).  Every such store therefore goes through `store16`, which passes a literal 0 there."""
import os
import re

CSRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2405_13938_amd", "csrc")


def sources():
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".hip", ".hpp")):
            with open(os.path.join(CSRC, name)) as f:
                yield name, f.read()


def call_arguments(text, start):
    """Top-level arguments of the call whose opening parenthesis is at text[start]."""
    depth, args, cur = 0, [], ""
    for ch in text[start:]:
        if ch in "([{<" and not (ch == "<" and depth == 0):
            depth += 1
        elif ch in ")]}>" and not (ch == ">" and depth == 0):
            depth -= 1
            if depth == 0:
                args.append(cur.strip())
                return args
        if ch == "," and depth == 1:
            args.append(cur.strip())
            cur = ""
        elif depth >= 1 and not (depth == 1 and ch == "(" and not cur and not args):
            cur += ch
    raise AssertionError("unbalanced call")


def test_every_16_byte_buffer_store_has_a_zero_scalar_offset():
    seen = 0
    for name, text in sources():
        for m in re.finditer(r"__builtin_amdgcn_raw_buffer_store_b128\s*\(", text):
            args = call_arguments(text, m.end() - 1)
            assert len(args) == 5, (name, args)
            # (data, resource, per-lane offset, scalar offset, cache policy)
            assert args[3] == "0", "%s: 16-byte buffer store with scalar offset %r" % (name, args[3])
            seen += 1
    assert seen >= 1


def test_16_byte_buffer_stores_are_made_in_one_place():
    users = [name for name, text in sources() if "__builtin_amdgcn_raw_buffer_store_b128" in text]
    assert users == ["exmy_common.hpp"], users  # store16 is the one caller


def test_no_packed_fp32_instructions_by_hand():
    for name, text in sources():
        assert not re.search(r"v_pk_(add|mul|fma)_f32", text), name
