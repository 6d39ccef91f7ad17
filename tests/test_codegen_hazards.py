"""Static check of the generated gfx950 code: a 16 x 16 x 16 MFMA that accumulates onto the result of a
16 x 16 x 32 MFMA (or the other way round) must sit enough wait states behind it.  The compiler leaves too
few (wrong sums on the GPU); the kernels add them with mfma_shape_change(), and this test fails if a change
of the source or of the flags loses them."""
import re

import pytest

from paper_2408_12588_amd import build as pab_build

MIN_WAIT_STATES = 10
MFMA = re.compile(r"^\s*v_mfma_f32_16x16x(16|32)_bf16\s+(\S+),\s*(\S+),\s*(\S+),\s*(\S+)")


def _regs(operand):
    m = re.match(r"[va]\[(\d+):(\d+)\]", operand)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"[va](\d+)$", operand)
    return {int(m.group(1))} if m else set()


def shape_change_distances(asm_text):
    """(function, line, states) for every MFMA whose C operand was written by an MFMA of the other depth;
    states = instructions in between, an s_nop N counting N + 1."""
    found, func, state, writers = [], None, 0, []   # writers: (registers, depth, state at issue)
    for ln, line in enumerate(asm_text.splitlines(), 1):
        text = line.split(";")[0].rstrip()
        if not text.strip():
            continue
        head = re.match(r"^(\w+):", text)
        if head and not text.startswith("."):
            func, state, writers = head.group(1), 0, []
            continue
        if not text.startswith(("\t", " ")) or text.strip().startswith("."):
            continue
        ins = text.strip()
        m = MFMA.match(text)
        if m:
            depth, dst, c = int(m.group(1)), _regs(m.group(2)), _regs(m.group(5))
            for regs, d, at in writers:
                if d != depth and regs & c:
                    found.append((func, ln, state - at - 1))
            writers = [w for w in writers if not (w[0] & dst)] + [(dst, depth, state)]
            state += 1
            continue
        nop = re.match(r"s_nop\s+(\d+)", ins)
        state += int(nop.group(1)) + 1 if nop else 1
        if not ins.startswith(("s_", "ds_", "global_", "buffer_")):      # a VALU write ends the chain
            out = _regs(ins.split()[1].rstrip(",")) if len(ins.split()) > 1 else set()
            writers = [w for w in writers if not (w[0] & out)]
    return found


def test_parser_sees_a_short_chain():
    asm = "\n".join(["kern:",
                     "\tv_mfma_f32_16x16x32_bf16 v[0:3], v[8:11], v[12:15], v[0:3]",
                     "\ts_nop 2",
                     "\tv_mfma_f32_16x16x16_bf16 v[0:3], v[8:9], v[12:13], v[0:3]",
                     "\ts_nop 7", "\ts_nop 1",
                     "\tv_mfma_f32_16x16x32_bf16 v[4:7], v[8:11], v[12:15], v[0:3]"])
    assert shape_change_distances(asm) == [("kern", 4, 3), ("kern", 7, 10)]


def test_wait_states_between_mfma_shapes(tmp_path):
    path = pab_build.device_asm(str(tmp_path / "pab.s"))
    chains = shape_change_distances(open(path).read())
    assert chains, "the D = 72 kernels chain a 16-column step onto 32-column steps; none found"
    short = [c for c in chains if c[2] < MIN_WAIT_STATES]
    assert not short, "MFMA shape change with too few wait states: %s" % short[:5]
