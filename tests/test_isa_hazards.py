"""Inline-assembly memory instructions and the hazards the compiler cannot see.

The kernels with a hand-kept memory schedule issue their loads from inline assembly.  The compiler's hazard handling
does not look inside such a statement: a memory instruction in it that reads a scalar register (its base address, or
m0 for a load that goes straight into LDS) right after a vector-ALU instruction wrote that register needs wait states
the compiler will not insert.  The helpers therefore start every such statement with five wait states (s_nop 4), and
this test compiles the sources that use them to assembly and checks every statement: each one that holds a memory
instruction has the wait states in front of it inside the statement, writes m0 from a scalar register only, and takes
its base from scalar registers.
"""
import re
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

import pytest

from paper_1502_03409_amd import build as B

SOURCES = ["lc_forward.hip", "lc_backward_data.hip", "lc_backward_weights.hip"]


def _assembly(src: Path, out: Path) -> str:
    flags = [f for f in B.FLAGS if not f.startswith("-W")]
    cmd = [B.HIPCC, *flags, "--cuda-device-only", "-S", str(src), "-o", str(out)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    return out.read_text()


def _blocks(text):
    lines = text.split("\n")
    i = 0
    while i < len(lines):
        if "ASMSTART" in lines[i]:
            j, body = i + 1, []
            while "ASMEND" not in lines[j]:
                body.append(lines[j].strip())
                j += 1
            yield [l.strip() for l in lines[max(0, i - 8):i]], body
            i = j
        i += 1


def test_inline_assembly_loads_carry_their_wait_states():
    with tempfile.TemporaryDirectory() as d:
        with ThreadPoolExecutor(max_workers=3) as ex:
            texts = list(ex.map(lambda s: _assembly(B.CSRC / s, Path(d) / (s + ".s")), SOURCES))
    n_mem = 0
    for name, text in zip(SOURCES, texts):
        for prev, body in _blocks(text):
            mem = [k for k, b in enumerate(body) if b.startswith(("global_load", "global_store", "buffer_"))]
            if not mem:
                continue
            n_mem += 1
            k = mem[0]
            assert len(mem) == 1, (name, body)
            # five wait states directly in front of the memory instruction, inside the statement
            assert k >= 1 and body[k - 1] == "s_nop 4", (name, body)
            # the base is a pair of scalar registers; an LDS-direct load sets m0 from a scalar register first
            assert re.search(r"s\[\d+:\d+\]$", body[k]), (name, body)
            if "_lds_" in body[k]:
                assert re.fullmatch(r"s_mov_b32 m0, s\d+", body[0]), (name, body)
    assert n_mem > 100      # the three kernels are there, with their unrolled loads
