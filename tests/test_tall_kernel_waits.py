"""Compile-time check of the hand-counted waits in the projection kernel for 129..256 rows.

The kernel loads its activations straight into LDS with inline-assembly instructions the compiler
does not track, and waits for them with explicit `s_waitcnt vmcnt(N)`: "at most N loads
outstanding" proves the activation loads have landed only if exactly N ordinary loads were issued
after them.  That is a property of the generated code (the compiler may drop or move loads: it
once dropped dead weight loads in a peeled loop tail and the wait became too weak), so this test
compiles the kernel to assembly and counts, for every explicit wait in every instance."""
import os
import re
import shutil
import subprocess

import pytest

CSRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2410_20488_amd", "csrc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Wno-pass-failed", "-S", "--cuda-device-only"]


def _functions(asm: str):
    """Yield (name, lines) of every k_gemm_tall instance in the assembly text."""
    cur, name = None, None
    for line in asm.splitlines():
        m = re.match(r"^(_ZN4firp11k_gemm_tall\w+):", line)
        if m:
            name, cur = m.group(1), []
        elif cur is not None:
            cur.append(line.strip())
            if line.strip().startswith("s_endpgm"):
                yield name, cur
                cur = None


def _events(lines):
    """The instruction stream reduced to what the waits depend on: 'dma' (a load into LDS), 'ld' (an
    ordinary vector load), ('wait', N) (an explicit wait: an s_waitcnt vmcnt inside an inline-assembly block)."""
    out, in_asm = [], False
    for l in lines:
        if l.startswith(";;#ASMSTART"):
            in_asm = True
        elif l.startswith(";;#ASMEND"):
            in_asm = False
        elif l.startswith("global_load_lds"):
            out.append("dma")
        elif re.match(r"(global|buffer|scratch|flat)_load", l):
            out.append("ld")
        elif in_asm:
            m = re.match(r"s_waitcnt vmcnt\((\d+)\)", l)
            if m:
                out.append(("wait", int(m.group(1))))
    return out


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_explicit_waits_match_the_loads_issued_after_the_lds_loads():
    r = subprocess.run(["hipcc", *FLAGS, os.path.join(CSRC, "gemm_tall.hip"), "-o", "-"], capture_output=True, text=True,
                       timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    seen = 0
    for name, lines in _functions(r.stdout):
        seen += 1
        # the inner loop: from its header label to the branch back to it
        head = next(i for i, l in enumerate(lines) if "Inner Loop Header" in l)
        label = lines[head].split(":")[0]
        back = max(i for i, l in enumerate(lines) if re.match(r"s_(branch|cbranch_\w+) " + re.escape(label) + r"$", l))
        prologue, body, rest = lines[:head], lines[head:back + 1], lines[back + 1:]
        # prologue then two trips through the loop, then what follows it
        stream = _events(prologue) + _events(body) * 2 + _events(rest)
        since, have_dma, waits = 0, False, 0
        for e in stream:
            if e == "dma":
                have_dma, since = True, 0
            elif e == "ld":
                since += 1
            elif have_dma:
                n = e[1]
                waits += 1
                # a wait for "everything" is always enough; otherwise the count must be exact
                assert n == 0 or n == since, f"{name}: explicit vmcnt({n}) with {since} loads issued after the last LDS load"
        assert waits >= 4, name
        # no peeled copy of the loop body: every LDS load outside the prologue sits inside the loop
        assert not any(e == "dma" for e in _events(rest)), f"{name}: LDS loads after the loop (a peeled tail)"
    assert seen == 4
