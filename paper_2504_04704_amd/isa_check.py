"""Checks the gfx950 assembly of the HIP sources for one hazard the compiler cannot cover.

A vector-memory instruction must not read a scalar register within five wait states of a VECTOR
instruction that wrote it (v_readlane, v_readfirstlane, v_cmp ...: how the compiler brings back a value
it parked in a vector register).  hipcc pads its own instructions, but it does not look into an inline
asm block, and several of this library's loads and stores are issued from such blocks with a scalar
base address.  `scan` finds every asm-block vector-memory instruction that reads a scalar register
written by a vector instruction fewer than five wait states earlier (counted conservatively: a scalar
move that rewrites the register in between does not end the search, exactly as the compiler's own
hazard recogniser counts).

A second rule of the same kind: a store of more than 64 bits reads its data registers over two more
cycles, so a vector-ALU instruction must not overwrite them within two wait states of the store;
`scan_store_data` finds asm-block stores that a vector-ALU write of their data follows too closely.

    python -m paper_2504_04704_amd.isa_check            # compiles the kernel sources and scans them
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor
from typing import List, NamedTuple

from . import build as B

WAIT_STATES = 5
KERNEL_SOURCES = ["split_pass.hip", "hold_pass.hip", "append_pass.hip", "staged_pass.hip"]
_VMEM = re.compile(r"^(global_|buffer_|scratch_|flat_)")
_LABEL = re.compile(r"^(_Z\w+):")


class Site(NamedTuple):
    line: int          # 1-based line of the vector-memory instruction
    function: str
    writer: str        # the vector instruction that wrote the scalar register
    wait_states: int   # wait states between the two
    reader: str


def _scalar_regs(text: str) -> set:
    regs = set()
    for m in re.finditer(r"\bs\[(\d+):(\d+)\]", text):
        regs.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"\bs(\d+)\b", text):
        regs.add(int(m.group(1)))
    if re.search(r"\bvcc\b", text):
        regs.update((106, 107))
    return regs


def _vector_writes(instr: str) -> set:
    """Scalar registers a vector-ALU instruction writes (its first operand; a compare in the short
    encoding writes vcc)."""
    if not instr.startswith("v_"):
        return set()
    parts = instr.split(None, 1)
    if len(parts) < 2:
        return set()
    first = parts[1].split(",")[0]
    regs = _scalar_regs(first)
    if parts[0].startswith("v_cmp") and not parts[0].endswith("_e64") and not regs:
        regs = {106, 107}
    return regs


def scan(asm: str) -> List[Site]:
    sites = []
    function, in_asm = "?", False
    recent = []  # (wait states the instruction provides, scalar registers it writes as a vector op, text)
    for no, raw in enumerate(asm.split("\n"), 1):
        s = raw.strip()
        m = _LABEL.match(s)
        if m:
            function, recent = m.group(1), []
            continue
        if "#ASMSTART" in s:
            in_asm = True
            continue
        if "#ASMEND" in s:
            in_asm = False
            continue
        if not s or s[0] in ";." or s.endswith(":"):
            continue
        if in_asm and _VMEM.match(s):
            reads = _scalar_regs(s)
            waited = 0
            for states, writes, text in reversed(recent):
                if waited >= WAIT_STATES:
                    break
                if writes & reads:
                    sites.append(Site(no, function, text, waited, s))
                    break
                waited += states
        nop = re.match(r"s_nop\s+(\d+)", s)
        recent.append((int(nop.group(1)) + 1 if nop else 1, _vector_writes(s), s))
        del recent[:-16]
    return sites


STORE_DATA_WAIT_STATES = 2
_WIDE_STORE = re.compile(r"^(global|flat|scratch)_store_dwordx[34]\b")


def _vector_regs(text: str) -> set:
    regs = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]", text):
        regs.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"\bv(\d+)\b", text):
        regs.add(int(m.group(1)))
    return regs


def scan_store_data(asm: str) -> List[Site]:
    sites = []
    function, in_asm = "?", False
    pending = []  # (data registers, wait states since the store, text)
    for no, raw in enumerate(asm.split("\n"), 1):
        s = raw.strip()
        m = _LABEL.match(s)
        if m:
            function, pending = m.group(1), []
            continue
        if "#ASMSTART" in s:
            in_asm = True
            continue
        if "#ASMEND" in s:
            in_asm = False
            continue
        if not s or s[0] in ";." or s.endswith(":"):
            continue
        nop = re.match(r"s_nop\s+(\d+)", s)
        states = int(nop.group(1)) + 1 if nop else 1
        written = set()
        if s.startswith("v_"):
            parts = s.split(None, 1)
            written = _vector_regs(parts[1].split(",")[0]) if len(parts) > 1 else set()
        still = []
        for data, waited, text in pending:
            if written & data:
                sites.append(Site(no, function, text, waited, s))
            elif waited + states < STORE_DATA_WAIT_STATES:
                still.append((data, waited + states, text))
        pending = still
        if in_asm and _WIDE_STORE.match(s):
            operands = s.split(None, 1)[1].split(",")
            pending.append((_vector_regs(operands[1]), 0, s))
    return sites


def assembly_of(source: str) -> str:
    """gfx950 assembly of one file of csrc/, with the library's own compile flags."""
    with tempfile.TemporaryDirectory(prefix="lagkv_isa_") as tmp:
        out = os.path.join(tmp, "k.s")
        cmd = [B.hipcc_path(), *B.HIPCC_FLAGS, "-I", os.path.join(B.ROOT, "include"), "-I", B.CSRC,
               "-S", "--cuda-device-only", "-o", out, os.path.join(B.CSRC, source)]
        proc = subprocess.run(cmd, capture_output=True, text=True)
        if proc.returncode != 0:
            raise RuntimeError(f"hipcc failed on {source}\n{proc.stderr}")
        with open(out) as f:
            return f.read()


def check_sources(sources=KERNEL_SOURCES) -> dict:
    with ThreadPoolExecutor(min(len(sources), os.cpu_count() or 1)) as ex:
        def both(src):
            asm = assembly_of(src)
            return scan(asm) + scan_store_data(asm)
        return dict(zip(sources, ex.map(both, sources)))


if __name__ == "__main__":
    bad = 0
    for src, sites in check_sources().items():
        print(f"{src}: {len(sites)} site(s)")
        for st in sites[:10]:
            print(f"  line {st.line} in {st.function}\n    {st.writer}\n    ... {st.wait_states} wait state(s) ...\n    {st.reader}")
        bad += len(sites)
    sys.exit(1 if bad else 0)
