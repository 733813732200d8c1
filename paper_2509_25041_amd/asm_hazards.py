"""Build-time check of the hand-written inline assembly in the HIP kernels.

The compiler keeps the hardware's wait states between its own instructions, but it does not see
inside an inline-assembly block.  On gfx950 a vector-memory instruction that reads a scalar register
needs five wait states after a *vector* instruction wrote that register (v_readlane_b32 /
v_readfirstlane_b32 / a v_cmp with a scalar destination: what the compiler emits when it reloads a
spilled scalar or makes a value uniform).  An assembly block whose first memory instruction follows
such a write too closely reads a stale address, which faults the GPU.  This module compiles a source
file to ISA and reports every such place; the assembly blocks carry their own s_nop for it.

A second check covers the loads that such blocks issue into vector registers and that the kernel
waits for much later (after a whole K step): to the compiler the destination holds its value as soon
as the block ends, so nothing but the source's own ordering keeps it from copying, spilling or using
the register before the data has arrived.  find_early_uses follows the instruction stream from every
such load to the next wait on the vector-memory counter and reports any instruction in between that
names a destination register.
"""
from __future__ import annotations

import os
import re
import subprocess
import tempfile
from typing import List

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
WAIT_STATES = 5
_MEM = ("global_", "buffer_", "flat_")


def _sregs(text: str) -> set:
    out = set()
    for m in re.finditer(r"\bs\[(\d+):(\d+)\]|\bs(\d+)\b", text):
        if m.group(1):
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def _cost(instr: str) -> int:
    m = re.match(r"s_nop (\d+)", instr)
    return int(m.group(1)) + 1 if m else 1


def isa_of(source: str) -> List[str]:
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "k.s")
        subprocess.run(["hipcc", "-O3", "-std=c++17", "--offload-arch=gfx950", "-x", "hip", "-Xclang", "-target-feature",
                        "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-I",
                        os.path.join(ROOT, "include"), "-I", CSRC, "-S", "--cuda-device-only", source, "-o", out],
                       check=True, stderr=subprocess.DEVNULL)
        with open(out) as fh:
            return fh.read().splitlines()


def find_hazards(lines: List[str]):
    """-> (number of inline-assembly blocks with memory instructions, list of hazard descriptions)"""
    blocks, found = 0, []
    i = 0
    while i < len(lines):
        if "#ASMSTART" not in lines[i]:
            i += 1
            continue
        j, body = i + 1, []
        while "#ASMEND" not in lines[j]:
            body.append(lines[j].strip())
            j += 1
        mem = [b for b in body if b.startswith(_MEM)]
        if mem:
            blocks += 1
            inside = 0                          # wait states the block provides ahead of its first memory instruction
            for b in body:
                if b.startswith(_MEM):
                    break
                inside += _cost(b)
            used = set()
            for b in mem:
                used |= _sregs(b)
            k, dist = i - 1, inside
            while k >= 0 and dist < WAIT_STATES:
                t = lines[k].strip()
                if t and not t.startswith((";", ".")) and not t.endswith(":"):
                    vector_writes_scalar = t.startswith(("v_readlane_b32", "v_readfirstlane_b32")) or (
                        t.startswith("v_cmp") and t.split(",")[0].split()[-1].startswith("s"))
                    if vector_writes_scalar and _sregs(t.split(",")[0]) & used:
                        found.append(f"line {k + 1}: `{t}` feeds `{mem[0]}` (line {i + 1}) after {dist} wait states")
                    dist += _cost(t)
                k -= 1
        i = j + 1
    return blocks, found


def _vregs(text: str) -> set:
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b", text):
        if m.group(1):
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


_ANYLOAD = re.compile(r"(global|buffer|flat|scratch)_load_")
_LOAD = re.compile(r"(global|buffer|flat)_load_(dword|dwordx2|dwordx3|dwordx4|ubyte|ushort|sbyte|sshort)\b")


def find_early_uses(lines: List[str], limit: int = 60000):
    """-> (number of in-flight loads followed, list of descriptions of too-early register uses)"""
    labels = {ln.strip()[:-1]: n for n, ln in enumerate(lines) if ln.strip().endswith(":") and ln.strip().startswith(".LBB")}
    loads, found = 0, []
    i = 0
    while i < len(lines):
        if "#ASMSTART" not in lines[i]:
            i += 1
            continue
        j, body = i + 1, []
        while "#ASMEND" not in lines[j]:
            body.append(lines[j].strip())
            j += 1
        for bi, b in enumerate(body):
            if not _LOAD.match(b):
                continue
            if any("vmcnt(0)" in later for later in body[bi + 1:]):
                continue                                    # waited for inside the block
            dest = _vregs(b.split(",")[0])
            rest = [x for x in body[bi + 1:] if _vregs(x) & dest]
            if rest:
                found.append(f"line {i + 1}: `{rest[0]}` names the destination of `{b}` in the same block")
            loads += 1
            # every path from the end of the block (both sides of conditional branches) to the first wait
            # that covers the load: s_waitcnt vmcnt(N) leaves at most N operations in flight and loads
            # complete in issue order, so it covers this one once N or more younger loads were issued
            younger0 = sum(1 for x in body[bi + 1:] if _ANYLOAD.match(x))
            todo, seen, steps, hit = [(j + 1, younger0)], set(), 0, None
            while todo and hit is None and steps < limit:
                k, younger = todo.pop()
                while k < len(lines) and steps < limit:
                    if (k, min(younger, 64)) in seen:
                        break
                    seen.add((k, min(younger, 64)))
                    t = lines[k].strip()
                    k += 1
                    if not t or t.startswith((";", ".")) or t.endswith(":") or t.startswith("//"):
                        continue
                    steps += 1
                    if t.startswith("s_endpgm"):
                        break
                    if t.startswith("s_waitcnt") and "vmcnt(" in t:
                        if younger >= int(re.search(r"vmcnt\((\d+)\)", t).group(1)):
                            break
                        continue
                    if t.startswith("s_branch"):
                        k = labels.get(t.split()[-1], len(lines))
                        continue
                    if t.startswith("s_cbranch"):
                        todo.append((labels.get(t.split()[-1], len(lines)), younger))
                        continue
                    if _vregs(t) & dest:
                        hit = f"line {k}: `{t}` names a destination of `{b}` (line {i + 1}) before a wait that covers it"
                        break
                    if _ANYLOAD.match(t):
                        younger += 1
            if hit:
                found.append(hit)
        i = j + 1
    return loads, found


def check(source_name: str = "ffn.hip"):
    return find_hazards(isa_of(os.path.join(CSRC, source_name)))


def check_early_uses(source_name: str = "ffn.hip"):
    return find_early_uses(isa_of(os.path.join(CSRC, source_name)))


if __name__ == "__main__":
    import sys
    n, bad = check(sys.argv[1] if len(sys.argv) > 1 else "ffn.hip")
    print("\n".join(bad))
    print(f"{n} inline-assembly memory blocks checked, {len(bad)} hazards")
    n2, bad2 = check_early_uses(sys.argv[1] if len(sys.argv) > 1 else "ffn.hip")
    print("\n".join(bad2))
    print(f"{n2} loads left in flight by assembly blocks followed, {len(bad2)} early uses")
    sys.exit(1 if bad or bad2 else 0)
