"""Check of the hand-placed waits in the fused dK/dV kernel and the few-query cross backward, on the compiler's assembly listing.

    python -m paper_2409_15373_amd.check_lds_waits [source.hip ...]

jfa_bwd_dkv_dma.hip issues its LDS operand reads as explicit instructions several matrix instructions ahead of
their use and waits for them with `s_waitcnt lgkmcnt(n)` counts written by hand.  The compiler does not know that
the destination registers of such a read are pending, so nothing but the source text keeps an instruction from
touching them too early, and a count that is too large makes a matrix instruction read stale registers without any
error.  This module compiles the source to gfx950 assembly (no GPU needed) and scans every kernel in it with a
conservative model of the counter: LDS operations complete in order; a wait for lgkmcnt(n) retires the oldest
pending operations until n are left; scalar loads, which share the counter, are ignored (they only make the real
wait stricter).  It reports every instruction that reads or overwrites a register of a read still pending, and the
deepest queue (the hardware counter has four bits).  The scan is linear in program order: at labels the state is
kept, which is exact for fall-through and conservative for joins in this code (its loops end in lgkmcnt(0)).
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile

from . import build as _build

_REG = re.compile(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b")


def _regs(text: str) -> set:
    out = set()
    for m in _REG.finditer(text):
        if m.group(1) is not None:
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def scan(listing: str) -> dict:
    """Scan an assembly listing; returns counts and the list of violations (line number, instruction, line of the read)."""
    pending = []   # (destination registers, line number), oldest first
    violations = []
    reads = waits = deepest = 0
    for ln, line in enumerate(listing.splitlines(), 1):
        t = line.split(";")[0].strip()
        if not t or t.startswith(".") or t.endswith(":"):
            continue
        op = t.split()[0]
        if op == "s_waitcnt":
            m = re.search(r"lgkmcnt\((\d+)\)", t)
            if m:
                waits += 1
                del pending[:max(0, len(pending) - int(m.group(1)))]
            continue
        used = _regs(t[len(op):])
        for dest, at in pending:
            if dest & used:
                violations.append((ln, t, at))
        if op.startswith("ds_read"):
            pending.append((_regs(t[len(op):].split(",")[0]), ln))
            reads += 1
        elif op.startswith("ds_"):
            pending.append((set(), ln))
        deepest = max(deepest, len(pending))
    return {"lds_reads": reads, "lgkmcnt_waits": waits, "deepest_queue": deepest, "violations": violations}


def behind_partial_vmcnt_wait(listing: str, count: int) -> list:
    """For every hand-written `s_waitcnt vmcnt(count) ...` in the listing: the vector-memory instructions in the program
    text between it and the next s_barrier, as (global -> LDS copies, global stores, anything else).

    The few-query cross backward waits for a block's K and V rows with vmcnt(16): the rows were requested a block ago
    and the only vector-memory instructions issued since are the previous block's stores of dK and dV, which may stay
    in flight.  That is right only if the loop body between two such waits holds exactly `count` store instructions
    (a full block executes them all) and nothing else that the counter counts but the 16 copies of the next block,
    which come first: fewer stores would let the wait pass with copies still in flight, and a scratch access or any
    other load would shift the count.
    """
    lines = listing.splitlines()
    found = []
    for i, line in enumerate(lines):
        if not re.search(r"s_waitcnt\s+vmcnt\(%d\)" % count, line.split(";")[0]):
            continue
        copies = stores = other = 0
        for later in lines[i + 1:]:
            t = later.split(";")[0].strip()
            if not t:
                continue
            op = t.split()[0]
            if op == "s_barrier":
                break
            if op.startswith("global_load_lds"):
                copies += 1
            elif op.startswith("global_store"):
                stores += 1
            elif op.startswith(("global_", "buffer_", "scratch_", "flat_")):
                other += 1
        found.append((copies, stores, other))
    return found


def listing_of(source: str) -> str:
    """The device assembly of one .hip source, compiled with the library's own flags."""
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "kernel.s")
        flags = [f for f in _build.FLAGS if f != "-Wall"]
        r = subprocess.run([_build.HIPCC] + flags + ["-S", "--cuda-device-only", source, "-o", out], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc -S failed for {source}:\n{r.stderr}")
        with open(out) as f:
            return f.read()


def main(argv) -> int:
    sources = argv or [os.path.join(_build.CSRC, "jfa_bwd_dkv_dma.hip")]
    bad = 0
    for src in sources:
        r = scan(listing_of(src))
        print(f"{os.path.basename(src)}: {r['lds_reads']} LDS reads, {r['lgkmcnt_waits']} lgkmcnt waits, deepest queue "
              f"{r['deepest_queue']}, {len(r['violations'])} violations")
        for ln, text, at in r["violations"][:20]:
            print(f"  line {ln}: {text}   touches the registers of the read at line {at}")
        bad += len(r["violations"]) + (r["deepest_queue"] > 15)
    if not argv:
        found = behind_partial_vmcnt_wait(listing_of(os.path.join(_build.CSRC, "jfa_bwd_cross_fewq.hip")), 16)
        print(f"jfa_bwd_cross_fewq.hip: vmcnt(16) waits followed by (copies, stores, other vector-memory instructions) = {found}")
        bad += found != [(16, 16, 0)]
    return 1 if bad else 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
