"""Check of the generated gfx950 code for one miscompilation pattern.

Matrix-core (MFMA) instructions ignore the lane mask.  When an MFMA is guarded by a condition the compiler takes for
lane-dependent, the guard becomes `s_and_saveexec` (mask the lanes) followed by `s_cbranch_execz` (skip the block when
no lane is left); for short blocks the compiler may drop that branch, because ordinary vector instructions do
nothing under an empty mask - an MFMA still runs, on whatever the registers hold.  The kernels avoid lane-dependent
guards around MFMAs (the wave index is read as a scalar); this check makes sure the compiler agreed: every MFMA that
follows a `saveexec` inside the same masked region must have a branch on the mask in front of it.

    python -m paper_2509_08721_amd.isa_check        # compiles every source of the library to assembly and checks it

A second scan is a report, not a pass/fail check (`--waits`): one counter covers a wave's loads and stores and they
retire in issue order, so a wait for a loaded value that was requested behind a store also waits for that store's
acknowledgement - a memory round trip in the middle of an epilogue.  `waits_behind_stores` lists the waits that
allow fewer outstanding operations than there are stores issued before them in program order (a linear scan: it does
not follow branches, so it over-reports where a store and the wait sit on different paths).

    python -m paper_2509_08721_amd.isa_check --waits
"""
from __future__ import annotations

import concurrent.futures as cf
import os
import re
import subprocess
import sys
import tempfile

from . import build as B


def unguarded_mfmas(asm_text: str):
    """[(function, line number, instruction)] of MFMAs reached after a saveexec with no branch on the mask between."""
    out = []
    fn = None
    pending = None          # line of a saveexec whose masked region has not yet seen a branch on exec or the mask's restore
    for i, raw in enumerate(asm_text.splitlines(), 1):
        line = raw.split(";")[0].strip()
        if not line:
            continue
        m = re.match(r"^(_Z\w+|\w+):$", line)
        if m and not line.startswith(".L"):
            fn, pending = m.group(1), None
            continue
        if line.startswith("."):        # local labels and directives: a label does not end the masked region
            continue
        op = line.split()[0]
        if re.match(r"s_(and|andn2|or|xor|nand|nor|xnor|orn2)_saveexec_b64", op):
            pending = i
        elif op.startswith("s_cbranch_exec") or (op in ("s_or_b64", "s_mov_b64", "s_andn2_b64", "s_xor_b64") and
                                                 re.match(r"^\S+\s+exec\b", line)):
            pending = None
        elif op.startswith("s_cbranch") or op in ("s_branch", "s_endpgm", "s_setpc_b64"):
            pending = None
        elif op.startswith("v_mfma") or op.startswith("v_smfmac"):
            if pending is not None:
                out.append((fn, i, line))
    return out


def waits_behind_stores(asm_text: str):
    """{function: [(line number, allowed outstanding, stores issued before in program order)]}."""
    out = {}
    fn, pending = None, 0
    for i, raw in enumerate(asm_text.splitlines(), 1):
        line = raw.split(";")[0].strip()
        if not line:
            continue
        m = re.match(r"^(_Z\w+):$", line)
        if m:
            fn, pending = m.group(1), 0
            continue
        if fn is None or line.startswith("."):
            continue
        op = line.split()[0]
        if op == "s_endpgm":
            pending = 0
        elif re.match(r"(global|buffer|scratch|flat)_(store|atomic)", op):
            pending += 1
        elif op == "s_waitcnt":
            m = re.search(r"vmcnt\((\d+)\)", line)
            if m:
                n = int(m.group(1))
                if pending > n:
                    out.setdefault(fn, []).append((i, n, pending))
                pending = min(pending, n)
    return out


def assemble(src: str, tmp: str) -> str:
    """The gfx950 assembly of one source of the library."""
    flags = [f for f in B.FLAGS if f not in ("-fPIC",)] + ["--cuda-device-only", "-S"]
    out = os.path.join(tmp, src.replace(".hip", ".s"))
    B._run([B._hipcc()] + flags + [os.path.join(B.CSRC, src), "-o", out])
    with open(out) as f:
        return f.read()


def check_sources(verbose: bool = True):
    hipcc = B._hipcc()
    flags = [f for f in B.FLAGS if f not in ("-fPIC",)] + ["--cuda-device-only", "-S"]
    bad = []
    with tempfile.TemporaryDirectory() as tmp:
        def one(src):
            out = os.path.join(tmp, src.replace(".hip", ".s"))
            B._run([hipcc] + flags + [os.path.join(B.CSRC, src), "-o", out])
            with open(out) as f:
                return src, unguarded_mfmas(f.read())
        with cf.ThreadPoolExecutor(max_workers=min(8, len(B.SOURCES))) as ex:
            for src, found in ex.map(one, B.SOURCES):
                if verbose:
                    print("%-22s %s" % (src, "ok" if not found else "%d MFMA(s) under a lane mask without a branch" % len(found)))
                bad += [(src,) + f for f in found]
    return bad


if __name__ == "__main__":
    if "--waits" in sys.argv[1:]:
        with tempfile.TemporaryDirectory() as tmp:
            for src in B.SOURCES:
                for fn, found in sorted(waits_behind_stores(assemble(src, tmp)).items()):
                    print("%-22s %-70s %3d wait(s) behind stores, first at line %d (vmcnt(%d), %d stores before)" % (
                        (src, fn[:70], len(found)) + found[0]))
        sys.exit(0)
    problems = check_sources()
    for p in problems[:20]:
        print("  %s: %s line %d: %s" % p)
    sys.exit(1 if problems else 0)
