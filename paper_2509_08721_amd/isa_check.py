"""Check of the generated gfx950 code for one miscompilation pattern.

Matrix-core (MFMA) instructions ignore the lane mask.  When an MFMA is guarded by a condition the compiler takes for
lane-dependent, the guard becomes `s_and_saveexec` (mask the lanes) followed by `s_cbranch_execz` (skip the block when
no lane is left); for short blocks the compiler may drop that branch, because ordinary vector instructions do
nothing under an empty mask - an MFMA still runs, on whatever the registers hold.  The kernels avoid lane-dependent
guards around MFMAs (the wave index is read as a scalar); this check makes sure the compiler agreed: every MFMA that
follows a `saveexec` inside the same masked region must have a branch on the mask in front of it.

    python -m paper_2509_08721_amd.isa_check        # compiles every source of the library to assembly and checks it
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
    problems = check_sources()
    for p in problems[:20]:
        print("  %s: %s line %d: %s" % p)
    sys.exit(1 if problems else 0)
