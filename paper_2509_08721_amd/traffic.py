"""HBM-side traffic per kernel launch, from rocprofv3 counter runs.

Two counter runs (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch) of ``bench.py`` give, per kernel
family, the bytes that crossed from the L2s to the memory fabric.  Each counter is scaled by what it
reads for a plain 1 GiB device copy in the same run (``bench.py --copy-probe``).  The table is stored
next to this module together with hashes of the kernel sources; ``lookup`` returns nothing once a
source has changed since the counters were taken.

Build the table (on the machine with the GPU, after the two rocprofv3 runs)::

    python -m paper_2509_08721_amd.traffic WORKLOAD FETCH_counter_collection.csv WRITE_counter_collection.csv "NOTE"
"""
from __future__ import annotations

import csv
import hashlib
import json
import os
import re
import sys
from collections import defaultdict

HERE = os.path.dirname(os.path.abspath(__file__))
TABLE = os.path.join(HERE, "hbm_traffic.json")
COPY_BYTES = 1 << 30

# bench.py's kernel names <- prefixes of the (demangled) kernel names in a trace, and the sources they live in
FAMILIES = {
    "k_gemm_skinny": (("k_skinny16",), ("kernels_decode.hip", "common.h")),
    "k_decode_attention": (("k_decode_attention16",), ("kernels_decode.hip", "common.h")),
    "k_lmhead_sample": (("k_lmhead_sample16", "k_lmhead_sample_big"), ("kernels_decode.hip", "kernels_mfma.hip", "common.h")),
    "k_gemm_big": (("k_gemm_big",), ("kernels_mfma.hip", "common.h")),   # a trace does not tell decode launches apart
    "k_flash_attention": (("k_flash_attention",), ("kernels_mfma.hip", "common.h")),
    "k_lmhead_score": (("k_lmhead_score(", "k_lmhead_score<", "k_lmhead_score"), ("kernels_mfma.hip", "common.h")),
}


def _short(name: str) -> str:
    m = re.match(r"_ZN4sapo(\d+)", name)
    if m:
        n = int(m.group(1))
        return name[m.end():m.end() + n]
    name = name.replace("void ", "")
    name = name.split("(")[0]
    return name.split("::")[-1] if name.startswith("sapo::") else name


def _family(short: str):
    for fam, (prefixes, _) in FAMILIES.items():
        for p in prefixes:
            p = p.rstrip("(<")
            if short == p or short.startswith(p + "<") or short.startswith(p + "("):
                return fam
    return None


def summarise(csv_path: str, counter: str):
    """-> ({family: (launches, mean KiB)}, KiB read for the 1 GiB copy)"""
    tot = defaultdict(float)
    cnt = defaultdict(int)
    copy_max = 0.0
    with open(csv_path) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] != counter:
                continue
            v = float(r["Counter_Value"])
            if "copyBuffer" in r["Kernel_Name"]:
                copy_max = max(copy_max, v)
            fam = _family(_short(r["Kernel_Name"]))
            if fam:
                tot[fam] += v
                cnt[fam] += 1
    return {k: (cnt[k], tot[k] / cnt[k]) for k in tot}, copy_max


def source_hashes(files):
    out = {}
    for fn in sorted(set(files)):
        with open(os.path.join(HERE, "csrc", fn), "rb") as f:
            out[fn] = hashlib.sha256(f.read()).hexdigest()
    return out


def build(workload: str, fetch_csv: str, write_csv: str, note: str) -> dict:
    fetch, fcopy = summarise(fetch_csv, "FETCH_SIZE")
    write, wcopy = summarise(write_csv, "WRITE_SIZE")
    if fcopy <= 0 or wcopy <= 0:
        raise SystemExit("no 1 GiB copy found in the counter files (run bench.py with --copy-probe)")
    fs, ws = (COPY_BYTES / 1024.0) / fcopy, (COPY_BYTES / 1024.0) / wcopy
    table = json.load(open(TABLE)) if os.path.exists(TABLE) else {}
    ent = {"note": note, "fetch_scale": round(fs, 4), "write_scale": round(ws, 4), "kernels": {}}
    for fam in fetch:
        n, fk = fetch[fam]
        wk = write.get(fam, (0, 0.0))[1]
        ent["kernels"][fam] = {
            "launches": n, "fetch_KiB_raw": round(fk, 1), "write_KiB_raw": round(wk, 1),
            "bytes_per_launch": round((fk * fs + wk * ws) * 1024.0),
            "sources": source_hashes(FAMILIES[fam][1]),
        }
    table[workload] = ent
    with open(TABLE, "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)
    return ent


def lookup(workload: str, kernel: str):
    """Bytes per launch for a bench kernel name, or None (no counters, or its sources changed since)."""
    if not os.path.exists(TABLE):
        return None
    ent = json.load(open(TABLE)).get(workload, {}).get("kernels", {}).get(kernel)
    if not ent:
        return None
    if source_hashes(ent["sources"].keys()) != ent["sources"]:
        return None
    return ent["bytes_per_launch"]


if __name__ == "__main__":
    if len(sys.argv) != 5:
        raise SystemExit(__doc__)
    e = build(*sys.argv[1:5])
    print(json.dumps(e, indent=1))
