"""Where the time of the persistent decode kernel goes, phase by phase (diagnostic).

Needs the diagnostic build of the library:

    SAPO_PERSIST_TRACE=1 python -m paper_2509_08721_amd.build
    SAPO_PERSIST=1 python -m paper_2509_08721_amd.persist_trace [workload] [new tokens]

Prints, per phase type of a layer and averaged over workgroups and phases: the time from one report to the next, the
part spent waiting for the previous phase, the part spent in the report itself, and the rest (weight requests, operand
loads, matrix products, reduction, epilogue), next to the step time of the same call."""
from __future__ import annotations

import ctypes as C
import os
import sys

import numpy as np


def main():
    import torch
    from . import sapo, workloads as W
    name = sys.argv[1] if len(sys.argv) > 1 else "halfb_rollout"
    n_new = int(sys.argv[2]) if len(sys.argv) > 2 else 64
    assert os.environ.get("SAPO_PERSIST") == "1", "set SAPO_PERSIST=1: the persistent kernel is opt-in"
    wl = W.WORKLOADS[name]
    gw = sapo.sapo_weights_create(wl.shape, W.make_weights(wl.shape, wl.weight_seed))
    prompts = torch.from_numpy(W.make_prompts(wl)).cuda()
    lib = sapo.load_library()
    if not hasattr(lib, "sapo_debug_persist_trace"):
        raise SystemExit("the library was not built with SAPO_PERSIST_TRACE=1")
    buf = (C.c_ulonglong * (256 * 5 * 4))()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        sapo.sapo_rollout_generate(gw, prompts, wl.group, n_new, wl.temperature, 1, stream=st)
        st.synchronize()
        lib.sapo_debug_persist_trace(buf, 1)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        sapo.sapo_rollout_generate(gw, prompts, wl.group, n_new, wl.temperature, 2, stream=st)
        e1.record(st)
        st.synchronize()
        lib.sapo_debug_persist_trace(buf, 0)
    ms = e0.elapsed_time(e1)
    print("%s: %d sequences, %d new tokens in %.2f ms (prefill included): %.1f us per step" % (
        name, wl.n_prompts * wl.group, n_new, ms, ms * 1e3 / n_new))
    t = np.frombuffer(buf, dtype=np.uint64).reshape(256, 5, 4).astype(np.float64)
    print("phases counted per type and workgroup: %d" % int(t[0, 0, 3]))
    layer = 0.0
    for k, phase in enumerate(("qkv", "attention", "o", "gate/up", "down")):
        n = np.maximum(t[:, k, 3], 1)
        tot, wait, rep = t[:, k, 0] / n * 0.01, t[:, k, 1] / n * 0.01, t[:, k, 2] / n * 0.01
        rest = tot - wait - rep
        layer += tot.mean()
        print("%-10s us per phase: total %.2f | wait mean %.2f min %.2f max %.2f | report %.2f | rest mean %.2f max %.2f" % (
            phase, tot.mean(), wait.mean(), wait.min(), wait.max(), rep.mean(), rest.mean(), rest.max()))
    print("sum over a layer's phases: %.1f us" % layer)


if __name__ == "__main__":
    main()
