"""CPU-side checks of the C ABI: the library loads and exports every function the header declares."""
import ctypes
import os
import re

import pytest

from paper_2509_08721_amd import sapo

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sapo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sapo_[a-z_]+)\s*\(", text)))


def test_header_declares_the_two_calls():
    names = declared_functions()
    assert "sapo_rollout_generate" in names and "sapo_score_logprobs" in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(sapo.LIB_PATH):
        from paper_2509_08721_amd import build
        build.build_library(verbose=False)
    lib = ctypes.CDLL(sapo.LIB_PATH)
    for name in declared_functions():
        assert hasattr(lib, name), name
    assert sorted(sapo.EXPORTED) == declared_functions()


def test_binding_has_same_names():
    for name in declared_functions():
        if name in ("sapo_last_error", "sapo_weights_uses_mfma", "sapo_debug_logits_workspace_bytes",
                    "sapo_profile_kernel_count", "sapo_profile_kernel_name"):
            continue
        assert hasattr(sapo, name), name


def test_config_struct_layout():
    assert ctypes.sizeof(sapo.sapo_model_config) == 13 * 4


def test_host_side_argument_validation_needs_no_gpu():
    """Calls that are rejected before any HIP call return error codes and a message."""
    lib = sapo.load_library()
    assert lib.sapo_rollout_workspace_bytes(None, 1, 1, 1, 1) == 0
    assert b"NULL" in lib.sapo_last_error()
    cfg = sapo.sapo_model_config(2, 64, 4, 3, 16, 172, 512, 1e-6, 1e4, 1, 0, 16, 256)
    out = ctypes.c_void_p()
    ptrs = (ctypes.c_void_p * 21)()
    rc = lib.sapo_weights_create(ctypes.byref(cfg), ptrs, 21, None, ctypes.byref(out))
    assert rc == sapo.SAPO_ESHAPE and b"n_kv_heads" in lib.sapo_last_error()
    cfg.n_kv_heads = 2
    rc = lib.sapo_weights_create(ctypes.byref(cfg), ptrs, 20, None, ctypes.byref(out))
    assert rc == sapo.SAPO_EINVAL
    rc = lib.sapo_weights_create(ctypes.byref(cfg), ptrs, 21, None, ctypes.byref(out))
    assert rc == sapo.SAPO_EINVAL and b"tensor 0" in lib.sapo_last_error()
    cfg.kv_page_tokens = 32
    assert lib.sapo_weights_create(ctypes.byref(cfg), ptrs, 21, None, ctypes.byref(out)) == sapo.SAPO_ESHAPE


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: bench.py --gpus N > 1 exits with a message that says so (before anything touches a device)."""
    import subprocess
    import sys
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_node_glue_imports_without_a_gpu():
    from paper_2509_08721_amd import node
    assert hasattr(node, "Node")


def test_boost_token_scales_one_head_row_exactly():
    """workloads.boost_token (input generation for the stop-token workloads): one LM-head row times 2^k, exactly,
    in both storage types, tied or not; everything else untouched, the original left alone."""
    import numpy as np
    from paper_2509_08721_amd import workloads as W
    for shape, key in ((W.MINI_BF16, "embed"), (W.MINI_BF16_HD128, "lm_head"), (W.TINY, "embed" if W.TINY.tied_embeddings else "lm_head")):
        w = W.make_weights(shape, 3, std=0.05)
        before = np.array(w[key], copy=True)
        b = W.boost_token(w, shape, 77, 3)
        assert np.array_equal(w[key], before)                      # a copy, not in place
        to_f = (lambda a: W.bf16_bits_to_f32(a)) if before.dtype == np.uint16 else (lambda a: a.astype(np.float32))
        assert np.array_equal(to_f(b[key][77]), to_f(before[77]) * np.float32(8.0))
        rest = np.ones(before.shape[0], dtype=bool)
        rest[77] = False
        assert np.array_equal(b[key][rest], before[rest])
        for other in ("embed", "lm_head", "final_norm"):
            if other != key and w.get(other) is not None:
                assert b[other] is w[other]
    wl = W.WORKLOADS["onehalfb_stop"]
    assert 0 <= wl.stop_token < wl.shape.vocab and wl.stop_boost > 0 and wl.n_seqs == 256
