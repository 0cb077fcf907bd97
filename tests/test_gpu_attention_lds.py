"""Decode attention with K/V staged through LDS (SAPO_ATTN_LDS=1, the measured alternative) against the default
register-direct reads: the same requests and the same arithmetic, so tokens and log-probs are bit-identical."""
import os

import numpy as np
import pytest

from paper_2509_08721_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sapo():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2509_08721_amd import sapo as binding
    binding.load_library()
    return binding


@pytest.mark.parametrize("shape_name,P,G,Lp,N", [
    ("MINI_BF16", 3, 4, 21, 40),      # partial prompt page, one or two page pairs per sequence
    ("MINI_BF16", 1, 2, 300, 70),     # 10..12 page pairs: both slots of some waves in use
    ("MINI_BF16", 8, 8, 32, 12),      # the full 64-row decode tile
    ("HALF_B", 1, 2, 540, 8),         # 17..18 page pairs over 8 waves: a wave's slots are filled a second time
])
def test_lds_staged_attention_is_bit_identical(sapo, shape_name, P, G, Lp, N):
    import torch
    shape = getattr(W, shape_name)
    weights = W.perturb_norm_gains(W.make_weights(shape, 61, std=0.05 if shape_name.startswith("MINI") else 0.02), 61)
    prompts = torch.from_numpy(np.random.default_rng(5).integers(0, shape.vocab, size=(P, Lp)).astype(np.int32)).cuda()

    def run():
        gw = sapo.sapo_weights_create(shape, weights)      # a fresh handle: the decode step is captured per handle
        assert gw.uses_mfma
        t, l = sapo.sapo_rollout_generate(gw, prompts, G, N, 1.0, 77)
        torch.cuda.synchronize()
        out = t.cpu().numpy(), l.cpu().numpy()
        gw.close()
        return out

    t0, l0 = run()
    os.environ["SAPO_ATTN_LDS"] = "1"
    try:
        t1, l1 = run()
    finally:
        os.environ.pop("SAPO_ATTN_LDS", None)
    assert t0.min() >= 0
    assert np.array_equal(t0, t1) and np.array_equal(l0, l1)
