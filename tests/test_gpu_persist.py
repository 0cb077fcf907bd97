"""The decode step's layers as one persistent kernel (up to 64 rows; opt-in, SAPO_PERSIST=1) against the same step as one kernel per phase:
the two run the same arithmetic in the same order, so tokens and log-probs must be identical bit for bit; and a call
must leave no fault mark (a wait that ran into its limit would show as -1 tokens)."""
import contextlib
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


@contextlib.contextmanager
def persistent_kernel():
    os.environ["SAPO_PERSIST"] = "1"
    try:
        yield
    finally:
        os.environ.pop("SAPO_PERSIST", None)


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("shape_name,P,G,Lp,N,temp", [
    ("MINI_BF16", 3, 4, 21, 12, 1.0),          # 12 rows, a partly filled prompt page
    ("MINI_BF16", 8, 8, 32, 24, 0.7),          # the full 64-row tile
    ("MINI_BF16", 1, 2, 200, 70, 1.0),         # long context: several page pairs per wave
    ("MINI_BF16_HD128", 2, 3, 17, 30, 1.0),    # head_dim 128, 6 query heads on one KV head, untied LM head
    ("MINI_BF16", 1, 1, 24, 40, 0.0),          # one row, greedy
])
def test_persistent_step_equals_one_kernel_per_phase(sapo, shape_name, P, G, Lp, N, temp):
    import torch
    shape = getattr(W, shape_name)
    w = W.perturb_norm_gains(W.make_weights(shape, 61, std=0.05), 61)
    gw = sapo.sapo_weights_create(shape, w)
    assert gw.uses_mfma
    prompts = dev(np.random.default_rng(7).integers(0, shape.vocab, size=(P, Lp)).astype(np.int32))
    print("persistent step: %s P %d G %d Lp %d N %d" % (shape_name, P, G, Lp, N), flush=True)
    with persistent_kernel():
        t_p, l_p = sapo.sapo_rollout_generate(gw, prompts, G, N, temp, 99)       # eager launches, persistent kernel
        torch.cuda.synchronize()
        assert sapo.sapo_rollout_last_stats(gw)["steps"] == N - 1
    t_k, l_k = sapo.sapo_rollout_generate(gw, prompts, G, N, temp, 99)
    torch.cuda.synchronize()
    t_p, l_p, t_k, l_k = t_p.cpu().numpy(), l_p.cpu().numpy(), t_k.cpu().numpy(), l_k.cpu().numpy()
    print("   -1 tokens: persistent %d, per-phase %d; first differing step %s" % (
        int((t_p < 0).sum()), int((t_k < 0).sum()),
        (int(np.argwhere((t_p != t_k).any(axis=0))[0][0]) if (t_p != t_k).any() else None)), flush=True)
    assert t_p.min() >= 0 and t_k.min() >= 0, "a decode step reported a fault"
    assert np.array_equal(t_p, t_k)
    assert np.array_equal(l_p.view(np.uint32), l_k.view(np.uint32))
    # the captured step replays the same kernel
    st = torch.cuda.Stream()
    with persistent_kernel(), torch.cuda.stream(st):
        t_g, l_g = sapo.sapo_rollout_generate(gw, prompts, G, N, temp, 99, stream=st)
        st.synchronize()
    assert np.array_equal(t_g.cpu().numpy(), t_p) and np.array_equal(l_g.cpu().numpy().view(np.uint32), l_p.view(np.uint32))
    gw.close()
