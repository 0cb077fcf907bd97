"""Decode attention that reads a prompt's full pages once per group of siblings (one launch with two kinds of
workgroups; a measured alternative, off unless SAPO_SHARE_PREFIX_MIN_PAIRS gives the number of shared page pairs
from which to use it):
against the oracle like every rollout, against the plain attention (same definition, another summation order),
eager launches against the replayed graph, and that the variant is the one that ran."""
import os

import numpy as np
import pytest

from oracle import sapo_oracle as O
from paper_2509_08721_amd import workloads as W
from tests.parity import measured_logit_eps, oracle_logprobs_for, teacher_forced_token_check

pytestmark = pytest.mark.gpu

LOGIT_TOL = 5e-2
LOGPROB_TOL = 2e-2
NEAR_TIE = 1e-3


@pytest.fixture(scope="module")
def sapo():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2509_08721_amd import sapo as binding
    binding.load_library()
    return binding


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


class min_pairs:
    def __init__(self, n):
        self.n = n

    def __enter__(self):
        os.environ["SAPO_SHARE_PREFIX_MIN_PAIRS"] = str(self.n)

    def __exit__(self, *a):
        os.environ.pop("SAPO_SHARE_PREFIX_MIN_PAIRS", None)


def rollout(sapo, shape, weights, prompts, G, N, temp, seed, threshold, profile=False, stream=None):
    import torch
    with min_pairs(threshold):
        gw = sapo.sapo_weights_create(shape, weights)          # a fresh handle: the decode step is captured per handle
        if profile:
            sapo.sapo_profile_start()
        if stream is None:
            t, l = sapo.sapo_rollout_generate(gw, dev(prompts), G, N, temp, seed)
        else:
            with torch.cuda.stream(stream):
                t, l = sapo.sapo_rollout_generate(gw, dev(prompts), G, N, temp, seed, stream=stream)
                stream.synchronize()
        torch.cuda.synchronize()
        prof = sapo.sapo_profile_stop() if profile else None
        out = t.cpu().numpy(), l.cpu().numpy()
        gw.close()
    return out + (prof,)


@pytest.mark.parametrize("shape_name,P,G,Lp,N,temp", [
    ("MINI_BF16", 3, 4, 70, 30, 1.0),      # 2 shared pairs, an odd number of full prompt pages, a partial page
    ("MINI_BF16", 1, 8, 300, 40, 1.0),     # 9 shared pairs over 8 waves: one wave takes two
    ("MINI_BF16", 8, 8, 64, 12, 0.7),      # the full 64-row decode tile; 2 shared pairs
    ("MINI_BF16", 2, 32, 32, 6, 1.0),      # 64 columns: every column of the four tiles in use
    ("HALF_B", 2, 8, 256, 6, 1.0),         # 7 query heads per KV head x 8 siblings = 56 columns; 8 shared pairs
])
def test_shared_prompt_attention(sapo, shape_name, P, G, Lp, N, temp):
    import torch
    shape = getattr(W, shape_name)
    mini = shape_name.startswith("MINI")
    weights = W.perturb_norm_gains(W.make_weights(shape, 141, std=0.05 if mini else 0.02), 141)
    prompts = np.random.default_rng(P * 10 + G).integers(0, shape.vocab, size=(P, Lp)).astype(np.int32)
    threshold = 1 if mini else 8
    t_s, l_s, prof = rollout(sapo, shape, weights, prompts, G, N, temp, 55, threshold, profile=True)
    steps = N - 1
    assert prof["k_decode_attention_shared"][1] == steps * shape.n_layers and "k_decode_attention" not in prof
    t_p, l_p, prof_p = rollout(sapo, shape, weights, prompts, G, N, temp, 55, 0, profile=True)
    assert prof_p["k_decode_attention"][1] == steps * shape.n_layers and "k_decode_attention_shared" not in prof_p
    assert t_s.min() >= 0 and t_s.max() < shape.vocab
    # the two attentions compute the same thing in another order; their half-rounded outputs differ in the last bit
    # here and there, which 24 layers turn into log-prob differences of about 1e-3 (both are checked against the
    # definition below; a prefix left out or counted twice would show as 1e-1 and more)
    assert np.max(np.abs(l_s[:, :2] - l_p[:, :2])) <= 5e-3
    same = (t_s == t_p).all(axis=1)
    assert same.mean() >= 0.9                                   # a near-tie may flip a row; the oracle check covers those
    assert np.max(np.abs(l_s[same] - l_p[same])) <= 5e-3
    # against the definition
    ma = O.Model(shape, weights)
    S = P * G
    seqs = list(range(S)) if mini and S <= 16 else sorted({0, 1, G - 1, G, S // 2, S - 1})
    eps = max(measured_logit_eps(sapo, sapo.sapo_weights_create(shape, weights), ma,
                                 np.concatenate([prompts[s // G], t_s[s]]), Lp - 1) for s in seqs[:3])
    assert eps <= LOGIT_TOL
    n, exact, near, bad = teacher_forced_token_check(ma, prompts, G, t_s, temp, 55, seqs, delta=NEAR_TIE + 2 * eps / temp)
    assert not bad, bad[:5]
    assert n - exact <= max(2, 0.02 * n), (n, exact, near[:5])
    ref = oracle_logprobs_for(ma, prompts, G, t_s, seqs)
    for s in seqs:
        assert np.max(np.abs(ref[s] - l_s[s])) <= LOGPROB_TOL
    # the replayed graph (side stream) gives the bytes of the eager launches
    t_g, l_g, _ = rollout(sapo, shape, weights, prompts, G, N, temp, 55, threshold, stream=torch.cuda.Stream())
    assert np.array_equal(t_g, t_s) and np.array_equal(l_g.view(np.uint32), l_s.view(np.uint32))


def test_an_ordinary_call_leaves_no_fault_behind(sapo):
    """Nothing to provoke on the device: the bound is wall-clock time and every workgroup exits by itself.  What the
    host can check is that an ordinary call leaves no fault behind: no token is -1."""
    shape = W.MINI_BF16
    weights = W.make_weights(shape, 142, std=0.05)
    prompts = np.random.default_rng(3).integers(0, shape.vocab, size=(2, 128)).astype(np.int32)
    t, l, _ = rollout(sapo, shape, weights, prompts, 4, 20, 1.0, 9, 1)
    assert t.min() >= 0 and np.isfinite(l).all()
