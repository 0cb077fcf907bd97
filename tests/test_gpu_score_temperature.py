"""Scoring at a temperature against the oracle, on the shape-generic and the MFMA path."""
import numpy as np
import pytest
import torch

from oracle import sapo_oracle as O
from paper_2509_08721_amd import sapo, workloads as W

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("shape_name,tol,std", [("TINY", 1e-4, 0.02), ("MINI_BF16", 2e-2, 0.05), ("MINI_BF16_HD128", 2e-2, 0.05)])
def test_scoring_at_a_temperature(shape_name, tol, std):
    shape = getattr(W, shape_name)
    w = W.perturb_norm_gains(W.make_weights(shape, 17, std=std), 17)
    gw = sapo.sapo_weights_create(shape, w)
    m = O.Model(shape, w)
    rng = np.random.default_rng(2)
    S, T, G = 6, 45, 3
    toks = rng.integers(0, shape.vocab, size=(S, T)).astype(np.int32)
    mask = (rng.random((S, T)) < 0.5).astype(np.uint8)
    rew = rng.random(S).astype(np.float32)
    base, adv1 = sapo.sapo_score_logprobs(gw, dev(toks), dev(mask), dev(rew), G)
    for temp in (0.7, 1.0, 2.5):
        lp, adv = sapo.sapo_score_logprobs_at(gw, dev(toks), dev(mask), dev(rew), G, temp)
        ref = O.score_logprobs(m, toks, mask, temperature=temp)
        assert np.max(np.abs(lp.cpu().numpy() - ref)) <= tol, temp
        assert torch.equal(adv, adv1)
        if temp == 1.0:
            assert torch.equal(lp, base)
        else:
            assert float((lp - base).abs().max()) > 10 * tol
    with pytest.raises(sapo.SapoError):
        sapo.sapo_score_logprobs_at(gw, dev(toks), dev(mask), dev(rew), G, 0.0)


def test_rollout_at_a_temperature_then_scoring_at_it():
    # the log-probs of the sampling distribution: a rollout at T, scored at T, is the on-policy case for the
    # clipped surrogate whatever T was
    shape = W.MINI_BF16
    w = W.make_weights(shape, 23, std=0.05)
    gw = sapo.sapo_weights_create(shape, w)
    prompts = np.random.default_rng(3).integers(0, shape.vocab, size=(2, 12)).astype(np.int32)
    G, N, temp = 4, 20, 0.7
    toks, lp_pol = sapo.sapo_rollout_generate(gw, dev(prompts), G, N, temp, 9)
    seqs = torch.cat([dev(prompts).repeat_interleave(G, dim=0), toks], dim=1).contiguous()
    mask = dev(W.make_completion_mask(2 * G, 12 + N, N))
    rew = dev(np.ones(2 * G, np.float32))
    at1, _ = sapo.sapo_score_logprobs(gw, seqs, mask, rew, G)
    att, _ = sapo.sapo_score_logprobs_at(gw, seqs, mask, rew, G, temp)
    assert float((at1[:, 12:] - lp_pol).abs().max()) <= 2e-2       # the rollout returns the policy's own (T = 1)
    m = O.Model(shape, w)
    ref = O.score_logprobs(m, seqs.cpu().numpy()[:2], mask.cpu().numpy()[:2], temperature=temp)
    assert np.max(np.abs(att.cpu().numpy()[:2] - ref)) <= 2e-2
