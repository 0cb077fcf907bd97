"""Edge cases of the two calls on the matrix-core kernels (the fp32 shape-generic path has its own in
test_gpu_tiny.py): the smallest and the largest sizes a model allows, masks that select nothing or a position with
no prediction behind it, a single row, batches that end inside a tile."""
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


@pytest.fixture(scope="module")
def model(sapo):
    shape = W.MINI_BF16
    w = W.perturb_norm_gains(W.make_weights(shape, 131, std=0.05), 131)
    gw = sapo.sapo_weights_create(shape, w)
    assert gw.uses_mfma
    return shape, w, gw, O.Model(shape, w)


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check_tokens(sapo, model, prompts, G, toks, lps, temp, seed):
    shape, w, gw, ma = model
    S, Lp = toks.shape[0], prompts.shape[1]
    assert toks.min() >= 0 and toks.max() < shape.vocab
    seqs = list(range(S))
    eps = max(measured_logit_eps(sapo, gw, ma, np.concatenate([prompts[s // G], toks[s]]), Lp - 1) for s in seqs)
    assert eps <= LOGIT_TOL
    n, exact, near, bad = teacher_forced_token_check(ma, prompts, G, toks, temp, seed, seqs,
                                                     delta=NEAR_TIE + 2 * eps / (temp if temp > 0 else 1.0))
    assert not bad, bad[:5]
    assert n - exact <= max(1, 0.02 * n), (n, exact, near[:5])
    ref = oracle_logprobs_for(ma, prompts, G, toks, seqs)
    for s in seqs:
        assert np.max(np.abs(ref[s] - lps[s])) <= LOGPROB_TOL


@pytest.mark.parametrize("P,G,Lp,N", [
    (1, 1, 1, 1),        # one prompt token, one new token: the prompt's forward and no decode step at all
    (2, 3, 1, 5),        # one-token prompts
    (3, 2, 16, 1),       # exactly one page of prompt, a single sampled token
    (1, 2, 17, 2),       # the first decode step crosses into the prompt's partial page
])
def test_smallest_rollouts(sapo, model, P, G, Lp, N):
    shape, w, gw, ma = model
    prompts = np.random.default_rng(P * 100 + Lp).integers(0, shape.vocab, size=(P, Lp)).astype(np.int32)
    toks, lps = sapo.sapo_rollout_generate(gw, dev(prompts), G, N, 1.0, 31)
    toks, lps = toks.cpu().numpy(), lps.cpu().numpy()
    assert toks.shape == (P * G, N) and sapo.sapo_rollout_last_stats(gw)["steps"] == N - 1
    check_tokens(sapo, model, prompts, G, toks, lps, 1.0, 31)


def test_rollout_up_to_the_longest_sequence_the_model_allows(sapo, model):
    shape, w, gw, ma = model
    Lp, N = 40, shape.max_seq - 40                      # the last token's position is max_seq - 1
    prompts = np.random.default_rng(8).integers(0, shape.vocab, size=(1, Lp)).astype(np.int32)
    toks, lps = sapo.sapo_rollout_generate(gw, dev(prompts), 2, N, 1.0, 32)
    check_tokens(sapo, model, prompts, 2, toks.cpu().numpy(), lps.cpu().numpy(), 1.0, 32)
    with pytest.raises(sapo.SapoError):
        sapo.sapo_rollout_generate(gw, dev(prompts), 2, N + 1, 1.0, 32)


def test_scoring_masks_that_select_nothing_or_only_position_0(sapo, model):
    shape, w, gw, ma = model
    rng = np.random.default_rng(9)
    S, T, G = 4, 50, 2
    toks = rng.integers(0, shape.vocab, size=(S, T)).astype(np.int32)
    rewards = np.array([1, 0, 1, 1], dtype=np.float32)
    none = np.zeros((S, T), dtype=np.uint8)
    lp, adv = sapo.sapo_score_logprobs(gw, dev(toks), dev(none), dev(rewards), G)
    assert np.all(lp.cpu().numpy() == 0.0)
    assert np.max(np.abs(adv.cpu().numpy() - O.group_advantages(rewards, G))) <= 1e-5 and np.all(adv.cpu().numpy()[2:] == 0.0)
    first = none.copy()
    first[:, 0] = 1                                       # nothing predicts position 0: log-prob 0 by definition
    lp, _ = sapo.sapo_score_logprobs(gw, dev(toks), dev(first), dev(rewards), G)
    assert np.all(lp.cpu().numpy() == 0.0)
    one = none.copy()
    one[3, T - 1] = 1                                     # a single scored row in the whole batch
    lp, _ = sapo.sapo_score_logprobs(gw, dev(toks), dev(one), dev(rewards), G)
    lp = lp.cpu().numpy()
    ref = O.score_logprobs(ma, toks, one)
    assert np.count_nonzero(lp) == 1 and abs(lp[3, T - 1] - ref[3, T - 1]) <= LOGPROB_TOL


@pytest.mark.parametrize("S,T,G", [(1, 1, 1),       # one row, one token: nothing to score
                                   (1, 2, 1),       # one prediction
                                   (3, 33, 3),      # rows end one past a 32-row fragment block
                                   (1, 512, 1)])    # the longest sequence the model allows
def test_scoring_smallest_and_largest_batches(sapo, model, S, T, G):
    shape, w, gw, ma = model
    assert T <= shape.max_seq
    rng = np.random.default_rng(S * 1000 + T)
    toks = rng.integers(0, shape.vocab, size=(S, T)).astype(np.int32)
    mask = np.ones((S, T), dtype=np.uint8)
    rewards = rng.random(S).astype(np.float32)
    lp, adv = sapo.sapo_score_logprobs(gw, dev(toks), dev(mask), dev(rewards), G)
    lp, adv = lp.cpu().numpy(), adv.cpu().numpy()
    ref = O.score_logprobs(ma, toks, mask)
    assert np.all(lp[:, 0] == 0.0) and np.max(np.abs(lp - ref)) <= LOGPROB_TOL
    assert np.max(np.abs(adv - O.group_advantages(rewards, G))) <= 1e-5
    if G == 1:
        assert np.all(adv == 0.0)                         # a group of one has no spread
    z = sapo.sapo_debug_logits(gw, dev(toks), [(S - 1, T - 1)]).cpu().numpy()[0]
    assert np.max(np.abs(z - O.forward_logits(ma, toks[S - 1], at=[T - 1])[0])) <= LOGIT_TOL
    with pytest.raises(sapo.SapoError):
        sapo.sapo_score_logprobs(gw, dev(np.zeros((1, shape.max_seq + 1), dtype=np.int32)),
                                 dev(np.ones((1, shape.max_seq + 1), dtype=np.uint8)), dev(np.zeros(1, dtype=np.float32)), 1)


@pytest.mark.parametrize("S,T", [(3, 200),      # 600 rows: the last 128-token and 256-token tiles both end inside
                                 (8, 128)])     # 1024 rows: whole tiles of either height
def test_both_tile_heights_of_the_token_parallel_gemm_give_the_same_bits(sapo, model, S, T):
    """The projections run on 256-token or 128-token tiles, chosen per launch from how full the rounds of resident
    workgroups are; SAPO_BIG_TILE forces one.  Same products in the same order: the log-probs must agree bit for bit,
    and with the oracle as everywhere."""
    import os
    shape, w, gw, ma = model
    rng = np.random.default_rng(S * 7 + T)
    toks = rng.integers(0, shape.vocab, size=(S, T)).astype(np.int32)
    mask = np.ones((S, T), dtype=np.uint8)
    rewards = rng.random(S).astype(np.float32)
    out = {}
    try:
        for tile in ("128", "256"):
            os.environ["SAPO_BIG_TILE"] = tile
            lp, _ = sapo.sapo_score_logprobs(gw, dev(toks), dev(mask), dev(rewards), 1)
            out[tile] = lp.cpu().numpy()
    finally:
        os.environ.pop("SAPO_BIG_TILE", None)
    assert np.array_equal(out["128"].view(np.uint32), out["256"].view(np.uint32))
    assert np.max(np.abs(out["256"] - O.score_logprobs(ma, toks, mask))) <= LOGPROB_TOL
