"""One whole round of Algorithm 1 on the GPU for one node, every step through the C ABI:
rollouts -> rewards -> training set (own + swarm datapoints) -> scoring -> policy update -> the new policy
generates the next round's rollouts.  The update is checked against the update oracle on the very training
set the GPU assembled; the rest of the chain has its own parity tests."""
import numpy as np
import pytest

from paper_2509_08721_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sapo():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2509_08721_amd import sapo as S
    S.load_library()
    return S


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def verifier(completions: np.ndarray) -> np.ndarray:
    """Stand-in for a rule-based verifier (Sec. 4.3): reward 1 when the completion's first token id is even."""
    return (completions[:, 0] % 2 == 0).astype(np.float32)


def test_one_round_of_algorithm_1(sapo):
    import torch
    from oracle import sapo_update_oracle as U
    shape = W.TINY
    P, G, Lp, N = 6, 4, 8, 12
    T = Lp + N
    own = W.perturb_norm_gains(W.make_weights(shape, 31, std=0.2), 31)
    other = W.make_weights(shape, 32, std=0.2)              # another node of the swarm
    rng = np.random.default_rng(33)
    prompts = rng.integers(0, shape.vocab, size=(P, Lp)).astype(np.int32)

    def rollouts(weights, seed):
        gw = sapo.sapo_weights_create(shape, weights)
        toks, _ = sapo.sapo_rollout_generate(gw, dev(prompts), G, N, 1.0, seed)
        torch.cuda.synchronize()
        gw.close()
        comp = toks.cpu().numpy()
        return np.concatenate([np.repeat(prompts, G, axis=0), comp], axis=1).astype(np.int32), verifier(comp)

    own_tok, own_rew = rollouts(own, 1001)
    ext_tok, ext_rew = rollouts(other, 1002)
    # training set: 3 own datapoints + 3 of the swarm's with non-zero advantage
    n_local, n_ext = 3, 3
    tok, rew, src, cnt = sapo.sapo_assemble_training_set(dev(own_tok), dev(own_rew), dev(ext_tok), dev(ext_rew), G, n_local,
                                                         n_ext, 77)
    torch.cuda.synchronize()
    cnt = cnt.cpu().numpy()
    assert cnt[0] == n_local and 0 < cnt[1] <= n_ext
    n_dp = int(cnt[0] + cnt[1])
    S = n_dp * G
    tok, rew = tok[:S].contiguous(), rew[:S].contiguous()
    mask = dev(W.make_completion_mask(S, T, N))
    gw = sapo.sapo_weights_create(shape, own)
    logp_old, adv = sapo.sapo_score_logprobs(gw, tok, mask, rew, G)
    torch.cuda.synchronize()
    assert float(adv.abs().max().cpu()) > 0

    tr = sapo.sapo_trainer_create(shape, own, lr=1e-3)
    loss, logp_new = sapo.sapo_policy_update(tr, tok, mask, logp_old, adv)
    torch.cuda.synchronize()
    # the trainer's forward is the scoring pass in another arrangement of the same fp32 arithmetic
    assert float((logp_new - logp_old).abs().max().cpu()) < 2e-4
    # on-policy, nothing is clipped: loss = -(sum of A over the masked tokens) / count
    a = adv.cpu().numpy()
    assert abs(float(loss.cpu()[0]) + float(a.mean())) < 1e-3
    # gradient against the oracle on the training set the GPU assembled
    params = U.parameter_list(shape, own)
    ref_loss, _, ref_g = U.loss_and_gradients(shape, params, tok.cpu().numpy(), mask.cpu().numpy(), logp_old.cpu().numpy(), a)
    assert abs(float(loss.cpu()[0]) - ref_loss) < 5e-4
    gmax = max(float(np.max(np.abs(x))) for x in ref_g)
    for i, b in enumerate(ref_g):
        g = sapo.sapo_trainer_read(tr, 1, i).cpu().numpy().astype(np.float64)
        assert float(np.max(np.abs(g - b))) <= 2e-4 * max(float(np.max(np.abs(b))), 1e-3 * gmax) + 1e-7, i

    # a few more steps on the same set, then the new policy: rollouts with positive advantage became more
    # likely relative to those with negative advantage
    for _ in range(3):
        sapo.sapo_policy_update(tr, tok, mask, logp_old, adv, want_logp=False)
    new = sapo.sapo_trainer_export(tr)
    gw2 = sapo.sapo_weights_create(shape, new)
    logp_after, _ = sapo.sapo_score_logprobs(gw2, tok, mask, rew, G)
    torch.cuda.synchronize()
    d = (logp_after - logp_old).sum(dim=1).cpu().numpy()
    assert d[a > 0].mean() > d[a < 0].mean()
    # and it generates the next round
    toks2, lps2 = sapo.sapo_rollout_generate(gw2, dev(prompts), G, N, 1.0, 2001)
    torch.cuda.synchronize()
    assert toks2.shape == (P * G, N) and np.all(np.isfinite(lps2.cpu().numpy()))
    assert tr.steps == 4
    gw.close(); gw2.close(); tr.close()


@pytest.mark.parametrize("shape_name,tol,std", [("TINY", 1e-4, 0.2), ("MINI_BF16", 2e-2, 0.05)])
def test_node_rounds(sapo, shape_name, tol, std):
    """Two rounds through paper_2509_08721_amd.node.Node (the same calls, packaged), on a stream of its own so that
    the decode step is replayed from a capture: the policy handle is refilled in place with the trainer's export each
    round, what it scores is what the oracle scores for the exported masters, and its next rollouts (replaying the
    step captured before the update) are those of a fresh handle."""
    import torch
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    torch.cuda.set_stream(side)
    try:
        node_rounds(sapo, getattr(W, shape_name), tol, std)
    finally:
        torch.cuda.synchronize()
        torch.cuda.set_stream(torch.cuda.default_stream())


def node_rounds(sapo, shape, tol, std):
    import torch
    from oracle import sapo_oracle as O
    from paper_2509_08721_amd.node import Node
    P, G, Lp, N = 4, 4, 8, 10
    rng = np.random.default_rng(91)
    prompts = dev(rng.integers(0, shape.vocab, size=(P, Lp)).astype(np.int32))
    node = Node(shape, W.add_qkv_bias(W.make_weights(shape, 41, std=std), shape, 41, std=0.1), G)
    other = Node(shape, W.make_weights(shape, 42, std=std), G)
    losses = []
    for rnd in range(2):
        own, _ = node.rollouts(prompts, N, 1.0, 100 + rnd)
        ext, _ = other.rollouts(prompts, N, 1.0, 200 + rnd)
        own_r = dev(verifier(own[:, Lp:].cpu().numpy()))
        ext_r = dev(verifier(ext[:, Lp:].cpu().numpy()))
        seqs, rew = node.training_set(own, own_r, ext, ext_r, 2, 2, 7 + rnd)
        assert seqs.shape[0] % G == 0 and seqs.shape[0] >= 2 * G and seqs.shape[1] == Lp + N
        losses.append(float(node.update(seqs, rew, N).cpu()[0]))
    torch.cuda.synchronize()
    assert node.rounds == 2 and node.trainer.steps == 2 and all(np.isfinite(losses))
    # the policy in use is the trainer's export (biases included)
    exported = sapo.sapo_trainer_export(node.trainer)
    mask = W.make_completion_mask(int(seqs.shape[0]), Lp + N, N)
    lp, _ = sapo.sapo_score_logprobs(node.policy, seqs, dev(mask), rew, G)
    ref = O.score_logprobs(O.Model(shape, exported), seqs.cpu().numpy(), mask)
    assert np.max(np.abs(lp.cpu().numpy() - ref)) < tol
    # the handle was refilled in place: its next rollouts (same buffers as the rounds before) are those of a handle
    # made from the exported masters
    fresh = sapo.sapo_weights_create(shape, exported)
    t_new, l_new = sapo.sapo_rollout_generate(fresh, prompts, G, N, 1.0, 300)
    own, l_own = node.rollouts(prompts, N, 1.0, 300)
    torch.cuda.synchronize()
    assert np.array_equal(own[:, Lp:].cpu().numpy(), t_new.cpu().numpy())
    assert np.array_equal(l_own.cpu().numpy().view(np.uint32), l_new.cpu().numpy().view(np.uint32))
    fresh.close()
    node.close(); other.close()


def test_training_set_with_fewer_own_datapoints_than_asked_for(sapo):
    """Algorithm 1's training set when the node's own pool is smaller than I^n: the swarm's datapoints sit after the
    empty own slots, and the node keeps all of them and no empty row (equal to the oracle's assembly, rows of
    datapoints that exist only)."""
    from oracle import sapo_oracle as O
    from paper_2509_08721_amd.node import Node
    shape = W.TINY
    G, T = 4, 12
    rng = np.random.default_rng(77)
    own_tok = rng.integers(1, shape.vocab, size=(2 * G, T)).astype(np.int32)        # 2 own datapoints, 4 asked for
    own_rew = rng.integers(0, 2, size=2 * G).astype(np.float32)
    ext_tok = rng.integers(1, shape.vocab, size=(6 * G, T)).astype(np.int32)
    ext_rew = np.tile(np.array([1, 0, 0, 1], dtype=np.float32), 6)                  # every swarm datapoint is informative
    node = Node(shape, W.make_weights(shape, 5), G)
    seqs, rew = node.training_set(dev(own_tok), dev(own_rew), dev(ext_tok), dev(ext_rew), 4, 3, 11)
    o_tok, o_rew, o_src, o_cnt = O.assemble_training_set(own_tok, own_rew, ext_tok, ext_rew, G, 4, 3, 11)
    assert list(o_cnt) == [2, 3]
    keep = np.repeat(np.asarray(o_src) >= 0, G)
    assert seqs.shape[0] == 5 * G and np.array_equal(seqs.cpu().numpy(), o_tok[keep]) and np.array_equal(rew.cpu().numpy(), o_rew[keep])
    assert (seqs.cpu().numpy() != 0).all()                                          # no empty slot's zero rows
    node.close()
