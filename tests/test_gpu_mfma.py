"""GPU parity of the bf16 MFMA kernels on small tile-aligned shapes: rollouts (64-token decode
path and the many-row path), scoring, teacher-forced logits, against the CPU oracle."""
import os

import numpy as np
import pytest

from oracle import sapo_oracle as O
from paper_2509_08721_amd import workloads as W
from tests.parity import measured_logit_eps, oracle_logprobs_for, teacher_forced_token_check

pytestmark = pytest.mark.gpu

LOGIT_TOL_BF16 = 5e-2
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


def make(sapo, shape, seed, std=0.05):
    w = W.perturb_norm_gains(W.make_weights(shape, seed, std=std), seed)
    gw = sapo.sapo_weights_create(shape, w)
    return w, gw


def check_rollout(sapo, shape, w, gw, P, G, Lp, N, temp, seed, max_flip_frac=0.05):
    ma = O.Model(shape, w)
    prompts = np.random.default_rng(seed).integers(0, shape.vocab, size=(P, Lp)).astype(np.int32)
    toks, lps = sapo.sapo_rollout_generate(gw, dev(prompts), G, N, temp, seed)
    toks, lps = toks.cpu().numpy(), lps.cpu().numpy()
    assert toks.min() >= 0 and toks.max() < shape.vocab
    S = P * G
    seqs = list(range(S)) if S <= 16 else sorted({0, 1, S // 2, S - 2, S - 1, G, 2 * G + 1})
    # stated band: literal 1e-3 plus twice the logit error measured on these very sequences (teacher-forced device
    # logits against the definition), scaled by 1/T
    eps = max(measured_logit_eps(sapo, gw, ma, np.concatenate([prompts[s // G], toks[s]]), Lp - 1) for s in seqs)
    assert eps <= LOGIT_TOL_BF16, eps
    band = NEAR_TIE + 2 * eps / (temp if temp > 0 else 1.0)
    n, exact, near, bad = teacher_forced_token_check(ma, prompts, G, toks, temp, seed, seqs, delta=band)
    assert not bad, bad[:10]
    assert n - exact <= max(2, max_flip_frac * n), (n, exact, near[:10])
    ref = oracle_logprobs_for(ma, prompts, G, toks, seqs)
    for s in seqs:
        assert np.max(np.abs(ref[s] - lps[s])) <= LOGPROB_TOL
    return prompts, toks, lps


@pytest.mark.parametrize("shape_name,P,G,Lp,N,temp", [
    ("MINI_BF16", 3, 4, 21, 40, 1.0),        # partial prompt page, several page pairs
    ("MINI_BF16", 8, 8, 32, 24, 0.7),        # full 64-sequence decode tile
    ("MINI_BF16", 1, 2, 200, 70, 1.0),       # long context: all four waves of the attention kernel busy
    ("MINI_BF16_HD128", 2, 3, 17, 30, 1.0),  # head_dim 128, 6 query heads on one KV head, untied LM head
    ("MINI_BF16", 9, 8, 16, 6, 1.0),         # 72 sequences: many-row decode path
    ("MINI_BF16", 2, 2, 5, 9, 0.0),          # greedy
    ("MINI_BF16_HD128", 33, 8, 17, 20, 1.0), # 264 sequences on one KV head: more attention workgroups than compute units
    ("MINI_BF16", 1, 1, 24, 40, 1.0),        # one question, one completion (the pass@1 judge's shape)
])
def test_mfma_rollout(sapo, shape_name, P, G, Lp, N, temp):
    shape = getattr(W, shape_name)
    w, gw = make(sapo, shape, 61)
    assert gw.uses_mfma
    prompts, toks, lps = check_rollout(sapo, shape, w, gw, P, G, Lp, N, temp, seed=4242)
    if temp == 0.0:
        assert np.array_equal(toks[0], toks[1])
    # determinism: same call twice gives identical bytes
    t2, l2 = sapo.sapo_rollout_generate(gw, dev(prompts), G, N, temp, 4242)
    assert np.array_equal(t2.cpu().numpy(), toks)
    assert np.array_equal(l2.cpu().numpy().view(np.uint32), lps.view(np.uint32))


@pytest.mark.parametrize("shape_name,S,T,G", [("MINI_BF16", 6, 300, 3), ("MINI_BF16_HD128", 4, 77, 2),
                                              ("MINI_BF16", 40, 260, 8)])
def test_mfma_scoring_and_logits(sapo, shape_name, S, T, G):
    shape = getattr(W, shape_name)
    w, gw = make(sapo, shape, 71)
    ma = O.Model(shape, w)
    rng = np.random.default_rng(5)
    toks = rng.integers(0, shape.vocab, size=(S, T)).astype(np.int32)
    mask = (rng.random((S, T)) < 0.5).astype(np.uint8)
    mask[0, :] = 0
    mask[1, :] = 1
    rewards = (rng.random(S) < 0.3).astype(np.float32)
    rewards[:G] = 1.0                                   # a zero-advantage group
    lp, adv = sapo.sapo_score_logprobs(gw, dev(toks), dev(mask), dev(rewards), G)
    lp, adv = lp.cpu().numpy(), adv.cpu().numpy()
    check = list(range(S)) if S <= 8 else [0, 1, 2, S // 2, S - 1]
    o_lp = O.score_logprobs(ma, toks[check], mask[check])
    assert np.isfinite(lp).all()
    assert np.max(np.abs(lp[check] - o_lp)) <= LOGPROB_TOL
    assert np.all(lp[mask == 0] == 0.0) and np.all(lp[:, 0] == 0.0)
    assert np.max(np.abs(adv - O.group_advantages(rewards, G))) <= 1e-5 and np.all(adv[:G] == 0.0)
    # batch-composition invariance (bit-exact: a row's arithmetic does not depend on its tile)
    lp1, _ = sapo.sapo_score_logprobs(gw, dev(toks[:G]), dev(mask[:G]), dev(rewards[:G]), G)
    assert np.array_equal(lp1.cpu().numpy(), lp[:G])
    # teacher-forced logits against the definition
    pos = [(s, t) for s in check[:3] for t in (0, T // 2, T - 1)]
    z = sapo.sapo_debug_logits(gw, dev(toks), pos).cpu().numpy()
    ea = 0.0
    for i, (s, t) in enumerate(pos):
        ea = max(ea, np.max(np.abs(z[i] - O.forward_logits(ma, toks[s, : t + 1], at=[t])[0])))
    assert ea <= LOGIT_TOL_BF16, ea


def test_mfma_matches_generic_kernels(sapo):
    """The same bf16 model on the shape-generic kernels and on the MFMA kernels."""
    shape = W.MINI_BF16
    w = W.perturb_norm_gains(W.make_weights(shape, 81, std=0.05), 81)
    gw = sapo.sapo_weights_create(shape, w)
    os.environ["SAPO_FORCE_GENERIC"] = "1"
    try:
        gg = sapo.sapo_weights_create(shape, w)
    finally:
        del os.environ["SAPO_FORCE_GENERIC"]
    assert gw.uses_mfma and not gg.uses_mfma
    rng = np.random.default_rng(1)
    toks = rng.integers(0, shape.vocab, size=(3, 90)).astype(np.int32)
    pos = [(0, 0), (1, 50), (2, 89)]
    za = sapo.sapo_debug_logits(gw, dev(toks), pos).cpu().numpy()
    zb = sapo.sapo_debug_logits(gg, dev(toks), pos).cpu().numpy()
    assert np.max(np.abs(za - zb)) <= 2e-2
    mask = np.ones((3, 90), dtype=np.uint8)
    rew = np.zeros(3, dtype=np.float32)
    la, _ = sapo.sapo_score_logprobs(gw, dev(toks), dev(mask), dev(rew), 3)
    lb, _ = sapo.sapo_score_logprobs(gg, dev(toks), dev(mask), dev(rew), 3)
    assert np.max(np.abs(la.cpu().numpy() - lb.cpu().numpy())) <= 2e-2


def test_mfma_rollout_logprobs_equal_scoring(sapo):
    """Decode with the KV cache equals teacher-forced recompute at the API level."""
    shape = W.MINI_BF16
    w, gw = make(sapo, shape, 91)
    prompts = np.random.default_rng(2).integers(0, shape.vocab, size=(4, 32)).astype(np.int32)
    toks, lps = sapo.sapo_rollout_generate(gw, dev(prompts), 4, 48, 1.0, 7)
    toks, lps = toks.cpu().numpy(), lps.cpu().numpy()
    seqs = np.concatenate([np.repeat(prompts, 4, axis=0), toks], axis=1).astype(np.int32)
    mask = W.make_completion_mask(16, 80, 48)
    lp, _ = sapo.sapo_score_logprobs(gw, dev(seqs), dev(mask), dev(np.zeros(16, dtype=np.float32)), 4)
    assert np.max(np.abs(lp.cpu().numpy()[:, 32:] - lps)) <= LOGPROB_TOL


@pytest.mark.parametrize("shape_name,P,G", [("MINI_BF16", 4, 4),          # 64-token decode kernels, fused sampler
                                            ("MINI_BF16", 9, 8),          # 72 sequences: FFN on the token-parallel GEMM, split-K
                                            ("MINI_BF16_HD128", 11, 6)])  # the same with head dim 128 and an untied LM head
def test_graph_replay_matches_eager_launches(sapo, shape_name, P, G):
    """On a non-default stream the decode step is captured once and replayed; the result must be
    bit-identical to eager launches, also when the cached graph is reused with another seed and
    temperature, and after the buffers change."""
    import torch
    shape = getattr(W, shape_name)
    w, gw = make(sapo, shape, 95)
    S, N = P * G, 25
    prompts = dev(np.random.default_rng(3).integers(0, shape.vocab, size=(P, 20)).astype(np.int32))
    eager = {}
    for seed, temp in ((1, 1.0), (2, 0.7), (3, 0.0)):
        t, l = sapo.sapo_rollout_generate(gw, prompts, G, N, temp, seed)      # default stream: eager
        eager[(seed, temp)] = (t.cpu().numpy(), l.cpu().numpy())
    side = torch.cuda.Stream()
    nbytes = sapo.sapo_rollout_workspace_bytes(gw, P, 20, G, N)
    ws = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
    out_t = torch.empty((S, N), dtype=torch.int32, device="cuda")
    out_l = torch.empty((S, N), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for rep in range(2):
            for (seed, temp), (et, el) in eager.items():
                sapo.sapo_rollout_generate(gw, prompts, G, N, temp, seed, workspace=ws, out_tokens=out_t,
                                           out_logprobs=out_l, stream=side)
                side.synchronize()
                assert np.array_equal(out_t.cpu().numpy(), et), (rep, seed)
                assert np.array_equal(out_l.cpu().numpy().view(np.uint32), el.view(np.uint32)), (rep, seed)
        # other buffers: the graph is rebuilt
        t2, l2 = sapo.sapo_rollout_generate(gw, prompts, G, N, 1.0, 1, stream=side)
        side.synchronize()
        assert np.array_equal(t2.cpu().numpy(), eager[(1, 1.0)][0])


def test_weights_update_in_place_keeps_the_captured_step(sapo):
    """sapo_weights_update: new values into the handle's own buffers.  A rollout call with the same workspace and
    output buffers as before then replays the decode step captured under the old values and must return what a
    handle created from the new values returns, byte for byte; scoring likewise."""
    import torch
    shape = W.MINI_BF16
    wa, gw = make(sapo, shape, 61)
    wb = W.perturb_norm_gains(W.make_weights(shape, 62, std=0.05), 62)
    P, G, Lp, N = 3, 4, 21, 40
    prompts = dev(np.random.default_rng(5).integers(0, shape.vocab, size=(P, Lp)).astype(np.int32))
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        ws = torch.empty(sapo.sapo_rollout_workspace_bytes(gw, P, Lp, G, N) + 256, dtype=torch.uint8, device="cuda")
        ot = torch.empty((P * G, N), dtype=torch.int32, device="cuda")
        ol = torch.empty((P * G, N), dtype=torch.float32, device="cuda")
        sapo.sapo_rollout_generate(gw, prompts, G, N, 1.0, 7, workspace=ws, out_tokens=ot, out_logprobs=ol, stream=side)
        side.synchronize()
        ta = ot.cpu().numpy().copy()
        sapo.sapo_weights_update(gw, wb, stream=side)
        sapo.sapo_rollout_generate(gw, prompts, G, N, 1.0, 7, workspace=ws, out_tokens=ot, out_logprobs=ol, stream=side)
        side.synchronize()
        tb, lb = ot.cpu().numpy().copy(), ol.cpu().numpy().copy()
        fresh = sapo.sapo_weights_create(shape, wb)
        tf, lf = sapo.sapo_rollout_generate(fresh, prompts, G, N, 1.0, 7, stream=side)
        side.synchronize()
    assert not np.array_equal(ta, tb)
    assert np.array_equal(tb, tf.cpu().numpy()) and np.array_equal(lb.view(np.uint32), lf.cpu().numpy().view(np.uint32))
    seqs = dev(np.concatenate([np.repeat(prompts.cpu().numpy(), G, axis=0), tb], axis=1).astype(np.int32))
    mask, rew = dev(W.make_completion_mask(P * G, Lp + N, N)), dev(W.make_rewards(P * G, 0.5, 3))
    l1, _ = sapo.sapo_score_logprobs(gw, seqs, mask, rew, G)
    l2, _ = sapo.sapo_score_logprobs(fresh, seqs, mask, rew, G)
    assert np.array_equal(l1.cpu().numpy().view(np.uint32), l2.cpu().numpy().view(np.uint32))
    # a list of the wrong length is refused and changes nothing
    lib = sapo.load_library()
    import ctypes as C
    bad = (C.c_void_p * 3)()
    assert lib.sapo_weights_update(gw.handle, bad, 3, None) == sapo.SAPO_EINVAL
    l3, _ = sapo.sapo_score_logprobs(gw, seqs, mask, rew, G)
    assert np.array_equal(l1.cpu().numpy().view(np.uint32), l3.cpu().numpy().view(np.uint32))
    gw.close(); fresh.close()
