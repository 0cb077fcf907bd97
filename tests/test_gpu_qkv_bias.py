"""Models with biases on the query / key / value projections, all three code paths (shape-generic fp32,
64-token decode + token-parallel prefill on the MFMA path, many-row decode), against the oracle."""
import numpy as np
import pytest
import torch

from oracle import sapo_oracle as O
from paper_2509_08721_amd import sapo, workloads as W
from tests.parity import oracle_logprobs_for, teacher_forced_token_check
from tests.test_gpu_mfma import check_rollout, dev, LOGPROB_TOL

pytestmark = pytest.mark.gpu


def test_bias_fp32_generic_path():
    shape = W.TINY
    w = W.add_qkv_bias(W.perturb_norm_gains(W.make_weights(shape, 31), 31), shape, 8, std=0.3)
    gw = sapo.sapo_weights_create(shape, w)
    m = O.Model(shape, w)
    prompts = np.random.default_rng(1).integers(0, shape.vocab, size=(2, 19)).astype(np.int32)
    G, N = 3, 21
    toks, lps = sapo.sapo_rollout_generate(gw, dev(prompts), G, N, 1.0, seed=5)
    toks, lps = toks.cpu().numpy(), lps.cpu().numpy()
    n, exact, near, bad = teacher_forced_token_check(m, prompts, G, toks, 1.0, 5, range(2 * G), delta=1e-3)
    assert not bad and len(near) <= 1
    ref = oracle_logprobs_for(m, prompts, G, toks, range(2 * G))
    for s in range(2 * G):
        assert np.max(np.abs(ref[s] - lps[s])) <= 1e-4
    # scoring of the same sequences reproduces the rollout's log-probs, and the oracle's
    seqs = np.concatenate([np.repeat(prompts, G, axis=0), toks], axis=1).astype(np.int32)
    mask = W.make_completion_mask(2 * G, 19 + N, N)
    lp, _ = sapo.sapo_score_logprobs(gw, dev(seqs), dev(mask), dev(np.ones(2 * G, np.float32)), G)
    assert np.max(np.abs(lp.cpu().numpy() - O.score_logprobs(m, seqs, mask))) <= 1e-4
    # the biases are really in: the same weights without them give other log-probs
    gw0 = sapo.sapo_weights_create(shape, W.perturb_norm_gains(W.make_weights(shape, 31), 31))
    lp0, _ = sapo.sapo_score_logprobs(gw0, dev(seqs), dev(mask), dev(np.ones(2 * G, np.float32)), G)
    assert float((lp0 - lp).abs().max()) > 1e-2


@pytest.mark.parametrize("shape_name,P,G,Lp,N", [("MINI_BF16", 3, 4, 21, 40), ("MINI_BF16_HD128", 2, 3, 17, 30),
                                                  ("MINI_BF16", 9, 8, 16, 6)])
def test_bias_mfma_paths(shape_name, P, G, Lp, N):
    shape = getattr(W, shape_name)
    w = W.add_qkv_bias(W.perturb_norm_gains(W.make_weights(shape, 61, std=0.05), 61), shape, 9, std=0.2)
    gw = sapo.sapo_weights_create(shape, w)
    assert gw.uses_mfma
    prompts, toks, lps = check_rollout(sapo, shape, w, gw, P, G, Lp, N, 1.0, seed=77)
    # teacher-forced scoring (token-parallel GEMM path) agrees with the oracle and with the rollout
    S, T = P * G, Lp + N
    seqs = np.concatenate([np.repeat(prompts, G, axis=0), toks], axis=1).astype(np.int32)
    mask = W.make_completion_mask(S, T, N)
    lp, _ = sapo.sapo_score_logprobs(gw, dev(seqs), dev(mask), dev(np.ones(S, np.float32)), G)
    lp = lp.cpu().numpy()
    assert np.max(np.abs(lp[:, Lp:] - lps)) <= LOGPROB_TOL
    ref = O.score_logprobs(O.Model(shape, w), seqs[:2], mask[:2])
    assert np.max(np.abs(lp[:2] - ref)) <= LOGPROB_TOL


def test_bias_replaced_after_a_graph_was_captured():
    shape = W.MINI_BF16
    w0 = W.perturb_norm_gains(W.make_weights(shape, 61, std=0.05), 61)
    w1 = W.add_qkv_bias(w0, shape, 9, std=0.2)
    gw = sapo.sapo_weights_create(shape, w0)
    ref = sapo.sapo_weights_create(shape, w1)
    prompts = dev(np.random.default_rng(2).integers(0, shape.vocab, size=(2, 16)).astype(np.int32))
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        ws = torch.empty(sapo.sapo_rollout_workspace_bytes(gw, 2, 16, 4, 12) + 256, dtype=torch.uint8, device="cuda")
        t0, _ = sapo.sapo_rollout_generate(gw, prompts, 4, 12, 1.0, 3, workspace=ws, stream=st)   # captures the decode step
        st.synchronize()
        for l, lw in enumerate(w1["layers"]):
            sapo.sapo_weights_set_qkv_bias(gw, l, dev(lw["bq"]), dev(lw["bk"]), dev(lw["bv"]), stream=st)
        t1, l1 = sapo.sapo_rollout_generate(gw, prompts, 4, 12, 1.0, 3, workspace=ws, stream=st)
        t2, l2 = sapo.sapo_rollout_generate(ref, prompts, 4, 12, 1.0, 3, stream=st)
        st.synchronize()
    assert torch.equal(t1, t2) and torch.equal(l1, l2)
    assert not torch.equal(t0, t1)
