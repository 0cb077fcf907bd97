"""Rollouts for prompts of different lengths (with and without a stop token) against the oracle."""
import numpy as np
import pytest
import torch

from oracle import sapo_oracle as O
from paper_2509_08721_amd import sapo, workloads as W
from tests.parity import measured_logit_eps

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def padded(prompts, Lp, vocab, seed):
    """Rows of different lengths in one [P, Lp] array; the padding is random ids (it must not matter)."""
    out = np.random.default_rng(seed).integers(0, vocab, size=(len(prompts), Lp)).astype(np.int32)
    for p, pr in enumerate(prompts):
        out[p, :len(pr)] = pr
    return out


def check_against_oracle(model, prompts, G, toks, lps, temp, seed, seqs, delta, lp_tol, max_flips):
    """Teacher-forced on the GPU's own prefix: token = argmax of the oracle's perturbed scores (up to a stated
    near-tie band), log-prob within lp_tol."""
    flips = 0
    N = toks.shape[1]
    for s in seqs:
        pr = prompts[s // G]
        L = len(pr)
        seq = np.concatenate([pr, toks[s]])
        z = O.forward_logits(model, seq[:-1], at=range(L - 1, L + N - 1))
        lp = O.log_softmax(z)
        assert np.max(np.abs(lp[np.arange(N), toks[s]] - lps[s])) <= lp_tol, (s, L)
        for t in range(N):
            y = O.perturbed_scores(z[t], temp, seed, s, t)
            v = int(np.argmax(y))
            if v != int(toks[s, t]):
                assert float(y[v]) - float(y[toks[s, t]]) <= delta, (s, t)
                flips += 1
    assert flips <= max_flips, flips


def test_ragged_fp32_matches_oracle_exactly_where_unique():
    shape = W.TINY
    w = W.perturb_norm_gains(W.make_weights(shape, 31), 31)
    gw = sapo.sapo_weights_create(shape, w)
    m = O.Model(shape, w)
    rng = np.random.default_rng(3)
    lens = [5, 16, 33, 17, 1]                       # below / at / above page boundaries, a one-token prompt
    prompts = [rng.integers(0, shape.vocab, size=n).astype(np.int32) for n in lens]
    G, N, seed = 3, 20, 77
    pad = padded(prompts, 33, shape.vocab, 1)
    toks, lps, _ = sapo.sapo_rollout_generate_ragged(gw, dev(pad), lens, G, N, 1.0, seed)
    toks, lps = toks.cpu().numpy(), lps.cpu().numpy()
    o_t, o_l = O.rollout_generate_ragged(m, prompts, G, N, 1.0, seed)
    check_against_oracle(m, prompts, G, toks, lps, 1.0, seed, range(len(lens) * G), 1e-3, 1e-4, 1)
    assert (toks == o_t).mean() > 0.9                # free-running agreement (a near-tie may fork a sequence)
    # other padding, same result
    t2, l2, _ = sapo.sapo_rollout_generate_ragged(gw, dev(padded(prompts, 33, shape.vocab, 2)), lens, G, N, 1.0, seed)
    assert np.array_equal(t2.cpu().numpy(), toks) and np.array_equal(l2.cpu().numpy(), lps)
    # a prompt's rows are those of a call with that prompt alone... for the first prompt (sequence ids 0 .. G-1)
    t3, l3 = sapo.sapo_rollout_generate(gw, dev(prompts[0][None, :]), G, N, 1.0, seed)
    assert np.array_equal(t3.cpu().numpy(), toks[:G]) and np.max(np.abs(l3.cpu().numpy() - lps[:G])) <= 1e-5
    # equal lengths reduce to the plain call
    same = rng.integers(0, shape.vocab, size=(3, 21)).astype(np.int32)
    a, la, _ = sapo.sapo_rollout_generate_ragged(gw, dev(same), [21, 21, 21], G, N, 1.0, seed)
    b, lb = sapo.sapo_rollout_generate(gw, dev(same), G, N, 1.0, seed)
    assert torch.equal(a, b) and torch.equal(la, lb)


@pytest.mark.parametrize("shape_name,lens,G,N", [("MINI_BF16", [21, 40, 7, 32], 4, 30), ("MINI_BF16_HD128", [17, 3], 3, 20),
                                                  ("MINI_BF16", [16, 9, 30, 12, 25, 31, 2, 19, 8], 8, 10)])
def test_ragged_mfma_paths(shape_name, lens, G, N):
    shape = getattr(W, shape_name)
    w = W.perturb_norm_gains(W.make_weights(shape, 61, std=0.05), 61)
    gw = sapo.sapo_weights_create(shape, w)
    assert gw.uses_mfma
    rng = np.random.default_rng(5)
    prompts = [rng.integers(0, shape.vocab, size=n).astype(np.int32) for n in lens]
    pad = padded(prompts, max(lens), shape.vocab, 1)
    st = torch.cuda.Stream()                         # graph replay of the decode step
    with torch.cuda.stream(st):
        toks, lps, _ = sapo.sapo_rollout_generate_ragged(gw, dev(pad), lens, G, N, 1.0, 11, stream=st)
        st.synchronize()
    toks, lps = toks.cpu().numpy(), lps.cpu().numpy()
    S = len(lens) * G
    seqs = range(S) if S <= 16 else [0, 1, G, 2 * G + 1, S // 2, S - 2, S - 1]
    ma = O.Model(shape, w)
    eps = max(measured_logit_eps(sapo, gw, ma, np.concatenate([prompts[s // G], toks[s]]), len(prompts[s // G]) - 1) for s in seqs)
    assert eps <= 5e-2, eps
    check_against_oracle(ma, prompts, G, toks, lps, 1.0, 11, seqs, 1e-3 + 2 * eps, 2e-2, max(2, int(0.05 * len(seqs) * N)))


def test_ragged_with_stop_token_fp32():
    shape = W.TINY
    w = W.make_weights(shape, 31)
    gw = sapo.sapo_weights_create(shape, w)
    rng = np.random.default_rng(4)
    lens = [9, 20, 14]
    prompts = [rng.integers(0, shape.vocab, size=n).astype(np.int32) for n in lens]
    pad = padded(prompts, 20, shape.vocab, 1)
    G, N = 4, 30
    t0, l0, none = sapo.sapo_rollout_generate_ragged(gw, dev(pad), lens, G, N, 1.0, 5)
    assert none is None
    t0, l0 = t0.cpu().numpy(), l0.cpu().numpy()
    vals, counts = np.unique(t0[:, 2:N - 2], return_counts=True)
    stop = int(vals[np.argmax(counts)])
    t1, l1, ln = sapo.sapo_rollout_generate_ragged(gw, dev(pad), lens, G, N, 1.0, 5, stop_token=stop)
    t1, l1, ln = t1.cpu().numpy(), l1.cpu().numpy(), ln.cpu().numpy()
    for s in range(len(lens) * G):
        where = np.nonzero(t0[s] == stop)[0]
        n = int(where[0]) + 1 if where.size else N
        assert ln[s] == n and np.array_equal(t1[s, :n], t0[s, :n]) and np.array_equal(l1[s, :n], l0[s, :n])
        assert (t1[s, n:] == stop).all() and not l1[s, n:].any()


def test_ragged_rejects_bad_lengths():
    shape = W.TINY
    gw = sapo.sapo_weights_create(shape, W.make_weights(shape, 31))
    pad = dev(np.zeros((2, 8), np.int32))
    for lens in ([0, 4], [9, 4]):
        with pytest.raises(sapo.SapoError):
            sapo.sapo_rollout_generate_ragged(gw, pad, lens, 2, 4, 1.0, 1)
