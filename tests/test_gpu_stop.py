"""Rollouts with a stop token against the oracle (fp32: exact tokens and lengths) and against the plain call."""
import numpy as np
import pytest
import torch

from oracle import sapo_oracle as O
from paper_2509_08721_amd import sapo, workloads as W

pytestmark = pytest.mark.gpu


def frequent_token(tok, lo, hi):
    vals, counts = np.unique(tok[:, lo:hi], return_counts=True)
    return int(vals[np.argmax(counts)])


def test_stop_token_fp32_matches_oracle():
    wl = W.WORKLOADS["tiny"]
    w = W.make_weights(wl.shape, wl.weight_seed)
    gw = sapo.sapo_weights_create(wl.shape, w)
    m = O.Model(wl.shape, w)
    prompts = W.make_prompts(wl)
    N = 40
    base, _ = O.rollout_generate(m, prompts, wl.group, N, wl.temperature, wl.rollout_seed)
    some_stop = False
    for stop in (frequent_token(base, 1, N - 1), int(base[0, 0]), int(base[-1, N - 1])):
        o_tok, o_lp, o_len = O.rollout_generate_stop(m, prompts, wl.group, N, wl.temperature, wl.rollout_seed, stop)
        some_stop = some_stop or bool((o_len < N).any())
        tok, lp, ln = sapo.sapo_rollout_generate_stop(gw, torch.from_numpy(prompts).cuda(), wl.group, N, wl.temperature,
                                                      wl.rollout_seed, stop)
        assert np.array_equal(tok.cpu().numpy(), o_tok)
        assert np.array_equal(ln.cpu().numpy(), o_len)
        assert np.max(np.abs(lp.cpu().numpy() - o_lp)) <= 1e-4
    assert some_stop


def test_stop_token_everyone_stops_early_fp32():
    # greedy decoding of one prompt: the siblings are identical, all stop at the same early step, and the
    # call returns before max_new steps have run
    wl = W.WORKLOADS["tiny"]
    w = W.make_weights(wl.shape, wl.weight_seed)
    gw = sapo.sapo_weights_create(wl.shape, w)
    m = O.Model(wl.shape, w)
    prompts = W.make_prompts(wl)[:1]
    N = 100
    base, _ = O.rollout_generate(m, prompts, 4, 8, 0.0, 1)
    stop = int(base[0, 3])
    o_tok, o_lp, o_len = O.rollout_generate_stop(m, prompts, 4, N, 0.0, 1, stop)
    assert (o_len <= 4).all()
    for stream in (None, torch.cuda.Stream()):
        tok, lp, ln = sapo.sapo_rollout_generate_stop(gw, torch.from_numpy(prompts).cuda(), 4, N, 0.0, 1, stop, stream=stream)
        torch.cuda.synchronize()
        assert np.array_equal(tok.cpu().numpy(), o_tok) and np.array_equal(ln.cpu().numpy(), o_len)
        assert np.max(np.abs(lp.cpu().numpy() - o_lp)) <= 1e-4


@pytest.mark.parametrize("P,G,Lp,N", [(3, 4, 21, 70), (9, 8, 16, 40)])
def test_stop_token_mfma_rows_are_prefixes_of_the_plain_call(P, G, Lp, N):
    shape = W.MINI_BF16
    gw = sapo.sapo_weights_create(shape, W.make_weights(shape, 7, std=0.05))
    assert gw.uses_mfma
    prompts = torch.from_numpy(np.random.default_rng(1).integers(0, shape.vocab, size=(P, Lp)).astype(np.int32)).cuda()
    st = torch.cuda.Stream()                       # a stream of its own: the decode step is replayed from a graph
    with torch.cuda.stream(st):
        tok, lp = sapo.sapo_rollout_generate(gw, prompts, G, N, 1.0, 5, stream=st)
        st.synchronize()
        tok, lp = tok.cpu().numpy(), lp.cpu().numpy()
        stop = frequent_token(tok, 2, N - 2)
        t2, l2, ln = sapo.sapo_rollout_generate_stop(gw, prompts, G, N, 1.0, 5, stop, stream=st)
        st.synchronize()
        t3, l3 = sapo.sapo_rollout_generate(gw, prompts, G, N, 1.0, 5, stream=st)    # the plain call is unchanged after it
        st.synchronize()
    t2, l2, ln = t2.cpu().numpy(), l2.cpu().numpy(), ln.cpu().numpy()
    assert np.array_equal(t3.cpu().numpy(), tok) and np.array_equal(l3.cpu().numpy(), lp)
    stopped = 0
    for s in range(P * G):
        where = np.nonzero(tok[s] == stop)[0]
        n = int(where[0]) + 1 if where.size else N
        stopped += bool(where.size)
        assert ln[s] == n
        assert np.array_equal(t2[s, :n], tok[s, :n]) and np.array_equal(l2[s, :n], lp[s, :n])
        assert (t2[s, n:] == stop).all() and not l2[s, n:].any()
    assert stopped > 0


def test_stop_token_bad_arguments():
    wl = W.WORKLOADS["tiny"]
    gw = sapo.sapo_weights_create(wl.shape, W.make_weights(wl.shape, wl.weight_seed))
    prompts = torch.from_numpy(W.make_prompts(wl)).cuda()
    for bad in (-1, wl.shape.vocab):
        with pytest.raises(sapo.SapoError):
            sapo.sapo_rollout_generate_stop(gw, prompts, wl.group, 4, 1.0, 1, bad)
