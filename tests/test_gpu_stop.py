"""Rollouts with a stop token against the oracle (fp32: exact tokens and lengths) and against the plain call;
ended sequences leaving the decode batch (MFMA path, more than 64 sequences)."""
import contextlib
import os

import numpy as np
import pytest
import torch

from oracle import sapo_oracle as O
from paper_2509_08721_amd import sapo, workloads as W

pytestmark = pytest.mark.gpu


@contextlib.contextmanager
def no_compaction():
    """The library keeps ended sequences in the batch while this is set (read at every call)."""
    os.environ["SAPO_NO_COMPACT"] = "1"
    try:
        yield
    finally:
        del os.environ["SAPO_NO_COMPACT"]


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
        with no_compaction():    # same rows per step as the plain call, hence the same kernels: exact equality
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


@pytest.mark.parametrize("P,N,boost,ragged,levels", [(12, 120, 3, False, [64]), (12, 120, 3, True, [64]),
                                                     (40, 130, 6, False, [256, 64])])
def test_ended_sequences_leave_the_batch(P, N, boost, ragged, levels):
    """More than 64 sequences on the MFMA path, a stop token whose logit swings widely (lengths from a few tokens
    to max_new): once the running sequences fit 256 / 64 rows the step goes on with that many rows.  Every row
    must still be the sample of its own sequence: checked per step against the oracle (teacher-forced, near-tie
    band of the bf16 path), log-probs to 2e-2, and against the same call with compaction off (identical up to the
    first look at step 32; later rows come from other kernels and may part at near-ties)."""
    from tests.parity import measured_logit_eps, oracle_logprobs_for, teacher_forced_token_check
    shape, G, Lp, stop, seed = W.MINI_BF16, 8, 16, 77, 5
    S = P * G
    w = W.boost_token(W.perturb_norm_gains(W.make_weights(shape, 7, std=0.05), 7), shape, stop, boost)
    gw = sapo.sapo_weights_create(shape, w)
    assert gw.uses_mfma
    rng = np.random.default_rng(1)
    prompts_np = rng.integers(0, shape.vocab, size=(P, Lp)).astype(np.int32)
    lens = rng.integers(3, Lp + 1, size=P).tolist() if ragged else None
    prompts = torch.from_numpy(prompts_np).cuda()

    def run(stream):
        if ragged:
            t, l, n = sapo.sapo_rollout_generate_ragged(gw, prompts, lens, G, N, 1.0, seed, stop_token=stop, stream=stream)
        else:
            t, l, n = sapo.sapo_rollout_generate_stop(gw, prompts, G, N, 1.0, seed, stop, stream=stream)
        torch.cuda.synchronize()
        return t.cpu().numpy(), l.cpu().numpy(), n.cpu().numpy(), sapo.sapo_rollout_last_stats(gw)

    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        with no_compaction():
            t0, l0, n0, stats0 = run(st)
        t1, l1, n1, stats1 = run(st)            # replayed graphs, one per batch size
        t2, l2, n2, stats2 = run(st)            # and again: the cached graphs serve the next call
    t3, l3, n3, stats3 = run(None)              # eager launches
    assert stats0["compactions"] == 0 and stats0["rows"] == S
    assert stats1["compactions"] == len(levels) and stats1["rows"] == levels[-1], (stats0, stats1)
    assert stats1 == stats2 == stats3
    for t, l, n in ((t2, l2, n2), (t3, l3, n3)):
        assert np.array_equal(t, t1) and np.array_equal(n, n1) and np.array_equal(l.view(np.uint32), l1.view(np.uint32))
    # the shape of a result: a row is its sequence's tokens up to the first stop token, then padding
    for t, l, n in ((t0, l0, n0), (t1, l1, n1)):
        for s in range(S):
            k = int(n[s])
            assert 1 <= k <= N and not (t[s, :k - 1] == stop).any()
            assert (t[s, k - 1] == stop) or k == N
            assert (t[s, k:] == stop).all() and not l[s, k:].any() and (l[s, :k] <= 0).all()
    assert (n1 < 32).any() and (n1 == N).sum() >= 8          # the lengths are spread out
    # up to the first look the two calls ran the same kernels on the same rows
    first = np.minimum(n0, 32)
    assert np.array_equal(first, np.minimum(n1, 32))
    for s in range(S):
        assert np.array_equal(t0[s, :first[s]], t1[s, :first[s]]) and np.array_equal(l0[s, :first[s]], l1[s, :first[s]])
    same_rows = sum(bool(np.array_equal(t0[s], t1[s])) for s in range(S))
    assert same_rows >= 0.8 * S, same_rows
    # against the oracle: the longest-running sequences (they went through every batch size) and two short ones
    order = np.argsort(n1, kind="stable")
    seqs = sorted({int(order[-1]), int(order[-2]), int(order[-3]), int(order[0]), int(order[S // 2])})
    ma = O.Model(shape, w)
    n_checked = n_exact = 0
    for s in seqs:
        k = int(n1[s])
        pr = prompts_np if not ragged else None
        if ragged:      # the oracle's helpers take equal-length prompts: sequence s alone, its prompt cut to length
            p_one = prompts_np[s // G: s // G + 1, :lens[s // G]]
            band = 1e-3 + 2 * measured_logit_eps(sapo, gw, ma, np.concatenate([p_one[0], t1[s, :k]]), p_one.shape[1] - 1)
            nn, ex, near, bad = teacher_forced_token_check_one(ma, p_one, t1[s], seed, s, k, band)
            ref = oracle_logprobs_one(ma, p_one[0], t1[s, :k])
        else:
            band = 1e-3 + 2 * measured_logit_eps(sapo, gw, ma, np.concatenate([pr[s // G], t1[s, :k]]), pr.shape[1] - 1)
            nn, ex, near, bad = teacher_forced_token_check(ma, pr, G, t1[:, :k], 1.0, seed, [s], delta=band)
            ref = oracle_logprobs_for(ma, pr, G, t1[:, :k], [s])[s]
        assert not bad, bad[:5]
        n_checked += nn
        n_exact += ex
        assert np.max(np.abs(ref - l1[s, :k])) <= 2e-2
    assert n_checked - n_exact <= max(2, 0.05 * n_checked)
    gw.close()


def teacher_forced_token_check_one(model, prompt_row, gpu_row, seed, s, k, delta):
    """teacher_forced_token_check for one sequence with its own prompt length (noise keyed on the sequence index s)."""
    Lp = prompt_row.shape[1]
    seq = np.concatenate([prompt_row[0], gpu_row[:k]])
    z = O.forward_logits(model, seq[: Lp + k - 1], at=[Lp - 1 + t for t in range(k)])
    n = exact = 0
    near, bad = [], []
    for t in range(k):
        y = O.perturbed_scores(z[t], 1.0, seed, s, t)
        v_star, v_gpu = int(np.argmax(y)), int(gpu_row[t])
        n += 1
        if v_star == v_gpu:
            exact += 1
            continue
        gap = float(y[v_star]) - float(y[v_gpu])
        (near if gap <= delta else bad).append((s, t, v_star, v_gpu, gap))
    return n, exact, near, bad


def oracle_logprobs_one(model, prompt, gpu_row):
    Lp, k = len(prompt), len(gpu_row)
    seq = np.concatenate([prompt, gpu_row])
    z = O.forward_logits(model, seq[:-1], at=range(Lp - 1, Lp + k - 1))
    return O.log_softmax(z)[np.arange(k), gpu_row]


def test_stop_token_bad_arguments():
    wl = W.WORKLOADS["tiny"]
    gw = sapo.sapo_weights_create(wl.shape, W.make_weights(wl.shape, wl.weight_seed))
    prompts = torch.from_numpy(W.make_prompts(wl)).cuda()
    for bad in (-1, wl.shape.vocab):
        with pytest.raises(sapo.SapoError):
            sapo.sapo_rollout_generate_stop(gw, prompts, wl.group, 4, 1.0, 1, bad)
