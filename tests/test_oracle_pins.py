"""Pins for the CPU oracle: every block is checked against something other than itself
(published vectors, closed forms, brute force in scalar loops, library routines, invariants)."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import sapo_oracle as O
from paper_2509_08721_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny_model(seed=7, gains=True, **kw):
    shape = W.scaled(W.WORKLOADS["tiny"], ).shape
    if kw:
        from dataclasses import replace
        shape = replace(shape, **kw)
    w = W.make_weights(shape, seed)
    if gains:
        w = W.perturb_norm_gains(w, seed)
    return shape, w, O.Model(shape, w)


# ----------------------------------------------------------------------------- RNG
def test_philox_known_answer_vectors():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) if not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        out = O.philox4x32_10(np.array(w[:4], dtype=np.uint32), np.array(w[4:6], dtype=np.uint32))
        assert [int(x) for x in out] == w[6:]


def test_philox_vectorised_equals_scalar_calls():
    rng = np.random.default_rng(0)
    ctr = rng.integers(0, 2**32, size=(50, 4), dtype=np.uint64).astype(np.uint32)
    key = rng.integers(0, 2**32, size=(2,), dtype=np.uint64).astype(np.uint32)
    batch = O.philox4x32_10(ctr, key)
    for i in range(50):
        assert np.array_equal(batch[i], O.philox4x32_10(ctr[i], key))


def test_sampling_stream_keying():
    """Noise is a pure function of (seed, seq, step, v): word v%4 of block v//4, counter
    (v//4, step, seq, 0), key = (seed low, seed high)."""
    seed, seq, step, V = 0x123456789ABCDEF, 5, 9, 37
    bits = O.sampling_uniform_bits(seed, seq, step, V)
    for v in (0, 1, 3, 4, 18, 36):
        blk = O.philox4x32_10(np.array([v // 4, step, seq, 0], dtype=np.uint32),
                              np.array([0x89ABCDEF, 0x01234567], dtype=np.uint32))
        assert bits[v] == blk[v % 4]
    # different seq / step / seed give different streams; longer vocab extends the same stream
    assert not np.array_equal(bits, O.sampling_uniform_bits(seed, seq + 1, step, V))
    assert not np.array_equal(bits, O.sampling_uniform_bits(seed, seq, step + 1, V))
    assert not np.array_equal(bits, O.sampling_uniform_bits(seed + 1, seq, step, V))
    assert np.array_equal(bits, O.sampling_uniform_bits(seed, seq, step, V + 11)[:V])


def test_uniform_open_interval_and_fp32_exact():
    x = np.array([0, 1, 511, 512, 2**32 - 1, 2**31], dtype=np.uint32)
    u = O.uniform_from_bits(x)
    assert u.min() == 2.0 ** -24 and u.max() == 1.0 - 2.0 ** -24
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)


def test_gumbel_moments():
    g = np.concatenate([O.gumbel_noise(42, s, 0, 50000) for s in range(8)]).astype(np.float64)
    n = g.size
    assert abs(g.mean() - 0.5772156649) < 4 * math.sqrt((math.pi ** 2 / 6) / n)
    assert abs(g.var() - math.pi ** 2 / 6) < 0.03
    assert g.min() > -2.82 and g.max() < 16.64


def test_gumbel_max_histogram_matches_softmax():
    """Chi-square of sampled-token counts against softmax(z/T) on a small vocab."""
    rng = np.random.default_rng(3)
    V, T = 12, 0.7
    z = rng.normal(0, 1.5, V)
    p = np.exp(z / T - np.max(z / T))
    p /= p.sum()
    n = 20000
    counts = np.zeros(V)
    for i in range(n):
        counts[O.sample_token(z, T, seed=99, seq=i % 64, step=i // 64)] += 1
    chi2 = np.sum((counts - n * p) ** 2 / (n * p))
    assert chi2 < 36.0          # 11 dof: P(chi2 > 36) ~ 1.6e-4
    # greedy limit
    assert O.sample_token(z, 0.0, 99, 0, 0) == int(np.argmax(z))


def test_argmax_ties_go_to_lowest_id():
    z = np.zeros(8)
    assert O.sample_token(z, 0.0, 1, 0, 0) == 0


# ----------------------------------------------------------------------------- RoPE
def test_rope_closed_forms():
    hd, theta = 16, 1e4
    # position 0 is the identity
    x = np.random.default_rng(0).normal(size=(3, 2, hd))
    assert np.allclose(O.rope_rotate(x, np.zeros(3, dtype=np.int64), theta), x, atol=0)
    # one-hot in slot i rotates into (cos m f_i, sin m f_i) in slots (i, i + hd/2); f_0 = 1
    for i in (0, 3, 7):
        e = np.zeros((1, 1, hd))
        e[0, 0, i] = 1.0
        m = 5
        f = theta ** (-2.0 * i / hd)
        r = O.rope_rotate(e, np.array([m]), theta)[0, 0]
        expect = np.zeros(hd)
        expect[i], expect[i + hd // 2] = math.cos(m * f), math.sin(m * f)
        assert np.allclose(r, expect, atol=1e-15)
    e = np.zeros((1, 1, hd)); e[0, 0, 0] = 1.0
    r = O.rope_rotate(e, np.array([2]), theta)[0, 0]
    assert abs(r[0] - math.cos(2.0)) < 1e-15 and abs(r[8] - math.sin(2.0)) < 1e-15
    # one-hot in the upper half slot rotates the other way round: (-sin, cos)
    e = np.zeros((1, 1, hd)); e[0, 0, 8 + 2] = 1.0
    f = theta ** (-4.0 / hd)
    r = O.rope_rotate(e, np.array([3]), theta)[0, 0]
    assert abs(r[2] + math.sin(3 * f)) < 1e-15 and abs(r[10] - math.cos(3 * f)) < 1e-15
    # norms preserved, inner product depends on m - n only
    q = np.random.default_rng(1).normal(size=(1, 1, hd))
    k = np.random.default_rng(2).normal(size=(1, 1, hd))
    def ip(m, n):
        return float(np.sum(O.rope_rotate(q, np.array([m]), theta) * O.rope_rotate(k, np.array([n]), theta)))
    assert abs(np.linalg.norm(O.rope_rotate(q, np.array([77]), theta)) - np.linalg.norm(q)) < 1e-12
    assert abs(ip(9, 4) - ip(1009, 1004)) < 1e-9
    assert abs(ip(9, 4) - ip(4, 9)) > 1e-3       # sign of the relative offset matters


# ----------------------------------------------------------------------------- attention
def brute_attention(q, k, v, q_pos0):
    """Scalar-loop softmax attention with an explicit probability row."""
    nq, hq, hd = q.shape
    nk, hkv, _ = k.shape
    rep = hq // hkv
    out = np.zeros((nq, hq, hd))
    for i in range(nq):
        for h in range(hq):
            kvh = h // rep
            sc = []
            for n in range(nk):
                if n <= q_pos0 + i:
                    sc.append(sum(q[i, h, e] * k[n, kvh, e] for e in range(hd)) / math.sqrt(hd))
            mx = max(sc)
            w = [math.exp(x - mx) for x in sc]
            tot = sum(w)
            for n, wn in enumerate(w):
                for e in range(hd):
                    out[i, h, e] += wn / tot * v[n, kvh, e]
    return out


def test_attention_vs_brute_force_gqa():
    rng = np.random.default_rng(5)
    q = rng.normal(size=(6, 4, 8))
    k = rng.normal(size=(9, 2, 8))
    v = rng.normal(size=(9, 2, 8))
    v[:, 1, :] += 100.0                    # KV heads differ wildly: a wrong head mapping shows
    got = O.attention(q, k, v, q_pos0=3)
    assert np.allclose(got, brute_attention(q, k, v, 3), atol=1e-12)
    assert np.all(got[:, :2, :] < 50) and np.all(got[:, 2:, :] > 50)   # heads 0,1 -> KV0; 2,3 -> KV1


def test_attention_vs_torch_sdpa():
    rng = np.random.default_rng(6)
    T, hq, hkv, hd = 10, 6, 2, 16
    q, k, v = rng.normal(size=(T, hq, hd)), rng.normal(size=(T, hkv, hd)), rng.normal(size=(T, hkv, hd))
    got = O.attention(q, k, v, 0)
    tq, tk, tv = (torch.from_numpy(a).permute(1, 0, 2)[None] for a in (q, k, v))
    tk = tk.repeat_interleave(hq // hkv, dim=1)
    tv = tv.repeat_interleave(hq // hkv, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.allclose(got, ref, atol=1e-12)


# ----------------------------------------------------------------------------- small blocks vs library
def test_rmsnorm_silu_logsoftmax_vs_torch():
    rng = np.random.default_rng(8)
    h, g = rng.normal(size=(5, 64)), rng.normal(size=64)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(h), (64,), torch.from_numpy(g), eps=1e-6).numpy()
    assert np.allclose(O.rmsnorm(h, g, 1e-6), ref, atol=1e-13)
    x = rng.normal(size=100) * 5
    assert np.allclose(O.silu(x), torch.nn.functional.silu(torch.from_numpy(x)).numpy(), atol=1e-14)
    z = rng.normal(size=(3, 50)) * 30
    lp = O.log_softmax(z)
    assert np.allclose(lp, torch.log_softmax(torch.from_numpy(z), -1).numpy(), atol=1e-12)
    assert np.allclose(np.exp(lp).sum(-1), 1.0, atol=1e-12)
    zz = np.array([[1000.0, -1000.0, 0.0]])          # extreme logits stay finite
    assert np.isfinite(O.log_softmax(zz)).all()


def test_round_bf16():
    x = np.array([1.0, 1.00390625, 1.005859375, 1.001953125, -3.14159, 1e-30, 65504.0])
    r = O.round_bf16(x)
    ref = torch.from_numpy(x).float().bfloat16().double().numpy()
    assert np.array_equal(r, ref)
    # ties to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> 1 ; 1 + 3*2^-8 -> 1 + 2^-6
    assert O.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert O.round_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6


# ----------------------------------------------------------------------------- whole forward
def scalar_forward(shape, wf, tokens):
    """Independent scalar-loop forward of the decoder (brute force on tiny inputs)."""
    d, hq, hkv, hd, F = shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ff
    T = len(tokens)

    def norm(vec, g):
        ms = sum(x * x for x in vec) / len(vec)
        return [x / math.sqrt(ms + shape.rms_eps) * float(gi) for x, gi in zip(vec, g)]

    def matvec(Wm, x):
        return [sum(float(Wm[o][i]) * x[i] for i in range(len(x))) for o in range(len(Wm))]

    def rot(vec, pos):
        out = list(vec)
        for i in range(hd // 2):
            ang = pos * shape.rope_theta ** (-2.0 * i / hd)
            a, b = vec[i], vec[i + hd // 2]
            out[i] = a * math.cos(ang) - b * math.sin(ang)
            out[i + hd // 2] = b * math.cos(ang) + a * math.sin(ang)
        return out

    hs = [[float(x) for x in wf["embed"][t]] for t in tokens]
    for lw in wf["layers"]:
        qs, ks, vs = [], [], []
        for t in range(T):
            a = norm(hs[t], lw["attn_norm"])
            q, k, v = matvec(lw["wq"], a), matvec(lw["wk"], a), matvec(lw["wv"], a)
            if "bq" in lw:
                q = [x + float(b) for x, b in zip(q, lw["bq"])]
                k = [x + float(b) for x, b in zip(k, lw["bk"])]
                v = [x + float(b) for x, b in zip(v, lw["bv"])]
            qs.append([rot(q[h * hd:(h + 1) * hd], t) for h in range(hq)])
            ks.append([rot(k[h * hd:(h + 1) * hd], t) for h in range(hkv)])
            vs.append([v[h * hd:(h + 1) * hd] for h in range(hkv)])
        for t in range(T):
            o = []
            for h in range(hq):
                kh = h // (hq // hkv)
                sc = [sum(qs[t][h][e] * ks[n][kh][e] for e in range(hd)) / math.sqrt(hd) for n in range(t + 1)]
                mx = max(sc)
                ws = [math.exp(x - mx) for x in sc]
                tot = sum(ws)
                o += [sum(ws[n] / tot * vs[n][kh][e] for n in range(t + 1)) for e in range(hd)]
            proj = matvec(lw["wo"], o)
            hs[t] = [x + y for x, y in zip(hs[t], proj)]
        for t in range(T):
            b = norm(hs[t], lw["ffn_norm"])
            gt, up = matvec(lw["w_gate"], b), matvec(lw["w_up"], b)
            act = [g / (1.0 + math.exp(-g)) * u for g, u in zip(gt, up)]
            dn = matvec(lw["w_down"], act)
            hs[t] = [x + y for x, y in zip(hs[t], dn)]
    lm = wf["embed"] if wf["lm_head"] is None else wf["lm_head"]
    return np.array([matvec(lm, norm(hs[t], wf["final_norm"])) for t in range(T)])


def test_forward_vs_scalar_loops():
    from dataclasses import replace
    shape = replace(W.TINY, n_layers=2, d_model=16, n_q_heads=4, n_kv_heads=2, head_dim=4, d_ff=12, vocab=20)
    w = W.perturb_norm_gains(W.make_weights(shape, 11, std=0.3), 11)
    m = O.Model(shape, w)
    tokens = np.array([3, 19, 0, 7, 7, 12])
    got = O.forward_logits(m, tokens)
    ref = scalar_forward(shape, W.weights_as_f32(shape, w), tokens)
    assert np.allclose(got, ref, atol=1e-12)


def test_qkv_bias_scalar_loops_and_closed_form():
    from dataclasses import replace
    shape = replace(W.TINY, n_layers=2, d_model=16, n_q_heads=4, n_kv_heads=2, head_dim=4, d_ff=12, vocab=20)
    w0 = W.perturb_norm_gains(W.make_weights(shape, 11, std=0.3), 11)
    w = W.add_qkv_bias(w0, shape, 5, std=0.5)
    tokens = np.array([3, 19, 0, 7, 7, 12])
    got = O.forward_logits(O.Model(shape, w), tokens)
    ref = scalar_forward(shape, W.weights_as_f32(shape, w), tokens)
    assert np.allclose(got, ref, atol=1e-12)
    assert np.abs(got - O.forward_logits(O.Model(shape, w0), tokens)).max() > 1e-3      # the biases matter
    # zero biases are no biases
    wz = W.add_qkv_bias(w0, shape, 5, std=0.0)
    assert np.array_equal(O.forward_logits(O.Model(shape, wz), tokens), O.forward_logits(O.Model(shape, w0), tokens))
    # closed form: with wq = wk = wv = 0 every key and value is the bias itself, so attention returns bv of the
    # head's KV group whatever the scores are, and one layer adds wo . repeat(bv) to the residual
    one = replace(shape, n_layers=1)
    w1 = W.add_qkv_bias(W.make_weights(one, 3, std=0.3), one, 9, std=0.7)
    lw = w1["layers"][0]
    for k in ("wq", "wk", "wv", "w_down"):
        lw[k] = np.zeros_like(lw[k])
    m = O.Model(one, w1)
    h = O.hidden_states(m, tokens)
    f = W.weights_as_f32(one, w1)
    rep = one.n_q_heads // one.n_kv_heads
    o = np.concatenate([np.asarray(lw["bv"], np.float64)[(hh // rep) * one.head_dim:(hh // rep + 1) * one.head_dim]
                        for hh in range(one.n_q_heads)])
    expect = np.asarray(f["embed"], np.float64)[tokens] + np.asarray(f["layers"][0]["wo"], np.float64) @ o
    assert np.allclose(h, O.rmsnorm(expect, np.asarray(f["final_norm"], np.float64), one.rms_eps), atol=1e-12)


def test_zero_layer_model_is_norm_times_embedding():
    from dataclasses import replace
    shape = replace(W.TINY, n_layers=0)
    w = W.perturb_norm_gains(W.make_weights(shape, 13), 13)
    m = O.Model(shape, w)
    tokens = np.array([5, 400, 5])
    z = O.forward_logits(m, tokens)
    E = w["embed"].astype(np.float64)
    for i, t in enumerate(tokens):
        e = E[t]
        x = e / math.sqrt(np.mean(e * e) + 1e-6) * w["final_norm"]
        assert np.allclose(z[i], E @ x, atol=1e-13)
    assert np.allclose(z[0], z[2])      # no layers: no position dependence


def test_causality_and_batch_invariance():
    shape, w, m = tiny_model()
    rng = np.random.default_rng(17)
    toks = rng.integers(0, shape.vocab, size=12)
    z = O.forward_logits(m, toks)
    toks2 = toks.copy(); toks2[8:] = (toks2[8:] + 1) % shape.vocab
    z2 = O.forward_logits(m, toks2)
    assert np.array_equal(z[:8], z2[:8]) and not np.allclose(z[8:], z2[8:])
    # a sequence scored alone equals its row in a batch
    batch = rng.integers(0, shape.vocab, size=(3, 12)).astype(np.int32)
    mask = W.make_completion_mask(3, 12, 6)
    full = O.score_logprobs(m, batch, mask)
    alone = O.score_logprobs(m, batch[1:2], mask[1:2])
    assert np.array_equal(full[1], alone[0])


def test_kv_cache_decode_equals_full_recompute():
    wl = W.WORKLOADS["tiny"]
    shape, w, m = tiny_model(seed=wl.weight_seed)
    prompts = W.make_prompts(wl)
    toks, lps, zs = O.rollout_generate(m, prompts, wl.group, wl.n_new, 1.0, wl.rollout_seed, return_logits=True)
    assert toks.shape == (8, 16) and toks.min() >= 0 and toks.max() < shape.vocab
    for s in range(wl.n_seqs):
        seq = np.concatenate([prompts[s // wl.group], toks[s]])
        zfull = O.forward_logits(m, seq, at=range(wl.prompt_len - 1, wl.prompt_len + wl.n_new - 1))
        assert np.allclose(zfull, zs[s], atol=1e-10)
        for t in range(wl.n_new):          # tokens re-derived from the recomputed logits are identical
            assert O.sample_token(zfull[t], 1.0, wl.rollout_seed, s, t) == toks[s, t]
    # rollout log-probs are what the scoring pass gives on the same sequences
    seqs = np.concatenate([np.repeat(prompts, wl.group, axis=0), toks], axis=1)
    mask = W.make_completion_mask(wl.n_seqs, wl.prompt_len + wl.n_new, wl.n_new)
    sc = O.score_logprobs(m, seqs, mask)
    assert np.allclose(sc[:, wl.prompt_len:], lps, atol=1e-6)
    assert np.all(sc[:, :wl.prompt_len] == 0.0)
    # siblings share the step-0 logits but draw different noise
    assert np.allclose(zs[0, 0], zs[1, 0], atol=0) and len({tuple(t) for t in toks}) > 1


def test_score_logprobs_properties():
    shape, w, m = tiny_model()
    rng = np.random.default_rng(21)
    toks = rng.integers(0, shape.vocab, size=(2, 10)).astype(np.int32)
    mask = np.ones((2, 10), dtype=np.uint8)
    lp = O.score_logprobs(m, toks, mask)
    assert np.all(lp[:, 0] == 0.0)                  # t = 0 is never scorable
    assert np.all(lp[:, 1:] < 0.0) and np.isfinite(lp).all()
    # each entry equals the log-softmax of the definition; probabilities over the vocab sum to 1
    for s in range(2):
        z = O.forward_logits(m, toks[s])
        full = O.log_softmax(z)
        assert np.allclose(np.exp(full).sum(-1), 1.0, atol=1e-12)
        for t in range(1, 10):
            assert abs(lp[s, t] - full[t - 1, toks[s, t]]) < 1e-6
    # an unlikely continuation (argmin of the logits) is scored finite and very negative
    z = O.forward_logits(m, toks[0, :5])
    worst = toks[0].copy(); worst[5] = int(np.argmin(z[4]))
    lpw = O.score_logprobs(m, worst[None], mask[:1])
    assert np.isfinite(lpw).all() and lpw[0, 5] <= lp[0, 5]
    # mask selects entries, does not change them
    mask2 = mask.copy(); mask2[:, ::2] = 0
    lp2 = O.score_logprobs(m, toks, mask2)
    assert np.array_equal(lp2[:, 1::2], lp[:, 1::2]) and np.all(lp2[:, ::2] == 0.0)


def test_temperature_changes_sampling_not_logprob_definition():
    shape, w, m = tiny_model()
    prompts = np.random.default_rng(2).integers(0, shape.vocab, size=(1, 6)).astype(np.int32)
    t0, l0 = O.rollout_generate(m, prompts, 2, 5, 0.0, seed=1)
    assert np.array_equal(t0[0], t0[1])             # greedy: siblings identical
    z = O.forward_logits(m, prompts[0])[-1]
    assert t0[0, 0] == int(np.argmax(z))
    assert abs(l0[0, 0] - O.log_softmax(z)[t0[0, 0]]) < 1e-6
    t7, l7 = O.rollout_generate(m, prompts, 2, 5, 0.7, seed=1)
    assert abs(l7[0, 0] - O.log_softmax(z)[t7[0, 0]]) < 1e-6   # log-prob is at T = 1


# ----------------------------------------------------------------------------- advantages
def test_group_advantages_closed_forms():
    G = 8
    r = np.array([1, 1, 0, 0, 0, 0, 0, 0], dtype=np.float32)        # k = 2 of 8
    a = O.group_advantages(r, G)
    assert np.allclose(a[:2], 1.7320508, atol=1e-5) and np.allclose(a[2:], -0.5773503, atol=1e-5)
    for k in range(1, G):
        r = np.array([1.0] * k + [0.0] * (G - k), dtype=np.float32)
        a = O.group_advantages(np.random.default_rng(k).permutation(r), G).astype(np.float64)
        p = k / G
        sd = math.sqrt(p * (1 - p))
        assert abs(a.sum()) < 1e-5
        assert abs(np.sum(a * a) - G * (sd / (sd + 1e-6)) ** 2) < 1e-4
        assert np.allclose(sorted(set(np.round(a, 5))), sorted({round((0 - p) / (sd + 1e-6), 5), round((1 - p) / (sd + 1e-6), 5)}))
    # equal rewards -> exactly zero (also for values whose mean is not exact in binary)
    for val in (0.0, 1.0, 0.3):
        a = O.group_advantages(np.full(8, val, dtype=np.float32), 8)
        assert np.all(a == 0.0)
    assert np.all(O.group_advantages(np.array([0.7, 0.1], dtype=np.float32), 1) == 0.0)   # G = 1
    # groups are independent runs of G consecutive sequences
    r = np.array([1, 0, 0, 0, 1, 1, 1, 0], dtype=np.float32)
    a = O.group_advantages(r, 4)
    assert np.allclose(a[:4], O.group_advantages(r[:4], 4)) and np.allclose(a[4:], O.group_advantages(r[4:], 4))
    # vs library: (r - mean) / (std + eps), population std
    r = np.random.default_rng(0).random(16).astype(np.float32)
    t = torch.from_numpy(r).double().reshape(2, 8)
    ref = ((t - t.mean(1, keepdim=True)) / (t.std(1, unbiased=False, keepdim=True) + 1e-6)).reshape(-1).numpy()
    assert np.allclose(O.group_advantages(r, 8), ref, atol=1e-6)
    # partial credit rewards are accepted (floats, not booleans)
    a = O.group_advantages(np.array([0.5, 1.0, 0.0, 0.5], dtype=np.float32), 4)
    assert abs(a[0]) < 1e-7 and a[1] > 0 > a[2]


# ----------------------------------------------------------------------------- clipped surrogate (Sec. 4.2)
def test_clipped_surrogate_hand_cases():
    # four tokens, one per (sign of A, side of the clip range); values worked by hand
    ln = np.log(np.array([[1.5, 0.5], [1.5, 0.5]]))
    lo = np.zeros((2, 2))
    mask = np.ones((2, 2), dtype=np.uint8)
    adv = np.array([1.0, -1.0])
    loss, g = O.clipped_surrogate_loss(ln, lo, mask, adv, 0.2, 0.28)
    # A=+1: rho 1.5 -> clipped 1.28 (flat), rho 0.5 -> 0.5 (unclipped is smaller)
    # A=-1: rho 1.5 -> -1.5 (unclipped is smaller), rho 0.5 -> -0.8 (clipped, flat)
    assert loss == pytest.approx(-(1.28 + 0.5 - 1.5 - 0.8) / 4, abs=1e-15)
    np.testing.assert_allclose(g, np.array([[0.0, -0.5 / 4], [1.5 / 4, 0.0]]), atol=1e-15)


def test_clipped_surrogate_on_policy_is_minus_mean_advantage():
    rng = np.random.default_rng(3)
    lp = rng.normal(-2.0, 1.0, (6, 9))
    mask = rng.random((6, 9)) < 0.6
    adv = rng.normal(0, 1, 6)
    loss, g = O.clipped_surrogate_loss(lp, lp, mask, adv)
    n = mask.sum()
    assert loss == pytest.approx(-(adv[:, None] * mask).sum() / n, abs=1e-14)
    np.testing.assert_allclose(g, -(adv[:, None] * mask) / n, atol=1e-15)


def test_clipped_surrogate_vs_torch_autograd_and_masking():
    rng = np.random.default_rng(11)
    S, T = 8, 16
    lo = rng.normal(-2.0, 1.0, (S, T))
    ln = lo + rng.normal(0, 0.25, (S, T))           # ratios on both sides of both clip bounds
    mask = rng.random((S, T)) < 0.5
    adv = rng.normal(0, 1, S)
    loss, g = O.clipped_surrogate_loss(ln, lo, mask, adv, 0.2, 0.28)
    x = torch.tensor(ln, dtype=torch.float64, requires_grad=True)
    rho = torch.exp(x - torch.tensor(lo))
    a = torch.tensor(adv)[:, None]
    term = torch.minimum(rho * a, torch.clamp(rho, 1 - 0.2, 1 + 0.28) * a)
    m = torch.tensor(mask)
    tl = -(term * m).sum() / m.sum()
    tl.backward()
    assert loss == pytest.approx(float(tl.detach()), abs=1e-14)
    np.testing.assert_allclose(g, x.grad.numpy(), atol=1e-14)
    assert (np.abs(g) > 0).sum() < mask.sum()       # some tokens really are clipped
    # what sits under a zero mask never matters
    ln2, lo2 = ln.copy(), lo.copy()
    ln2[~mask] = np.nan
    lo2[~mask] = np.inf
    loss2, g2 = O.clipped_surrogate_loss(ln2, lo2, mask, adv, 0.2, 0.28)
    assert loss2 == loss and np.array_equal(g2, g)
    # nothing masked: zero loss, zero gradient
    l0, g0 = O.clipped_surrogate_loss(ln, lo, np.zeros((S, T), bool), adv)
    assert l0 == 0.0 and not g0.any()


def test_clipped_surrogate_gradient_is_the_derivative():
    rng = np.random.default_rng(5)
    S, T = 4, 6
    lo = rng.normal(-2.0, 1.0, (S, T))
    ln = lo + rng.normal(0, 0.3, (S, T))
    mask = np.ones((S, T), bool)
    adv = rng.normal(0, 1, S)
    _, g = O.clipped_surrogate_loss(ln, lo, mask, adv)
    h = 1e-6
    for s in range(S):
        for t in range(T):
            rho = math.exp(ln[s, t] - lo[s, t])
            if min(abs(rho - 0.8), abs(rho - 1.28)) < 1e-3:
                continue                              # a kink
            up, dn = ln.copy(), ln.copy()
            up[s, t] += h
            dn[s, t] -= h
            fd = (O.clipped_surrogate_loss(up, lo, mask, adv)[0] - O.clipped_surrogate_loss(dn, lo, mask, adv)[0]) / (2 * h)
            assert g[s, t] == pytest.approx(fd, abs=1e-8)


# ----------------------------------------------------------------------------- training-set assembly (Sec. 3.2)
def test_uniform_subset_is_uniform_and_respects_eligibility():
    elig = np.array([1, 0, 1, 1, 0, 1, 1, 1, 0, 1], bool)          # 7 eligible of 10
    k, trials = 3, 6000
    hits = np.zeros(10)
    first = np.zeros(10)
    pairs = np.zeros((10, 10))
    for seed in range(trials):
        s = O.uniform_subset(elig, k, seed * 7919 + 1, O.STREAM_EXTERNAL)
        assert len(s) == k and len(set(s.tolist())) == k and elig[s].all()
        hits[s] += 1
        first[s[0]] += 1
        for a in s:
            for b in s:
                if a < b:
                    pairs[a, b] += 1
    p = k / 7
    sd = math.sqrt(trials * p * (1 - p))
    assert (np.abs(hits[elig] - trials * p) < 4.5 * sd).all()        # marginal inclusion probability k / E
    assert not hits[~elig].any()
    assert (np.abs(first[elig] - trials / 7) < 4.5 * math.sqrt(trials / 7 * 6 / 7)).all()   # order is uniform too
    pp = k * (k - 1) / (7 * 6)                                        # pair inclusion of a uniform k-subset
    e = np.nonzero(elig)[0]
    for i, a in enumerate(e):
        for b in e[i + 1:]:
            assert abs(pairs[a, b] - trials * pp) < 4.5 * math.sqrt(trials * pp * (1 - pp))


def test_uniform_subset_edges_and_streams():
    elig = np.ones(6, bool)
    assert sorted(O.uniform_subset(elig, 6, 5, 1).tolist()) == list(range(6))       # k = E: everything
    assert sorted(O.uniform_subset(elig, 9, 5, 1).tolist()) == list(range(6))       # k > E: everything, no more
    assert len(O.uniform_subset(elig, 0, 5, 1)) == 0
    assert len(O.uniform_subset(np.zeros(6, bool), 3, 5, 1)) == 0
    a, b = O.uniform_subset(np.ones(64, bool), 64, 5, 1), O.uniform_subset(np.ones(64, bool), 64, 5, 2)
    assert not np.array_equal(a, b)                                                 # streams differ
    assert np.array_equal(a, O.uniform_subset(np.ones(64, bool), 64, 5, 1))         # and are reproducible
    # the keys are the generator's published stream, not the token sampler's (counter word 3 differs)
    k = O.subset_keys(5, 1, 4)
    ref = O.philox4x32_10(np.array([[2, 0, 0, 1]], np.uint32), np.array([5, 0], np.uint32))[0, 0]
    assert k[2] == ref and k[2] != O.sampling_uniform_bits(5, 0, 0, 12)[8]


def test_assemble_training_set_structure():
    rng = np.random.default_rng(2)
    G, T = 4, 9
    lt = rng.integers(0, 1000, (5 * G, T)).astype(np.int32)
    et = rng.integers(1000, 2000, (6 * G, T)).astype(np.int32)
    lr = rng.integers(0, 2, 5 * G).astype(np.float32)
    er = rng.integers(0, 2, 6 * G).astype(np.float32)
    er[0:G] = 1.0           # external datapoint 0: all right  -> zero advantage
    er[2 * G:3 * G] = 0.0   # external datapoint 2: all wrong  -> zero advantage
    er[G:2 * G] = [1, 0, 0, 0]; er[3 * G:4 * G] = [0, 1, 1, 0]; er[4 * G:5 * G] = [1, 1, 0, 1]; er[5 * G:] = [0, 0, 1, 0]
    tok, rew, src, (nl, ne) = O.assemble_training_set(lt, lr, et, er, G, 3, 5, seed=77)
    assert (nl, ne) == (3, 4)                       # only 4 external datapoints have a non-zero advantage
    assert tok.shape == (8 * G, T) and src.shape == (8,)
    assert sorted(src[3:7].tolist()) == [5 + 1, 5 + 3, 5 + 4, 5 + 5] and src[7] == -1
    assert len(set(src[:3].tolist())) == 3 and all(0 <= g < 5 for g in src[:3])
    for slot, g in enumerate(src):
        rows = slice(slot * G, (slot + 1) * G)
        if g < 0:
            assert not tok[rows].any() and not rew[rows].any()
        elif g < 5:
            assert np.array_equal(tok[rows], lt[g * G:(g + 1) * G]) and np.array_equal(rew[rows], lr[g * G:(g + 1) * G])
        else:
            h = g - 5
            assert np.array_equal(tok[rows], et[h * G:(h + 1) * G]) and np.array_equal(rew[rows], er[h * G:(h + 1) * G])
    # every selected external group has a non-zero advantage under the scoring call's own definition
    adv = O.group_advantages(rew, G)
    for slot in range(3, 7):
        assert np.abs(adv[slot * G:(slot + 1) * G]).max() > 0
    # J = 0 reduces to the node's own rollouts (the paper's remark on standard RL fine-tuning)
    tok0, _, src0, (nl0, ne0) = O.assemble_training_set(lt, lr, et, er, G, 5, 0, seed=77)
    assert (nl0, ne0) == (5, 0) and sorted(src0.tolist()) == [0, 1, 2, 3, 4]


# ----------------------------------------------------------------------------- stop token
def test_stop_token_rows_are_prefixes_of_unstopped_rows():
    shape, w, m = tiny_model(seed=4)
    prompts = np.random.default_rng(0).integers(0, shape.vocab, size=(2, 6))
    G, N, seed = 3, 24, 9
    tok, lp = O.rollout_generate(m, prompts, G, N, 1.0, seed)
    # a stop token that some rows do sample and some do not
    vals, counts = np.unique(tok[:, 2:N - 2], return_counts=True)
    stop = int(vals[np.argmax(counts)])
    t2, l2, ln = O.rollout_generate_stop(m, prompts, G, N, 1.0, seed, stop)
    hit = 0
    for s in range(tok.shape[0]):
        where = np.nonzero(tok[s] == stop)[0]
        n = int(where[0]) + 1 if where.size else N
        hit += bool(where.size)
        assert ln[s] == n
        assert np.array_equal(t2[s, :n], tok[s, :n]) and np.array_equal(l2[s, :n], lp[s, :n])
        assert (t2[s, n:] == stop).all() and not l2[s, n:].any()
    assert 0 < hit
    # a token nobody samples: identical to the unstopped call
    unused = next(v for v in range(shape.vocab) if v not in set(tok.ravel().tolist()))
    t3, l3, ln3 = O.rollout_generate_stop(m, prompts, G, N, 1.0, seed, unused)
    assert np.array_equal(t3, tok) and np.array_equal(l3, lp) and (ln3 == N).all()


# ----------------------------------------------------------------------------- prompts of different lengths
def test_ragged_rollout_reduces_to_the_batch_call_and_ignores_padding():
    shape, w, m = tiny_model(seed=4)
    rng = np.random.default_rng(0)
    G, N, seed = 2, 6, 9
    same = rng.integers(0, shape.vocab, size=(3, 7))
    t0, l0 = O.rollout_generate(m, same, G, N, 1.0, seed)
    t1, l1 = O.rollout_generate_ragged(m, [same[0], same[1], same[2]], G, N, 1.0, seed)
    assert np.array_equal(t0, t1) and np.array_equal(l0, l1)
    # a prompt's rows depend on its own tokens and its sequence indices only
    rag = [same[0][:3], same[1], same[2][:5]]
    t2, l2 = O.rollout_generate_ragged(m, rag, G, N, 1.0, seed)
    assert np.array_equal(t2[G:2 * G], t0[G:2 * G]) and np.array_equal(l2[G:2 * G], l0[G:2 * G])
    assert not np.array_equal(t2[:G], t0[:G])
    t3, _ = O.rollout_generate(m, same[2][None, :5], G, N, 1.0, seed, first_seq=2 * G)
    assert np.array_equal(t3, t2[2 * G:])


# ----------------------------------------------------------------------------- scoring at a temperature
def test_score_logprobs_at_a_temperature():
    shape, w, m = tiny_model(seed=6)
    rng = np.random.default_rng(1)
    toks = rng.integers(0, shape.vocab, size=(2, 9))
    mask = np.ones((2, 9), np.uint8)
    base = O.score_logprobs(m, toks, mask)
    assert np.array_equal(O.score_logprobs(m, toks, mask, temperature=1.0), base)
    for temp in (0.5, 0.7, 3.0):
        lp = O.score_logprobs(m, toks, mask, temperature=temp)
        # library routine on the teacher-forced logits
        for s in range(2):
            z = O.forward_logits(m, toks[s])
            ref = torch.log_softmax(torch.tensor(z) / temp, dim=-1).numpy()
            assert np.allclose(lp[s, 1:], ref[np.arange(8), toks[s, 1:]], atol=1e-6)
        assert not np.allclose(lp[:, 1:], base[:, 1:], atol=1e-3)
    # a very high temperature flattens the distribution to uniform over the vocabulary
    hot = O.score_logprobs(m, toks, mask, temperature=1e9)
    assert np.allclose(hot[:, 1:], -math.log(shape.vocab), atol=1e-6)
    # a low temperature sharpens it: the greedy token's log-prob tends to 0
    z = O.forward_logits(m, toks[0])
    greedy = toks[0].copy()
    greedy[1:] = np.argmax(z[:-1], axis=-1)
    z2 = O.forward_logits(m, greedy[:2])
    g2 = np.array([[greedy[0], int(np.argmax(z2[0]))]])
    assert O.score_logprobs(m, g2, np.ones((1, 2), np.uint8), temperature=1e-3)[0, 1] > -1e-3
