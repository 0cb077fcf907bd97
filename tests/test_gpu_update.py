"""GPU parity of the local policy update (sapo_policy_update) against the update oracle:
log-probs, loss, the gradient of every tensor, the Adam state and the updated parameters."""
import numpy as np
import pytest

from paper_2509_08721_amd import workloads as W

pytestmark = pytest.mark.gpu

from dataclasses import replace

SHAPES = {
    # several 128-position tiles per sequence: the causal shortcuts of the attention products
    "tiny_long": replace(W.TINY, max_seq=512),
    # the tiny configuration's model
    "tiny": W.TINY,
    # sizes that are not multiples of the GEMM tile, untied head, one KV head
    "ragged_untied": W.ModelShape(n_layers=1, d_model=96, n_q_heads=3, n_kv_heads=1, head_dim=32, d_ff=80, vocab=300,
                                  rms_eps=1e-5, rope_theta=1e6, tied_embeddings=False, dtype="f32", max_seq=64),
    # a head dim the fused attention kernels do not take: attention as batched GEMMs over T x T score matrices
    "hd24": W.ModelShape(n_layers=2, d_model=48, n_q_heads=4, n_kv_heads=2, head_dim=24, d_ff=64, vocab=96,
                         rms_eps=1e-6, rope_theta=1e4, tied_embeddings=True, dtype="f32", max_seq=512),
    # head_dim 128
    "hd128": W.ModelShape(n_layers=2, d_model=64, n_q_heads=2, n_kv_heads=1, head_dim=128, d_ff=72, vocab=130,
                          rms_eps=1e-6, rope_theta=1e4, tied_embeddings=True, dtype="f32", max_seq=128),
}


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


def make_case(shape, seed, S, T, masked, std=0.25, spread=0.4):
    """Weights with visible logit differences, gains off 1, advantages of both signs (one zero), old
    log-probs off the new ones by up to +-spread so that both clip bounds are hit."""
    from oracle import sapo_update_oracle as U
    w = W.perturb_norm_gains(W.make_weights(shape, seed, std=std), seed)
    rng = np.random.default_rng([seed, 1])
    tokens = rng.integers(0, shape.vocab, size=(S, T)).astype(np.int32)
    mask = np.zeros((S, T), dtype=np.uint8)
    mask[:, T - masked:] = 1
    mask[0, T - masked + 1] = 0
    adv = rng.standard_normal(S).astype(np.float32)
    adv[1] = 0.0
    params = U.parameter_list(shape, w)
    zero_old = np.zeros((S, T), dtype=np.float32)
    _, lp, _ = U.loss_and_gradients(shape, params, tokens, mask, zero_old, adv)
    u = rng.uniform(-spread, spread, size=lp.shape)
    # keep the ratio exp(-u) clear of the two clip bounds: there fp32 and fp64 may pick different branches
    near = (np.abs(np.exp(-u) - 1.28) < 0.02) | (np.abs(np.exp(-u) - 0.8) < 0.02)
    u[near] = 0.0
    logp_old = (lp + u * (mask != 0)).astype(np.float32)
    return w, params, tokens, mask, logp_old, adv


# the ABI takes Adam's constants as fp32: those values are the constants
ADAM = dict(lr=float(np.float32(1e-3)), beta1=float(np.float32(0.9)), beta2=float(np.float32(0.999)),
            eps=float(np.float32(1e-8)))


def read_all(sapo, tr, what):
    """The tensors of the input list, then (for a model with projection biases) the per-layer bias vectors."""
    n = tr.n_in + (tr.shape.n_layers if tr.has_bias else 0)
    return [sapo.sapo_trainer_read(tr, what, i).cpu().numpy().astype(np.float64) for i in range(n)]


@pytest.mark.parametrize("name,S,T,masked", [("tiny", 8, 32, 16), ("ragged_untied", 3, 13, 9), ("hd128", 4, 70, 33),
                                             ("tiny", 16, 64, 30),    # 1024 tokens: split weight-gradient GEMMs
                                             ("tiny_long", 2, 300, 140),
                                             ("hd24", 3, 40, 20), ("hd24", 2, 272, 100)])
def test_update_matches_oracle(sapo, name, S, T, masked):
    import torch
    from oracle import sapo_update_oracle as U
    shape = SHAPES[name]
    w, params, tokens, mask, logp_old, adv = make_case(shape, 700 + len(name), S, T, masked)
    ref_loss, ref_lp, ref_g = U.loss_and_gradients(shape, params, tokens, mask, logp_old, adv)
    rho = np.exp(ref_lp - logp_old)[mask != 0]
    assert (rho > 1.28).any() and (rho < 0.8).any()          # the case exercises both clip bounds

    tr = sapo.sapo_trainer_create(shape, w)
    assert tr.steps == 0
    before = read_all(sapo, tr, 0)
    for a, b in zip(before, params):
        assert np.array_equal(a, b)                            # masters = the stored values
    loss, lp = sapo.sapo_policy_update(tr, dev(tokens), dev(mask), dev(logp_old), dev(adv))
    torch.cuda.synchronize()
    assert tr.steps == 1
    # forward: fp32 against fp64
    assert np.max(np.abs(lp.cpu().numpy() - ref_lp)) < 2e-4
    assert abs(float(loss.cpu()[0]) - ref_loss) < 1e-4 * max(1.0, abs(ref_loss))
    # gradient of every tensor
    g = read_all(sapo, tr, 1)
    gmax = max(float(np.max(np.abs(x))) for x in ref_g)
    assert gmax > 1e-4
    for i, (a, b) in enumerate(zip(g, ref_g)):
        err = float(np.max(np.abs(a - b)))
        assert err <= 2e-4 * max(float(np.max(np.abs(b))), 1e-3 * gmax) + 1e-7, (i, err, float(np.max(np.abs(b))))
    # Adam on the gradient the kernels produced: moments and parameters, fp32 against fp64
    st = U.AdamState(before)
    want = U.adam_step(before, g, st, **ADAM)
    m, v, after = read_all(sapo, tr, 2), read_all(sapo, tr, 3), read_all(sapo, tr, 0)
    for i in range(len(want)):
        assert np.allclose(m[i], st.m[i], rtol=1e-6, atol=1e-30)
        assert np.allclose(v[i], st.v[i], rtol=1e-6, atol=1e-30)
        assert np.max(np.abs(after[i] - want[i])) <= 1e-6 * 1e-3 + 2e-7 * np.max(np.abs(want[i])), i
    # a second step on the same batch: bias corrections of t = 2
    loss2, _ = sapo.sapo_policy_update(tr, dev(tokens), dev(mask), dev(logp_old), dev(adv), want_logp=False)
    torch.cuda.synchronize()
    assert tr.steps == 2
    g2 = read_all(sapo, tr, 1)
    want2 = U.adam_step(after, g2, st, **ADAM)
    after2 = read_all(sapo, tr, 0)
    for i in range(len(want2)):
        assert np.max(np.abs(after2[i] - want2[i])) <= 1e-6 * 1e-3 + 2e-7 * np.max(np.abs(want2[i])), i
    # and the second gradient against the oracle at the parameters the first step produced
    ref_loss2, _, ref_g2 = U.loss_and_gradients(shape, after, tokens, mask, logp_old, adv)
    assert abs(float(loss2.cpu()[0]) - ref_loss2) < 1e-4 * max(1.0, abs(ref_loss2))
    for a, b in zip(g2, ref_g2):
        assert float(np.max(np.abs(a - b))) <= 2e-4 * max(float(np.max(np.abs(b))), 1e-3 * gmax) + 1e-7
    tr.close()


def test_update_is_reproducible_and_lowers_the_loss(sapo):
    import torch
    shape = SHAPES["tiny"]
    w, params, tokens, mask, logp_old, adv = make_case(shape, 811, 6, 24, 12)
    outs = []
    for _ in range(2):
        tr = sapo.sapo_trainer_create(shape, w, lr=1e-4)
        losses = []
        for _ in range(4):
            loss, _ = sapo.sapo_policy_update(tr, dev(tokens), dev(mask), dev(logp_old), dev(adv), want_logp=False)
            losses.append(float(loss.cpu()[0]))
        torch.cuda.synchronize()
        outs.append((losses, [sapo.sapo_trainer_read(tr, 0, i).cpu().numpy() for i in range(tr.n_in)]))
        tr.close()
    assert outs[0][0] == outs[1][0]
    for a, b in zip(outs[0][1], outs[1][1]):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    assert outs[0][0][-1] < outs[0][0][0]


def test_bf16_model_masters_and_export(sapo):
    """A bf16 model: the masters start at the bf16 values, the update runs in fp32, the export rounds to
    nearest even; the exported tensors build a policy the rollout call accepts."""
    import torch
    from oracle import sapo_update_oracle as U
    from oracle import sapo_oracle as O
    shape = W.MINI_BF16
    w = W.make_weights(shape, 909, std=0.05)
    params = U.parameter_list(shape, w)
    rng = np.random.default_rng(3)
    S, T = 4, 20
    tokens = rng.integers(0, shape.vocab, size=(S, T)).astype(np.int32)
    mask = np.zeros((S, T), dtype=np.uint8)
    mask[:, 8:] = 1
    adv = np.array([1.0, -1.0, 0.5, -0.5], dtype=np.float32)
    _, lp, _ = U.loss_and_gradients(shape, params, tokens, mask, np.zeros((S, T), np.float32), adv)
    logp_old = lp.astype(np.float32)
    ref_loss, _, ref_g = U.loss_and_gradients(shape, params, tokens, mask, logp_old, adv)
    tr = sapo.sapo_trainer_create(shape, w)
    loss, lp_new = sapo.sapo_policy_update(tr, dev(tokens), dev(mask), dev(logp_old), dev(adv))
    torch.cuda.synchronize()
    assert np.max(np.abs(lp_new.cpu().numpy() - lp)) < 2e-4
    assert abs(float(loss.cpu()[0]) - ref_loss) < 1e-5
    g = read_all(sapo, tr, 1)
    gmax = max(float(np.max(np.abs(x))) for x in ref_g)
    for a, b in zip(g, ref_g):
        assert float(np.max(np.abs(a - b))) <= 2e-4 * max(float(np.max(np.abs(b))), 1e-3 * gmax) + 1e-7
    masters = read_all(sapo, tr, 0)
    out = sapo.sapo_trainer_export(tr)
    flat = [out["embed"]] + [lw[k] for lw in out["layers"] for k in sapo.LAYER_TENSORS] + [out["final_norm"]]
    assert out["lm_head"] is None
    for a, mst, (shp, gain) in zip(flat, masters, tr.tensor_shapes):
        assert tuple(a.shape) == shp
        if gain:
            assert a.dtype == np.float32 and np.array_equal(a.astype(np.float64), mst)
        else:
            assert a.dtype == np.uint16
            assert np.array_equal(W.bf16_bits_to_f32(a).astype(np.float64), O.round_bf16(mst))
    # the exported policy differs from the old one and runs
    assert any(not np.array_equal(a, b) for a, b in zip(flat[1:], [lw[k] for lw in w["layers"] for k in sapo.LAYER_TENSORS]))
    gw = sapo.sapo_weights_create(shape, out)
    prompts = rng.integers(0, shape.vocab, size=(2, 8)).astype(np.int32)
    toks, lps = sapo.sapo_rollout_generate(gw, dev(prompts), 2, 6, 1.0, 5)
    torch.cuda.synchronize()
    assert toks.shape == (4, 6) and np.all(np.isfinite(lps.cpu().numpy()))
    gw.close()
    tr.close()


def test_update_rejects_bad_arguments(sapo):
    import torch
    shape = SHAPES["tiny"]
    w, params, tokens, mask, logp_old, adv = make_case(shape, 5, 2, 8, 4)
    tr = sapo.sapo_trainer_create(shape, w)
    assert sapo.sapo_trainer_workspace_bytes(tr, 2, 1) == 0
    assert sapo.sapo_trainer_workspace_bytes(tr, 0, 8) == 0
    assert sapo.sapo_trainer_workspace_bytes(tr, 2, shape.max_seq + 1) == 0
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    with pytest.raises(sapo.SapoError) as e:
        sapo.sapo_policy_update(tr, dev(tokens), dev(mask), dev(logp_old), dev(adv), workspace=small)
    assert e.value.code == sapo.SAPO_EWORKSPACE or e.value.code == sapo.SAPO_EINVAL
    with pytest.raises(sapo.SapoError):
        sapo.sapo_policy_update(tr, dev(tokens), dev(mask), dev(logp_old), dev(adv), eps_low=1.5)
    assert tr.steps == 0
    with pytest.raises(sapo.SapoError):
        sapo.sapo_trainer_create(shape, w, lr=0.0)
    bad = W.ModelShape(n_layers=1, d_model=32, n_q_heads=3, n_kv_heads=2, head_dim=8, d_ff=16, vocab=32)
    with pytest.raises(sapo.SapoError):
        sapo.sapo_trainer_create(bad, W.make_weights(bad, 1))
    tr.close()


def test_update_on_the_0p5b_shapes(sapo):
    """The 0.5B model itself (24 layers, d 896, F 4864, 14 query / 2 KV heads of 64, vocabulary 151936, bf16 values as
    fp32 masters) on two sequences the oracle differentiates in seconds: the kernels, tiles and packed layouts of
    the full training set with fewer rows.  Also: the update's log-probs against the scoring call's (the bf16 MFMA
    path), two independent implementations of the same forward."""
    import torch
    from oracle import sapo_update_oracle as U
    shape = W.HALF_B
    w = W.make_weights(shape, 201)
    S, T, masked = 2, 128, 64
    rng = np.random.default_rng(77)
    tokens = rng.integers(0, shape.vocab, size=(S, T)).astype(np.int32)
    mask = W.make_completion_mask(S, T, masked)
    adv = np.array([0.8, -1.3], dtype=np.float32)
    params = U.parameter_list(shape, w)
    _, lp, _ = U.loss_and_gradients(shape, params, tokens, mask, np.zeros((S, T), np.float32), adv)
    u = rng.uniform(-0.4, 0.4, size=lp.shape)
    u[(np.abs(np.exp(-u) - 1.28) < 0.02) | (np.abs(np.exp(-u) - 0.8) < 0.02)] = 0.0
    logp_old = (lp + u * (mask != 0)).astype(np.float32)
    ref_loss, ref_lp, ref_g = U.loss_and_gradients(shape, params, tokens, mask, logp_old, adv)

    tr = sapo.sapo_trainer_create(shape, w)
    loss, lp_new = sapo.sapo_policy_update(tr, dev(tokens), dev(mask), dev(logp_old), dev(adv))
    torch.cuda.synchronize()
    assert np.max(np.abs(lp_new.cpu().numpy() - ref_lp)) < 2e-4
    assert abs(float(loss.cpu()[0]) - ref_loss) < 1e-4
    gmax = max(float(np.max(np.abs(x))) for x in ref_g)
    worst = 0.0
    for i, b in enumerate(ref_g):
        g = sapo.sapo_trainer_read(tr, 1, i).cpu().numpy().astype(np.float64)
        err = float(np.max(np.abs(g - b)))
        worst = max(worst, err / max(float(np.max(np.abs(b))), 1e-3 * gmax))
        assert err <= 2e-4 * max(float(np.max(np.abs(b))), 1e-3 * gmax) + 1e-7, (i, err, float(np.max(np.abs(b))))
    print("0.5B update: worst relative gradient error %.2e" % worst)
    tr.close()
    # the scoring call on the same tokens (bf16 weights, half MFMA operands): log-prob tolerance of that path
    gw = sapo.sapo_weights_create(shape, w)
    lp_score, _ = sapo.sapo_score_logprobs(gw, dev(tokens), dev(mask), dev(np.zeros(S, np.float32)), 2)
    torch.cuda.synchronize()
    assert np.max(np.abs(lp_score.cpu().numpy() - ref_lp)) < 2e-2
    gw.close()


def test_update_degenerate_batches(sapo):
    """Nothing masked: loss 0, zero gradient, parameters unchanged (Adam of a zero gradient).  All advantages zero:
    the same.  The shortest sequences the call accepts (T = 2)."""
    import torch
    shape = SHAPES["tiny"]
    w, params, tokens, mask, logp_old, adv = make_case(shape, 9, 4, 8, 4)
    tr = sapo.sapo_trainer_create(shape, w)
    before = read_all(sapo, tr, 0)
    loss, lp = sapo.sapo_policy_update(tr, dev(tokens), dev(np.zeros_like(mask)), dev(logp_old), dev(adv))
    torch.cuda.synchronize()
    assert float(loss.cpu()[0]) == 0.0 and not lp.cpu().numpy().any()
    assert all(not g.any() for g in read_all(sapo, tr, 1))
    assert all(np.array_equal(a, b) for a, b in zip(before, read_all(sapo, tr, 0)))
    loss, _ = sapo.sapo_policy_update(tr, dev(tokens), dev(mask), dev(logp_old), dev(np.zeros_like(adv)))
    torch.cuda.synchronize()
    assert float(loss.cpu()[0]) == 0.0
    assert all(not g.any() for g in read_all(sapo, tr, 1))
    assert all(np.array_equal(a, b) for a, b in zip(before, read_all(sapo, tr, 0)))
    assert tr.steps == 2
    # T = 2: one prediction per sequence
    from oracle import sapo_update_oracle as U
    t2 = tokens[:, :2].copy()
    m2 = np.ones((4, 2), dtype=np.uint8)
    lo2 = np.full((4, 2), -6.0, dtype=np.float32)
    ref_loss, ref_lp, ref_g = U.loss_and_gradients(shape, params, t2, m2, lo2, adv)
    loss, lp = sapo.sapo_policy_update(tr, dev(t2), dev(m2), dev(lo2), dev(adv))
    torch.cuda.synchronize()
    assert np.max(np.abs(lp.cpu().numpy() - ref_lp)) < 2e-4 and abs(float(loss.cpu()[0]) - ref_loss) < 1e-4 * max(1.0, abs(ref_loss))
    gmax = max(float(np.max(np.abs(x))) for x in ref_g)
    for g, b in zip(read_all(sapo, tr, 1), ref_g):
        assert float(np.max(np.abs(g - b))) <= 2e-4 * max(float(np.max(np.abs(b))), 1e-3 * gmax) + 1e-7
    tr.close()


@pytest.mark.parametrize("which", ["mini", "halfb_4_layers"])
def test_update_with_bf16_operands(sapo, which):
    """sapo_trainer_set_matmul_pieces(tr, 1): the large GEMMs take their operands rounded to bf16 (fp32 accumulation).
    An operand then carries a relative error of up to 2^-9, a product 2^-8, so a contraction is off by a small
    multiple of 2^-8 of its typical term: the tolerances are those of the bf16 scoring path (log-probs 2e-2) and
    5e-2 of a tensor's largest gradient entry, on models with the weight scale of the workloads (the stress cases of
    the fp32-accurate tests have logits in the tens, where bf16 log-probs are off by 0.1 and clip branches flip)."""
    import torch
    from dataclasses import replace
    from oracle import sapo_update_oracle as U
    shape, seed, S, T, masked = ((W.MINI_BF16, 909, 4, 64, 40) if which == "mini"
                                 else (replace(W.HALF_B, n_layers=4), 201, 2, 128, 64))
    w = W.make_weights(shape, seed)
    rng = np.random.default_rng(77)
    tokens = rng.integers(0, shape.vocab, size=(S, T)).astype(np.int32)
    mask = W.make_completion_mask(S, T, masked)
    adv = rng.standard_normal(S).astype(np.float32)
    params = U.parameter_list(shape, w)
    _, lp0, _ = U.loss_and_gradients(shape, params, tokens, mask, np.zeros((S, T), np.float32), adv)
    u = rng.uniform(-0.4, 0.4, size=lp0.shape)
    u[(np.abs(np.exp(-u) - 1.28) < 0.05) | (np.abs(np.exp(-u) - 0.8) < 0.05)] = 0.0   # clear of the clip bounds by 2 x 2e-2
    logp_old = (lp0 + u * (mask != 0)).astype(np.float32)
    ref_loss, ref_lp, ref_g = U.loss_and_gradients(shape, params, tokens, mask, logp_old, adv)
    tr = sapo.sapo_trainer_create(shape, w)
    for bad in (0, 4):
        with pytest.raises(sapo.SapoError):
            sapo.sapo_trainer_set_matmul_pieces(tr, bad)
    sapo.sapo_trainer_set_matmul_pieces(tr, 1)
    loss, lp = sapo.sapo_policy_update(tr, dev(tokens), dev(mask), dev(logp_old), dev(adv))
    torch.cuda.synchronize()
    lp_err = float(np.max(np.abs(lp.cpu().numpy() - ref_lp)))
    assert 1e-5 < lp_err < 2e-2          # bf16 operands are really in use, and within the bf16 path's tolerance
    assert abs(float(loss.cpu()[0]) - ref_loss) < 5e-3
    gmax = max(float(np.max(np.abs(x))) for x in ref_g)
    for i, b in enumerate(ref_g):
        g = sapo.sapo_trainer_read(tr, 1, i).cpu().numpy().astype(np.float64)
        assert float(np.max(np.abs(g - b))) <= 5e-2 * max(float(np.max(np.abs(b))), 1e-3 * gmax) + 1e-7, i
    g_err1 = max(float(np.max(np.abs(sapo.sapo_trainer_read(tr, 1, i).cpu().numpy() - b))) / max(float(np.max(np.abs(b))), 1e-3 * gmax)
                 for i, b in enumerate(ref_g))
    # two pieces (operands of 16 significant bits, three partial products): errors of 2^-16 of a product, of either
    # sign.  Log-probs to 5e-4, gradients to 1e-3 of a tensor's largest entry, and far closer than one piece.
    tr1 = sapo.sapo_trainer_create(shape, w)
    sapo.sapo_trainer_set_matmul_pieces(tr1, 2)
    loss2, lp2 = sapo.sapo_policy_update(tr1, dev(tokens), dev(mask), dev(logp_old), dev(adv))
    torch.cuda.synchronize()
    lp_err2 = float(np.max(np.abs(lp2.cpu().numpy() - ref_lp)))
    assert lp_err2 < 5e-4 and lp_err2 < lp_err / 8
    assert abs(float(loss2.cpu()[0]) - ref_loss) < 2e-4
    g_err2 = 0.0
    for i, b in enumerate(ref_g):
        g = sapo.sapo_trainer_read(tr1, 1, i).cpu().numpy().astype(np.float64)
        rel = float(np.max(np.abs(g - b))) / max(float(np.max(np.abs(b))), 1e-3 * gmax)
        assert rel <= 1e-3, i
        g_err2 = max(g_err2, rel)
    assert g_err2 < g_err1 / 8
    print("pieces 1: logp %.2e grad %.2e; pieces 2: logp %.2e grad %.2e" % (lp_err, g_err1, lp_err2, g_err2))
    tr1.close()
    # back to three pieces: fp32 accuracy again
    tr2 = sapo.sapo_trainer_create(shape, w)
    sapo.sapo_trainer_set_matmul_pieces(tr2, 1)
    sapo.sapo_trainer_set_matmul_pieces(tr2, 3)
    _, lp3 = sapo.sapo_policy_update(tr2, dev(tokens), dev(mask), dev(logp_old), dev(adv))
    torch.cuda.synchronize()
    assert np.max(np.abs(lp3.cpu().numpy() - ref_lp)) < 2e-4
    tr.close(); tr2.close()


def test_update_in_micro_batches(sapo):
    """A workspace too small for the whole training set: the call works through it a few sequences at a time and
    adds the gradients up; same loss and log-probs, same gradient up to the order of fp32 additions, same parity bar."""
    import torch
    from oracle import sapo_update_oracle as U
    shape = SHAPES["tiny"]
    S, T = 8, 32
    w, params, tokens, mask, logp_old, adv = make_case(shape, 4711, S, T, 16)
    ref_loss, ref_lp, ref_g = U.loss_and_gradients(shape, params, tokens, mask, logp_old, adv)
    gmax = max(float(np.max(np.abs(x))) for x in ref_g)
    results = []
    for s_micro in (8, 3, 1):
        tr = sapo.sapo_trainer_create(shape, w)
        nbytes = sapo.sapo_trainer_workspace_bytes_for(tr, S, T, s_micro)
        assert nbytes > 0 and (s_micro == 8) == (nbytes == sapo.sapo_trainer_workspace_bytes(tr, S, T))
        ws = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
        loss, lp = sapo.sapo_policy_update(tr, dev(tokens), dev(mask), dev(logp_old), dev(adv), workspace=ws)
        torch.cuda.synchronize()
        g = read_all(sapo, tr, 1)
        results.append((float(loss.cpu()[0]), lp.cpu().numpy(), g, read_all(sapo, tr, 0)))
        assert np.max(np.abs(results[-1][1] - ref_lp)) < 2e-4 and abs(results[-1][0] - ref_loss) < 1e-4 * max(1.0, abs(ref_loss))
        for a, b in zip(g, ref_g):
            assert float(np.max(np.abs(a - b))) <= 2e-4 * max(float(np.max(np.abs(b))), 1e-3 * gmax) + 1e-7
        assert tr.steps == 1
        tr.close()
    for other in results[1:]:
        assert np.allclose(other[1], results[0][1], rtol=0, atol=1e-5)     # per-row work: the batch size does not enter
        for a, b in zip(other[2], results[0][2]):
            assert float(np.max(np.abs(a - b))) <= 1e-5 * max(float(np.max(np.abs(b))), 1e-3 * gmax)
    # not even one sequence fits
    tr = sapo.sapo_trainer_create(shape, w)
    small = torch.empty(sapo.sapo_trainer_workspace_bytes_for(tr, S, T, 1) // 2, dtype=torch.uint8, device="cuda")
    with pytest.raises(sapo.SapoError) as e:
        sapo.sapo_policy_update(tr, dev(tokens), dev(mask), dev(logp_old), dev(adv), workspace=small)
    assert e.value.code == sapo.SAPO_EWORKSPACE and tr.steps == 0
    tr.close()


def test_update_with_projection_biases(sapo):
    """A model with biases on its query / key / value projections: they are trained with everything else; their
    gradient is checked like every tensor's, and the exported policy (biases included) scores as the oracle does."""
    import torch
    from oracle import sapo_update_oracle as U
    from oracle import sapo_oracle as O
    shape = SHAPES["tiny"]
    S, T = 6, 24
    w, _, tokens, mask, _, adv = make_case(shape, 321, S, T, 12)
    w = W.add_qkv_bias(w, shape, 321, std=0.3)
    params = U.parameter_list(shape, w)
    assert len(params) == 1 + 9 * shape.n_layers + 1 + shape.n_layers
    _, lp0, _ = U.loss_and_gradients(shape, params, tokens, mask, np.zeros((S, T), np.float32), adv)
    rng = np.random.default_rng(5)
    u = rng.uniform(-0.4, 0.4, size=lp0.shape)
    u[(np.abs(np.exp(-u) - 1.28) < 0.02) | (np.abs(np.exp(-u) - 0.8) < 0.02)] = 0.0
    logp_old = (lp0 + u * (mask != 0)).astype(np.float32)
    ref_loss, ref_lp, ref_g = U.loss_and_gradients(shape, params, tokens, mask, logp_old, adv)
    tr = sapo.sapo_trainer_create(shape, w)
    assert tr.has_bias
    loss, lp = sapo.sapo_policy_update(tr, dev(tokens), dev(mask), dev(logp_old), dev(adv))
    torch.cuda.synchronize()
    assert np.max(np.abs(lp.cpu().numpy() - ref_lp)) < 2e-4 and abs(float(loss.cpu()[0]) - ref_loss) < 1e-4 * max(1.0, abs(ref_loss))
    g = read_all(sapo, tr, 1)
    assert len(g) == len(ref_g)
    gmax = max(float(np.max(np.abs(x))) for x in ref_g)
    for i, (a, b) in enumerate(zip(g, ref_g)):
        assert float(np.max(np.abs(a - b))) <= 2e-4 * max(float(np.max(np.abs(b))), 1e-3 * gmax) + 1e-7, i
    assert all(np.max(np.abs(b)) > 0 for b in ref_g[-shape.n_layers:])        # the bias gradients are not trivially zero
    # Adam moved the biases; the exported policy carries them
    new = sapo.sapo_trainer_export(tr)
    for l, lw in enumerate(new["layers"]):
        old_b = np.concatenate([w["layers"][l]["bq"], w["layers"][l]["bk"], w["layers"][l]["bv"]])
        new_b = np.concatenate([lw["bq"], lw["bk"], lw["bv"]])
        step = np.abs(new_b - old_b)
        assert step.max() <= 1.001e-3 and step.max() > 0.9e-3               # first Adam step: lr * g / (|g| + eps)
    gw = sapo.sapo_weights_create(shape, new)
    rew = np.zeros(S, dtype=np.float32)
    lp_gpu, _ = sapo.sapo_score_logprobs(gw, dev(tokens), dev(mask), dev(rew), 2)
    torch.cuda.synchronize()
    ref = O.score_logprobs(O.Model(shape, new), tokens, mask)
    assert np.max(np.abs(lp_gpu.cpu().numpy() - ref)) < 1e-4
    gw.close(); tr.close()
