"""The number format of the matrix-core path, stated in include/sapo.h at sapo_weights_create: weights are held as IEEE
half (a value half cannot hold is refused), activations are rounded to half and clamped to +-65504 (results stay
finite; a debug call counts the clamped values).  Up to the limit the results follow the definition (the oracle)."""
import numpy as np
import pytest

from oracle import sapo_oracle as O
from paper_2509_08721_amd import workloads as W

pytestmark = pytest.mark.gpu

LOGPROB_TOL = 2e-2
HALF_MAX = 65504.0
SHAPE = W.MINI_BF16_HD128          # untied LM head: the embedding can be scaled without touching a packed matrix


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


def with_embedding_peak(weights, peak):
    """The same model with the embedding table scaled so that its largest entry is `peak` (all gains are 1, so the
    first projection's operand is the embedding row itself)."""
    e = W.bf16_bits_to_f32(weights["embed"])
    out = dict(weights)
    out["embed"] = W.f32_to_bf16_bits((e * np.float32(peak / np.abs(e).max())).astype(np.float32))
    return out


def batch(seed, S=4, T=48):
    rng = np.random.default_rng(seed)
    tokens = rng.integers(0, SHAPE.vocab, size=(S, T)).astype(np.int32)
    mask = np.zeros((S, T), dtype=np.uint8)
    mask[:, T // 2:] = 1
    return tokens, mask, rng.random(S).astype(np.float32)


def test_ordinary_weights_clamp_nothing_and_tiny_weights_are_counted(sapo):
    w = W.make_weights(SHAPE, 71, std=0.05)
    gw = sapo.sapo_weights_create(SHAPE, w)
    assert gw.uses_mfma
    tokens, _, _ = batch(1)
    assert sapo.sapo_debug_half_clamped(gw, dev(tokens)) == 0
    packed = [w["lm_head"]] + [lw[k] for lw in w["layers"] for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")]
    tiny = sum(int(((a != 0) & (a < 2.0 ** -14)).sum()) for a in (np.abs(W.bf16_bits_to_f32(m)) for m in packed))
    stats = sapo.sapo_weights_half_stats(gw)
    assert stats == {"half_path": True, "below_normal_range": tiny} and tiny > 0


def test_activations_up_to_the_limit_follow_the_definition(sapo):
    w = with_embedding_peak(W.make_weights(SHAPE, 71, std=0.05), 6.0e4)      # residual rows reach 6.0e4 < 65504
    gw = sapo.sapo_weights_create(SHAPE, w)
    tokens, mask, rewards = batch(2)
    assert sapo.sapo_debug_half_clamped(gw, dev(tokens)) == 0
    lp, _ = sapo.sapo_score_logprobs(gw, dev(tokens), dev(mask), dev(rewards), 4)
    lp = lp.cpu().numpy()
    ref = O.score_logprobs(O.Model(SHAPE, w), tokens, mask)
    assert np.isfinite(lp).all()
    assert np.max(np.abs(lp - ref)[mask.astype(bool)]) <= LOGPROB_TOL


def test_activations_beyond_the_limit_are_clamped_counted_and_stay_finite(sapo):
    w = with_embedding_peak(W.make_weights(SHAPE, 71, std=0.05), 2.0e5)      # a few per cent of the entries exceed 65504
    gw = sapo.sapo_weights_create(SHAPE, w)
    tokens, mask, rewards = batch(3)
    rows = W.bf16_bits_to_f32(w["embed"])[tokens]                            # the first projection's operand, unclamped
    beyond = int((np.abs(rows) > HALF_MAX).sum())
    assert beyond > 0
    # every layer's operands are counted; the first projection's alone has `beyond` clamped values
    assert sapo.sapo_debug_half_clamped(gw, dev(tokens)) >= beyond
    lp, _ = sapo.sapo_score_logprobs(gw, dev(tokens), dev(mask), dev(rewards), 4)
    lp = lp.cpu().numpy()
    assert np.isfinite(lp).all() and (lp <= 0).all()
    toks, lps = sapo.sapo_rollout_generate(gw, dev(tokens[:2, :16]), 2, 8, 1.0, 5)
    toks = toks.cpu().numpy()
    assert toks.min() >= 0 and toks.max() < SHAPE.vocab and np.isfinite(lps.cpu().numpy()).all()


@pytest.mark.parametrize("value", [1.0e5, -7.0e4, np.inf, np.nan])
def test_weights_outside_the_half_range_are_refused(sapo, value):
    w = W.make_weights(SHAPE, 71, std=0.05)
    bad = dict(w)
    bad["layers"] = [dict(lw) for lw in w["layers"]]
    m = W.bf16_bits_to_f32(w["layers"][1]["w_up"]).copy()
    m[3, 5] = value
    bad["layers"][1]["w_up"] = W.f32_to_bf16_bits(m)
    with pytest.raises(sapo.SapoError, match="IEEE half"):
        sapo.sapo_weights_create(SHAPE, bad)
    # the same through an update of a good handle; filled again with valid weights the handle works as a fresh one
    gw = sapo.sapo_weights_create(SHAPE, w)
    with pytest.raises(sapo.SapoError, match="IEEE half"):
        sapo.sapo_weights_update(gw, bad)
    sapo.sapo_weights_update(gw, w)
    tokens, mask, rewards = batch(4)
    lp, _ = sapo.sapo_score_logprobs(gw, dev(tokens), dev(mask), dev(rewards), 4)
    lp_fresh, _ = sapo.sapo_score_logprobs(sapo.sapo_weights_create(SHAPE, w), dev(tokens), dev(mask), dev(rewards), 4)
    assert np.array_equal(lp.cpu().numpy(), lp_fresh.cpu().numpy())
