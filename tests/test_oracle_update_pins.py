"""Pins of the policy-update oracle (oracle/sapo_update_oracle.py) against things other than itself:
the numpy oracle's forward pass and loss, finite differences of those, torch.optim.Adam, closed forms."""
import math

import numpy as np
import pytest
import torch

from oracle import sapo_oracle as O
from oracle import sapo_update_oracle as U
from paper_2509_08721_amd import workloads as W

SMALL = W.ModelShape(n_layers=2, d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8, d_ff=48, vocab=64,
                     rms_eps=1e-6, rope_theta=1e4, tied_embeddings=True, dtype="f32", max_seq=64)
SMALL_UNTIED = W.ModelShape(n_layers=1, d_model=32, n_q_heads=2, n_kv_heads=1, head_dim=16, d_ff=40, vocab=48,
                            rms_eps=1e-5, rope_theta=1e6, tied_embeddings=False, dtype="f32", max_seq=64)


def make_case(shape, seed, S=4, T=12, masked=7, std=0.3, biases=False):
    """Weights large enough for the logits to differ visibly between tokens, gains off 1, a batch with
    advantages of both signs and old log-probs off the new ones by up to +-0.4 (both clip bounds are hit)."""
    w = W.perturb_norm_gains(W.make_weights(shape, seed, std=std), seed)
    if biases:
        w = W.add_qkv_bias(w, shape, seed, std=0.3)
    rng = np.random.default_rng([seed, 1])
    tokens = rng.integers(0, shape.vocab - 3, size=(S, T)).astype(np.int32)   # the last 3 ids never occur
    mask = np.zeros((S, T), dtype=np.uint8)
    mask[:, T - masked:] = 1
    mask[0, T - masked] = 0          # a hole in one mask
    adv = rng.standard_normal(S).astype(np.float32)
    adv[1] = 0.0                      # a zero-advantage sequence
    params = U.parameter_list(shape, w)
    lp64 = numpy_logprobs(shape, params, tokens, mask)
    logp_old = (lp64 + rng.uniform(-0.4, 0.4, size=lp64.shape) * (mask != 0)).astype(np.float32)
    return params, tokens, mask, logp_old, adv


def numpy_logprobs(shape, params, tokens, mask):
    """Teacher-forced log-probs in float64 from the numpy oracle's own blocks."""
    m = O.Model(shape, U.weights_from_parameters(shape, params))
    S, T = tokens.shape
    out = np.zeros((S, T))
    for s in range(S):
        x = O.hidden_states(m, tokens[s])
        lp = O.log_softmax(O.logits_from_hidden(m, x[:-1]))
        out[s, 1:] = lp[np.arange(T - 1), tokens[s, 1:]]
    return out * (mask != 0)


def numpy_loss(shape, params, tokens, mask, logp_old, adv):
    return O.clipped_surrogate_loss(numpy_logprobs(shape, params, tokens, mask), logp_old, mask, adv)[0]


@pytest.mark.parametrize("shape,biases", [(SMALL, False), (SMALL_UNTIED, False), (SMALL, True), (SMALL_UNTIED, True)])
def test_forward_and_loss_equal_numpy_oracle(shape, biases):
    params, tokens, mask, logp_old, adv = make_case(shape, 11, biases=biases)
    loss, lp, _ = U.loss_and_gradients(shape, params, tokens, mask, logp_old, adv)
    ref = numpy_logprobs(shape, params, tokens, mask)
    assert np.max(np.abs(lp - ref)) < 1e-11
    assert abs(loss - numpy_loss(shape, params, tokens, mask, logp_old, adv)) < 1e-12
    # and the float32 scoring call of the numpy oracle
    m = O.Model(shape, U.weights_from_parameters(shape, params))
    assert np.max(np.abs(O.score_logprobs(m, tokens, mask) - lp)) < 1e-5
    # both clip bounds and the unclipped range occur in this case
    rho = np.exp(lp - logp_old)[mask != 0]
    assert (rho > 1.28).any() and (rho < 0.8).any() and ((rho > 0.8) & (rho < 1.28)).any()


@pytest.mark.parametrize("shape,biases", [(SMALL, False), (SMALL_UNTIED, False), (SMALL, True), (SMALL_UNTIED, True)])
def test_gradient_equals_finite_differences_of_numpy_loss(shape, biases):
    params, tokens, mask, logp_old, adv = make_case(shape, 23, biases=biases)
    _, _, grads = U.loss_and_gradients(shape, params, tokens, mask, logp_old, adv)
    assert len(grads) == len(params) == (1 + 9 * shape.n_layers + 1 + (0 if shape.tied_embeddings else 1)
                                         + (shape.n_layers if biases else 0))
    rng = np.random.default_rng(5)
    h = 1e-6
    gmax = max(float(np.max(np.abs(g))) for g in grads)
    for ti, (a, g) in enumerate(zip(params, grads)):
        assert g.shape == a.shape
        idxs = [tuple(rng.integers(0, n) for n in a.shape) for _ in range(3)]
        if ti == 0:
            idxs.append((int(tokens[2, 5]), 3))            # an embedding row that is used
        for idx in idxs:
            pp = [x.copy() for x in params]
            pp[ti][idx] += h
            up = numpy_loss(shape, pp, tokens, mask, logp_old, adv)
            pp[ti][idx] -= 2 * h
            dn = numpy_loss(shape, pp, tokens, mask, logp_old, adv)
            fd = (up - dn) / (2 * h)
            assert abs(fd - g[idx]) <= 2e-6 * gmax + 1e-9, (ti, idx, fd, g[idx])


def test_parameters_the_loss_cannot_see_have_zero_gradient():
    shape = SMALL_UNTIED
    params, tokens, mask, logp_old, adv = make_case(shape, 31)
    _, _, grads = U.loss_and_gradients(shape, params, tokens, mask, logp_old, adv)
    # untied head: embedding rows of ids that never occur as inputs get no gradient; every head row does
    # (the log-sum-exp sees all of them)
    unused = np.setdiff1d(np.arange(shape.vocab), tokens[:, :-1])
    assert unused.size >= 3 and np.all(grads[0][unused] == 0.0)
    assert np.all(np.abs(grads[-1]).sum(axis=1) > 0.0)
    # a sequence with zero advantage contributes nothing: dropping it (and rescaling by the token count)
    keep = np.array([0, 2, 3])
    n_all, n_keep = int(mask.sum()), int(mask[keep].sum())
    _, _, g2 = U.loss_and_gradients(shape, params, tokens[keep], mask[keep], logp_old[keep], adv[keep])
    for a, b in zip(grads, g2):
        assert np.allclose(a * n_all, b * n_keep, rtol=1e-9, atol=1e-13)


def test_on_policy_gradient_is_the_policy_gradient():
    """With logp_old = logp_new nothing is clipped: g = -(1/N) sum_masked A_s * d logp / d theta, i.e. the
    gradient of the linear function -(1/N) sum A_s logp (REINFORCE with the group-relative advantage)."""
    shape = SMALL
    params, tokens, mask, _, adv = make_case(shape, 41)
    lp = numpy_logprobs(shape, params, tokens, mask)
    _, _, g = U.loss_and_gradients(shape, params, tokens, mask, lp, adv)
    n = int(mask.sum())
    h = 1e-6
    rng = np.random.default_rng(6)
    for ti in (0, 2, 5, 9, len(params) - 1):
        idx = tuple(rng.integers(0, k) for k in params[ti].shape)
        pp = [x.copy() for x in params]
        pp[ti][idx] += h
        up = -(numpy_logprobs(shape, pp, tokens, mask) * adv[:, None]).sum() / n
        pp[ti][idx] -= 2 * h
        dn = -(numpy_logprobs(shape, pp, tokens, mask) * adv[:, None]).sum() / n
        assert abs((up - dn) / (2 * h) - g[ti][idx]) < 1e-7 * max(1.0, np.max(np.abs(g[ti])))


def test_adam_equals_torch_optim_and_closed_form():
    rng = np.random.default_rng(7)
    p0 = [rng.standard_normal((5, 3)), rng.standard_normal(4)]
    tp = [torch.tensor(a.copy(), requires_grad=True) for a in p0]
    opt = torch.optim.Adam(tp, lr=1e-3)          # the library's defaults are the paper's "default hyper-parameters"
    st = U.AdamState(p0)
    p = [a.copy() for a in p0]
    for step in range(4):
        grads = [rng.standard_normal(a.shape) * 10.0 ** rng.integers(-6, 2) for a in p0]
        for t, g in zip(tp, grads):
            t.grad = torch.tensor(g.copy())
        opt.step()
        p = U.adam_step(p, grads, st)
        for a, t in zip(p, tp):
            assert np.allclose(a, t.detach().numpy(), rtol=0, atol=1e-12)
        if step == 0:   # first step: mhat = g, vhat = g^2
            for a, a0, g in zip(p, p0, grads):
                assert np.allclose(a, a0 - 1e-3 * g / (np.abs(g) + 1e-8), rtol=0, atol=1e-15)
    assert st.t == 4
    # zero gradient: nothing moves
    q = U.adam_step(p0, [np.zeros_like(a) for a in p0], U.AdamState(p0))
    assert all(np.array_equal(a, b) for a, b in zip(q, p0))


def test_update_lowers_the_loss():
    shape = SMALL
    params, tokens, mask, logp_old, adv = make_case(shape, 53)
    st = U.AdamState(params)
    l0, new = U.policy_update(shape, params, st, tokens, mask, logp_old, adv, lr=1e-4)
    l1 = numpy_loss(shape, new, tokens, mask, logp_old, adv)
    assert math.isfinite(l0) and l1 < l0
    assert abs(l0 - numpy_loss(shape, params, tokens, mask, logp_old, adv)) < 1e-12
