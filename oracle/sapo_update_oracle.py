"""CPU oracle for the local policy update of a SAPO node (Algorithm 1, the PolicyGradient step).

TEST INFRASTRUCTURE ONLY.  Imported by the tests, never by the product path; shares no code
with the HIP kernels.

What it follows (SAPO paper):
  * Algorithm 1 / Sec. 3.2: after the training set is assembled and rewarded the node updates
    its policy with a policy-gradient algorithm;
  * Sec. 4.2: that algorithm is GRPO without a KL term, with the probability ratio clipped to
    [1 - 0.2, 1 + 0.28], optimised by Adam with its default hyper-parameters (learning rate
    1e-3; the defaults of Kingma & Ba, ICLR'15, Algorithm 1: beta1 0.9, beta2 0.999, eps 1e-8,
    no weight decay).

One update = one gradient step on the whole training set:
    logp_new = teacher-forced log-probs of the batch under the current parameters,
    loss     = clipped surrogate (token-level mean over the masked tokens),
    g        = d loss / d parameters,
    Adam step on every parameter (embedding, matrices, RMSNorm gains).

The forward pass is restated here with torch CPU float64 operations so that reverse-mode
differentiation (torch.autograd, used as a library primitive) yields g; the update rule is
written out in numpy.  The forward is the same decoder as sapo_oracle.py's (RMSNorm, rotary
positions with the rotate-half pairing, grouped-query attention, SwiGLU, tied or untied LM head).

Pins (tests/test_oracle_update_pins.py): the torch forward equals the numpy oracle's log-probs;
the gradient equals central finite differences of the *numpy* oracle's loss, for entries of
every kind of tensor; a parameter the loss cannot depend on (an unused embedding row, when the
head is untied) has zero gradient; the Adam step equals torch.optim.Adam's and the closed form of
the first step (-lr * g / (|g| + eps)); a step along the update lowers the loss.
"""
from __future__ import annotations

import math
from typing import List, Sequence

import numpy as np
import torch

from . import sapo_oracle as O

LAYER_MATS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


def parameter_list(shape, weights: dict) -> List[np.ndarray]:
    """The trainable tensors as float64 arrays in the order of the library's tensor list:
    embed, per layer (attn_norm, wq, wk, wv, wo, ffn_norm, w_gate, w_up, w_down), final_norm,
    lm_head (only when the head is untied), then, if the model has projection biases, one vector
    [bq | bk | bv] per layer."""
    out = [O._stored_to_f64(weights["embed"])]
    for lw in weights["layers"][: shape.n_layers]:
        out += [O._stored_to_f64(lw[k]) for k in LAYER_MATS]
    out.append(O._stored_to_f64(weights["final_norm"]))
    if weights.get("lm_head") is not None:
        out.append(O._stored_to_f64(weights["lm_head"]))
    if any("bq" in lw for lw in weights["layers"][: shape.n_layers]):
        # optional biases of the query / key / value projections: one vector [bq | bk | bv] per layer, after
        # everything else (a layer without them gets zeros, which are then trained like the others)
        for lw in weights["layers"][: shape.n_layers]:
            if "bq" in lw:
                out.append(np.concatenate([lw["bq"], lw["bk"], lw["bv"]]).astype(np.float64))
            else:
                out.append(np.zeros(shape.q_dim + 2 * shape.kv_dim))
    return out


def weights_from_parameters(shape, params: Sequence[np.ndarray]) -> dict:
    """Inverse of parameter_list (float32 arrays, for the numpy oracle's Model)."""
    it = iter(params)
    w = {"embed": np.asarray(next(it)), "layers": []}
    for _ in range(shape.n_layers):
        w["layers"].append({k: np.asarray(next(it)) for k in LAYER_MATS})
    w["final_norm"] = np.asarray(next(it))
    rest = list(it)
    w["lm_head"] = np.asarray(rest.pop(0)) if (not shape.tied_embeddings) else None
    if rest:
        assert len(rest) == shape.n_layers
        q, kv = shape.q_dim, shape.kv_dim
        for lw, b in zip(w["layers"], rest):
            b = np.asarray(b)
            lw["bq"], lw["bk"], lw["bv"] = b[:q], b[q:q + kv], b[q + kv:]
    return w


# --------------------------------------------------------------------------- #
# forward pass in torch float64
# --------------------------------------------------------------------------- #
def _rmsnorm(h, gain, eps):
    return h * torch.rsqrt(torch.mean(h * h, dim=-1, keepdim=True) + eps) * gain


def _rope(x, theta):
    """x[T, heads, hd] at positions 0..T-1; pair (i, i + hd/2) rotated by pos * theta^(-2i/hd)."""
    T, _, hd = x.shape
    half = hd // 2
    freq = theta ** (-2.0 * torch.arange(half, dtype=torch.float64) / hd)
    ang = torch.arange(T, dtype=torch.float64)[:, None] * freq[None, :]
    c, s = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return torch.cat([x1 * c - x2 * s, x2 * c + x1 * s], dim=-1)


def _sequence_logprobs(shape, p: Sequence[torch.Tensor], tokens: np.ndarray) -> torch.Tensor:
    """log softmax(z_{t-1})[tokens[t]] for t = 1..T-1 of one sequence; entry 0 is 0."""
    T = len(tokens)
    hq, hkv, hd = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    rep = hq // hkv
    tok = torch.as_tensor(np.asarray(tokens, dtype=np.int64))
    h = p[0][tok]
    causal = torch.tril(torch.ones(T, T, dtype=torch.bool))
    n_plain = 1 + 9 * shape.n_layers + 1 + (0 if shape.tied_embeddings else 1)
    biases = p[n_plain:] if len(p) > n_plain else None      # per layer [bq | bk | bv], added before the rotary embedding
    qd, kvd = hq * hd, hkv * hd
    i = 1
    for layer in range(shape.n_layers):
        g1, wq, wk, wv, wo, g2, wg, wu, wd = p[i:i + 9]
        i += 9
        a = _rmsnorm(h, g1, shape.rms_eps)
        q, k, v = a @ wq.T, a @ wk.T, a @ wv.T
        if biases is not None:
            b = biases[layer]
            q, k, v = q + b[:qd], k + b[qd:qd + kvd], v + b[qd + kvd:]
        q = _rope(q.reshape(T, hq, hd), shape.rope_theta)
        k = _rope(k.reshape(T, hkv, hd), shape.rope_theta)
        v = v.reshape(T, hkv, hd)
        heads = []
        for hh in range(hq):
            s = (q[:, hh, :] @ k[:, hh // rep, :].T) / math.sqrt(hd)
            s = s.masked_fill(~causal, float("-inf"))
            heads.append(torch.softmax(s, dim=-1) @ v[:, hh // rep, :])
        h = h + torch.cat(heads, dim=-1) @ wo.T
        b = _rmsnorm(h, g2, shape.rms_eps)
        h = h + (torch.nn.functional.silu(b @ wg.T) * (b @ wu.T)) @ wd.T
    x = _rmsnorm(h, p[i], shape.rms_eps)
    head = p[0] if shape.tied_embeddings else p[i + 1]
    lp = torch.log_softmax(x[:-1] @ head.T, dim=-1)
    picked = lp[torch.arange(T - 1), tok[1:]]
    return torch.cat([torch.zeros(1, dtype=torch.float64), picked])


def _surrogate(logp_new, logp_old, mask, adv, eps_low, eps_high):
    """-(mean over masked tokens) of min(rho A, clip(rho, 1 - eps_low, 1 + eps_high) A)  (Sec. 4.2)."""
    n = int(mask.sum())
    if n == 0:
        return logp_new.sum() * 0.0
    rho = torch.exp(logp_new - logp_old)
    a = adv[:, None]
    term = torch.minimum(rho * a, torch.clamp(rho, 1.0 - eps_low, 1.0 + eps_high) * a)
    return -(term * mask).sum() / n


def loss_and_gradients(shape, params: Sequence[np.ndarray], tokens: np.ndarray, completion_mask: np.ndarray,
                       logp_old: np.ndarray, advantages: np.ndarray, eps_low: float = 0.2, eps_high: float = 0.28):
    """(loss, logp_new float64 [S, T], [d loss / d tensor, float64, in parameter_list order]).

    Masked positions at t = 0 have no prediction behind them: their log-prob is the constant 0
    (as in the scoring call), so they enter the loss but carry no gradient."""
    p = [torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True) for a in params]
    tokens = np.asarray(tokens)
    S, T = tokens.shape
    mk = torch.as_tensor((np.asarray(completion_mask) != 0).astype(np.float64))
    rows = []
    for s in range(S):
        lp = _sequence_logprobs(shape, p, tokens[s])
        rows.append(lp * mk[s])     # unmasked entries are 0, as the scoring call returns them
    logp_new = torch.stack(rows)
    loss = _surrogate(logp_new, torch.as_tensor(np.asarray(logp_old, dtype=np.float64)), mk,
                      torch.as_tensor(np.asarray(advantages, dtype=np.float64)), eps_low, eps_high)
    loss.backward()
    grads = [(t.grad if t.grad is not None else torch.zeros_like(t)).numpy().copy() for t in p]
    return float(loss.detach()), logp_new.detach().numpy().copy(), grads


# --------------------------------------------------------------------------- #
# Adam (Kingma & Ba, Algorithm 1), float64
# --------------------------------------------------------------------------- #
class AdamState:
    def __init__(self, params: Sequence[np.ndarray]):
        self.t = 0
        self.m = [np.zeros_like(np.asarray(a, dtype=np.float64)) for a in params]
        self.v = [np.zeros_like(np.asarray(a, dtype=np.float64)) for a in params]


def adam_step(params: Sequence[np.ndarray], grads: Sequence[np.ndarray], st: AdamState, lr: float = 1e-3,
              beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8) -> List[np.ndarray]:
    """One step: m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;  theta <- theta - lr * mhat / (sqrt(vhat) + eps)
    with mhat = m / (1 - b1^t), vhat = v / (1 - b2^t).  Returns the new parameters; `st` is advanced."""
    st.t += 1
    c1, c2 = 1.0 - beta1 ** st.t, 1.0 - beta2 ** st.t
    out = []
    for i, (a, g) in enumerate(zip(params, grads)):
        g = np.asarray(g, dtype=np.float64)
        st.m[i] = beta1 * st.m[i] + (1.0 - beta1) * g
        st.v[i] = beta2 * st.v[i] + (1.0 - beta2) * g * g
        out.append(np.asarray(a, dtype=np.float64) - lr * (st.m[i] / c1) / (np.sqrt(st.v[i] / c2) + eps))
    return out


def policy_update(shape, params, st: AdamState, tokens, completion_mask, logp_old, advantages, eps_low=0.2,
                  eps_high=0.28, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8):
    """One PolicyGradient step of Algorithm 1: (loss before the step, new parameters)."""
    loss, _, grads = loss_and_gradients(shape, params, tokens, completion_mask, logp_old, advantages, eps_low, eps_high)
    return loss, adam_step(params, grads, st, lr, beta1, beta2, eps)
