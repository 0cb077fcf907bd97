"""CPU oracle for the SAPO node hot path: rollout generation and log-prob scoring.

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, numpy/fp64 statement of what
the path computes.  It is imported by the tests, by the smoke check and by the
benchmark's CPU-baseline leg, never by the product path, and it shares no code
with the HIP kernels.

What it follows (SAPO paper):
  * Sec. 3.1: node n holds a policy pi^n and answers each question q with a
    rollout R^n(q) of L^n sampled answers               -> rollout_generate()
  * Sec. 3.2: a node re-encodes any rollout, its own or one shared by the
    swarm, and computes token-level values under its own policy, however
    unlikely the rollout is under that policy           -> score_logprobs()
  * Sec. 3.2 / Sec. 4.2 / Sec. 5: GRPO consumes group-relative advantages;
    rollouts of a group whose rewards are all equal have zero advantage and
    are discarded                                        -> group_advantages()
  * Sec. 4.2: the local update is GRPO without a KL term and with asymmetric
    clipping (0.2 / 0.28) of the probability ratio       -> clipped_surrogate_loss()
  * Sec. 3.2 / Algorithm 1: the training set is I datapoints of the node's own
    and J sampled uniformly from the swarm's after discarding those with zero
    advantage                                            -> assemble_training_set()
The paper names the policy only as a 0.5B-parameter decoder-only LM; the block
structure used here (RMSNorm, rotary positions with the rotate-half pairing,
grouped-query attention, SwiGLU FFN, tied LM head) is the reading recorded in
the design notes.  Sampling is exact sampling from softmax(z / T) done by
Gumbel-max with noise from Philox4x32-10 (Salmon et al., SC'11) keyed on
(seed, sequence, step) so that it can be reproduced element by element.

All arithmetic is float64 on float32- or bf16-valued weights: the definition,
with no rounding of activations anywhere.

Pins (tests/test_oracle_*.py): Philox known-answer vectors, Gumbel moments,
sampler histogram vs softmax, brute-force attention, rotary closed forms,
KV-cache decode == full recompute, log-softmax normalisation, advantage closed
forms, zero-layer model, causality, batch invariance, library routines
(torch CPU) for the individual blocks; for the clipped surrogate: hand-worked
tokens on each side of each clip bound, the on-policy closed form, torch
autograd, finite differences, mask invariance; for the assembly: inclusion,
first-draw and pair frequencies of the sampled subsets against those of a
uniform subset, eligibility, edge sizes, stream separation, row-exact gathers.
"""
from __future__ import annotations

import math
from typing import Optional, Sequence

import numpy as np

# --------------------------------------------------------------------------- #
# Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw, SC'11)
# --------------------------------------------------------------------------- #
_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85
_MASK32 = np.uint64(0xFFFFFFFF)
_SH32 = np.uint64(32)


def philox4x32_10(counter: np.ndarray, key: np.ndarray) -> np.ndarray:
    """counter uint32[..., 4], key uint32[..., 2] (broadcastable) -> uint32[..., 4].

    Ten rounds; each round multiplies counter words 0 and 2 by the two round
    constants (32x32 -> 64 bit), and mixes high/low halves with words 1, 3 and
    the key; the key is bumped by the Weyl constants between rounds.
    """
    counter = np.asarray(counter, dtype=np.uint32)
    key = np.asarray(key, dtype=np.uint32)
    c0, c1, c2, c3 = (counter[..., i].astype(np.uint64) for i in range(4))
    k0 = key[..., 0].astype(np.uint64)
    k1 = key[..., 1].astype(np.uint64)
    for r in range(10):
        if r > 0:
            k0 = (k0 + np.uint64(_PHILOX_W0)) & _MASK32
            k1 = (k1 + np.uint64(_PHILOX_W1)) & _MASK32
        p0 = _PHILOX_M0 * c0
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> _SH32, p0 & _MASK32
        hi1, lo1 = p1 >> _SH32, p1 & _MASK32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0) & _MASK32, lo1, (hi0 ^ c3 ^ k1) & _MASK32, lo0
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def sampling_uniform_bits(seed: int, seq: int, step: int, vocab: int) -> np.ndarray:
    """uint32[vocab] raw random words for (seed, sequence, step).

    Key = (low, high) 32-bit halves of the 64-bit seed.  Vocab entry v uses word
    v mod 4 of the block with counter (v div 4, step, sequence, 0).
    """
    nblk = (vocab + 3) // 4
    ctr = np.zeros((nblk, 4), dtype=np.uint32)
    ctr[:, 0] = np.arange(nblk, dtype=np.uint32)
    ctr[:, 1] = np.uint32(step)
    ctr[:, 2] = np.uint32(seq)
    key = np.array([seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF], dtype=np.uint32)
    return philox4x32_10(ctr, key).reshape(-1)[:vocab]


def uniform_from_bits(x: np.ndarray) -> np.ndarray:
    """u = (2 (x >> 9) + 1) 2^-24: 23 random bits, strictly inside (0, 1), exact in fp32."""
    return ((x >> np.uint32(9)).astype(np.float64) * 2.0 + 1.0) * (2.0 ** -24)


def gumbel_noise(seed: int, seq: int, step: int, vocab: int) -> np.ndarray:
    """float32[vocab] standard Gumbel noise g = -ln(-ln u), evaluated in fp64 then rounded."""
    u = uniform_from_bits(sampling_uniform_bits(seed, seq, step, vocab))
    return (-np.log(-np.log(u))).astype(np.float32)


# --------------------------------------------------------------------------- #
# Precision helpers
# --------------------------------------------------------------------------- #
def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round float64 values to the nearest bf16 value (through fp32, ties to even)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(np.float64)


def _stored_to_f64(a: Optional[np.ndarray]) -> Optional[np.ndarray]:
    """A weight tensor as stored (float32, or uint16 holding bf16 bit patterns) -> float64."""
    if a is None:
        return None
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


class Model:
    """Model description + float64 copies of the weights (values unchanged)."""

    def __init__(self, shape, weights: dict):
        self.n_layers = shape.n_layers
        self.d = shape.d_model
        self.hq = shape.n_q_heads
        self.hkv = shape.n_kv_heads
        self.hd = shape.head_dim
        self.f = shape.d_ff
        self.vocab = shape.vocab
        self.eps = float(shape.rms_eps)
        self.theta = float(shape.rope_theta)
        assert self.hq % self.hkv == 0 and self.hd % 2 == 0
        self.embed = _stored_to_f64(weights["embed"])
        self.layers = [{k: _stored_to_f64(v) for k, v in lw.items()} for lw in weights["layers"][: self.n_layers]]
        self.final_norm = _stored_to_f64(weights["final_norm"])
        lm = weights.get("lm_head")
        self.lm_head = self.embed if lm is None else _stored_to_f64(lm)


# --------------------------------------------------------------------------- #
# Blocks of the decoder
# --------------------------------------------------------------------------- #
def rmsnorm(h: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """h[..., d] -> h * rsqrt(mean(h^2) + eps) * gain."""
    ms = np.mean(h * h, axis=-1, keepdims=True)
    return h / np.sqrt(ms + eps) * gain


def rope_rotate(x: np.ndarray, positions: np.ndarray, theta: float) -> np.ndarray:
    """Rotary position embedding, rotate-half pairing.

    x[n, heads, hd], positions[n] (absolute, 0-based).  For i < hd/2 the pair
    (x_i, x_{i+hd/2}) is rotated by the angle positions * theta^(-2i/hd).
    """
    hd = x.shape[-1]
    half = hd // 2
    freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = positions.astype(np.float64)[:, None] * freq[None, :]          # [n, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, q_pos0: int) -> np.ndarray:
    """Causal grouped-query softmax attention for one sequence.

    q[nq, Hq, hd] are the queries at absolute positions q_pos0 .. q_pos0+nq-1,
    k, v[nk, Hkv, hd] the keys/values at positions 0 .. nk-1.  Query head h
    reads KV head h // (Hq/Hkv).  Query at position m sees keys n <= m.
    Returns [nq, Hq, hd].
    """
    nq, hq, hd = q.shape
    nk, hkv, _ = k.shape
    rep = hq // hkv
    out = np.empty_like(q)
    qpos = q_pos0 + np.arange(nq)
    visible = np.arange(nk)[None, :] <= qpos[:, None]                     # [nq, nk]
    for h in range(hq):
        kh, vh = k[:, h // rep, :], v[:, h // rep, :]
        s = (q[:, h, :] @ kh.T) / math.sqrt(hd)
        s = np.where(visible, s, -np.inf)
        s = s - np.max(s, axis=-1, keepdims=True)
        p = np.exp(s)
        p = p / np.sum(p, axis=-1, keepdims=True)
        out[:, h, :] = p @ vh
    return out


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def _layer(m: Model, lw: dict, h: np.ndarray, positions: np.ndarray, k_prev, v_prev):
    """One decoder layer on h[n, d] (one sequence, n consecutive positions).

    k_prev/v_prev[n_prev, Hkv, hd] hold this sequence's cached keys/values of
    earlier positions (or None).  Returns (h_out, k_all, v_all).
    """
    n = h.shape[0]
    a = rmsnorm(h, lw["attn_norm"], m.eps)
    q, k, v = a @ lw["wq"].T, a @ lw["wk"].T, a @ lw["wv"].T
    if "bq" in lw:   # optional biases of the three projections (the 0.5B model family the paper ran has them)
        q, k, v = q + lw["bq"], k + lw["bk"], v + lw["bv"]
    q, k, v = q.reshape(n, m.hq, m.hd), k.reshape(n, m.hkv, m.hd), v.reshape(n, m.hkv, m.hd)
    q = rope_rotate(q, positions, m.theta)
    k = rope_rotate(k, positions, m.theta)
    if k_prev is not None:
        k = np.concatenate([k_prev, k], axis=0)
        v = np.concatenate([v_prev, v], axis=0)
    o = attention(q, k, v, int(positions[0]))
    h = h + o.reshape(n, m.hq * m.hd) @ lw["wo"].T
    b = rmsnorm(h, lw["ffn_norm"], m.eps)
    act = silu(b @ lw["w_gate"].T) * (b @ lw["w_up"].T)
    h = h + act @ lw["w_down"].T
    return h, k, v


def hidden_states(m: Model, tokens: np.ndarray, cache: Optional[list] = None) -> np.ndarray:
    """Final-norm'd hidden states for one sequence of token ids.

    tokens int[n] are the tokens at positions n_prev .. n_prev+n-1 where n_prev
    is the number of positions already in `cache` (a per-layer list of [k, v]
    that is extended in place; None = no cache, start at position 0).
    Returns float64 [n, d].
    """
    n_prev = 0 if cache is None or cache[0][0] is None else cache[0][0].shape[0]
    positions = n_prev + np.arange(len(tokens))
    h = m.embed[np.asarray(tokens, dtype=np.int64)]
    for li, lw in enumerate(m.layers):
        kp, vp = (None, None) if cache is None else cache[li]
        h, k, v = _layer(m, lw, h, positions, kp, vp)
        if cache is not None:
            cache[li] = [k, v]
    return rmsnorm(h, m.final_norm, m.eps)


def logits_from_hidden(m: Model, x: np.ndarray) -> np.ndarray:
    """x[n, d] (final-norm'd) -> logits z[n, vocab]."""
    return x @ m.lm_head.T


def forward_logits(m: Model, tokens: np.ndarray, at: Optional[Sequence[int]] = None) -> np.ndarray:
    """Full-recompute forward of one sequence; logits after consuming tokens[0..t] for t in `at`
    (all positions when None).  float64 [len(at), vocab]."""
    x = hidden_states(m, tokens)
    if at is not None:
        x = x[np.asarray(at, dtype=np.int64)]
    return logits_from_hidden(m, x)


def log_softmax(z: np.ndarray) -> np.ndarray:
    zmax = np.max(z, axis=-1, keepdims=True)
    return z - (zmax + np.log(np.sum(np.exp(z - zmax), axis=-1, keepdims=True)))


# --------------------------------------------------------------------------- #
# Sampling
# --------------------------------------------------------------------------- #
def perturbed_scores(z: np.ndarray, temperature: float, seed: int, seq: int, step: int) -> np.ndarray:
    """float32[vocab] scores y_v = z_v / T + g_v whose argmax is the sampled token.

    The decision is taken in fp32 (both sides of a parity check take it in the
    same precision): z is rounded to fp32, divided by T in fp32, and the fp32
    Gumbel noise added in fp32.
    T == 0 means greedy decoding: y = z.
    """
    z32 = np.asarray(z, dtype=np.float64).astype(np.float32)
    if temperature == 0.0:
        return z32
    g = gumbel_noise(seed, seq, step, z32.shape[0])
    return (z32 / np.float32(temperature)).astype(np.float32) + g


def sample_token(z: np.ndarray, temperature: float, seed: int, seq: int, step: int) -> int:
    """Exact sample from softmax(z / T) by Gumbel-max; ties go to the lowest id."""
    return int(np.argmax(perturbed_scores(z, temperature, seed, seq, step)))


# --------------------------------------------------------------------------- #
# The two calls of the path
# --------------------------------------------------------------------------- #
def rollout_generate(m: Model, prompts: np.ndarray, group: int, max_new: int, temperature: float,
                     seed: int, return_logits: bool = False, first_seq: int = 0):
    """Generate `group` sampled completions of max_new tokens for each prompt.

    prompts int[P, Lp].  Sequence s = first_seq + p * group + g (the index that keys the noise).  Returns
    (tokens int32 [S, max_new], logprobs float32 [S, max_new]) with
    logprobs[s, t] = log softmax(z)[token] at temperature 1 (the policy's own
    log-prob, the quantity the scoring pass reproduces).  Incremental decoding
    with a per-sequence KV cache; the prompt is run once per prompt and its
    cache copied to the siblings.
    """
    prompts = np.asarray(prompts)
    P, Lp = prompts.shape
    S = P * group
    out_tok = np.zeros((S, max_new), dtype=np.int32)
    out_lp = np.zeros((S, max_new), dtype=np.float32)
    all_logits = np.zeros((S, max_new, m.vocab), dtype=np.float64) if return_logits else None
    for p in range(P):
        pcache = [[None, None] for _ in range(m.n_layers)]
        x_last = hidden_states(m, prompts[p], pcache)[-1:]
        for g in range(group):
            s = p * group + g
            cache = [[k.copy(), v.copy()] for k, v in pcache]
            x = x_last
            for t in range(max_new):
                z = logits_from_hidden(m, x)[0]
                tok = sample_token(z, temperature, seed, first_seq + s, t)
                out_tok[s, t] = tok
                out_lp[s, t] = log_softmax(z)[tok]
                if return_logits:
                    all_logits[s, t] = z
                if t + 1 < max_new:
                    x = hidden_states(m, np.array([tok]), cache)
    if return_logits:
        return out_tok, out_lp, all_logits
    return out_tok, out_lp


def rollout_generate_ragged(m: Model, prompts: Sequence[np.ndarray], group: int, max_new: int, temperature: float,
                            seed: int):
    """Prompts of different lengths: prompt p (a 1-D array of its own length) is answered exactly as
    if it were alone, by the sequences p * group .. p * group + group - 1."""
    toks, lps = [], []
    for p, prompt in enumerate(prompts):
        t, l = rollout_generate(m, np.asarray(prompt)[None, :], group, max_new, temperature, seed, first_seq=p * group)
        toks.append(t)
        lps.append(l)
    return np.concatenate(toks, axis=0), np.concatenate(lps, axis=0)


def rollout_generate_stop(m: Model, prompts: np.ndarray, group: int, max_new: int, temperature: float,
                          seed: int, stop_token: int):
    """rollout_generate with a stop token: an answer ends with the first stop_token it samples
    (that token and its log-prob are kept); the rest of its row is stop_token with log-prob 0.
    Nothing else changes: the sampler's noise is keyed on (seed, sequence, step), so a row equals
    the unstopped row up to and including its stop.  Returns (tokens, logprobs, lengths int32 [S]),
    lengths counting the stop token, max_new where none was sampled."""
    prompts = np.asarray(prompts)
    P, Lp = prompts.shape
    S = P * group
    out_tok = np.full((S, max_new), stop_token, dtype=np.int32)
    out_lp = np.zeros((S, max_new), dtype=np.float32)
    lengths = np.full(S, max_new, dtype=np.int32)
    for p in range(P):
        pcache = [[None, None] for _ in range(m.n_layers)]
        x_last = hidden_states(m, prompts[p], pcache)[-1:]
        for g in range(group):
            s = p * group + g
            cache = [[k.copy(), v.copy()] for k, v in pcache]
            x = x_last
            for t in range(max_new):
                z = logits_from_hidden(m, x)[0]
                tok = sample_token(z, temperature, seed, s, t)
                out_tok[s, t] = tok
                out_lp[s, t] = log_softmax(z)[tok]
                if tok == stop_token:
                    lengths[s] = t + 1
                    break
                if t + 1 < max_new:
                    x = hidden_states(m, np.array([tok]), cache)
    return out_tok, out_lp, lengths


def score_logprobs(m: Model, tokens: np.ndarray, completion_mask: np.ndarray, temperature: float = 1.0) -> np.ndarray:
    """Teacher-forced per-token log-probs under the policy.

    tokens int[S, T], completion_mask uint8[S, T].  out[s, t] =
    log softmax(z_{t-1} / temperature)[tokens[s, t]] where z_{t-1} are the logits after
    consuming tokens[s, 0..t-1], for every masked (s, t) with t >= 1; 0.0
    elsewhere.  float32 [S, T].  temperature 1 is the policy's own distribution; another value
    gives the log-probs of the distribution a rollout at that temperature was sampled from.
    """
    tokens = np.asarray(tokens)
    S, T = tokens.shape
    out = np.zeros((S, T), dtype=np.float32)
    for s in range(S):
        tpos = np.nonzero(np.asarray(completion_mask[s]) != 0)[0]
        tpos = tpos[tpos >= 1]
        if tpos.size == 0:
            continue
        x = hidden_states(m, tokens[s])
        lp = log_softmax(logits_from_hidden(m, x[tpos - 1]) / temperature)
        out[s, tpos] = lp[np.arange(tpos.size), tokens[s, tpos]]
    return out


def group_advantages(rewards: np.ndarray, group: int, eps: float = 1e-6) -> np.ndarray:
    """Group-relative advantages: for each run of `group` consecutive sequences,
    A = (r - mean) / (std + eps) with the population std; a group whose rewards
    are all equal gets exactly 0.  float32 [S]."""
    r = np.asarray(rewards, dtype=np.float64)
    assert r.ndim == 1 and r.size % group == 0
    out = np.zeros(r.shape, dtype=np.float64)
    for g0 in range(0, r.size, group):
        rg = r[g0:g0 + group]
        if np.all(rg == rg[0]):
            continue
        mu = np.mean(rg)
        sd = math.sqrt(np.mean((rg - mu) ** 2))
        out[g0:g0 + group] = (rg - mu) / (sd + eps)
    return out.astype(np.float32)


def score(m: Model, tokens, completion_mask, rewards, group: int):
    """The scoring call: (log-probs [S, T], advantages [S])."""
    return score_logprobs(m, tokens, completion_mask), group_advantages(rewards, group)


def clipped_surrogate_loss(logp_new: np.ndarray, logp_old: np.ndarray, completion_mask: np.ndarray,
                           advantages: np.ndarray, eps_low: float = 0.2, eps_high: float = 0.28):
    """GRPO's clipped surrogate as the paper configures it (Sec. 4.2): no KL term,
    asymmetric clipping of the probability ratio to [1 - eps_low, 1 + eps_high] (0.2 / 0.28).

    Per masked token (s, t): rho = exp(logp_new - logp_old), A = advantages[s],
        term = min(rho * A, clip(rho, 1 - eps_low, 1 + eps_high) * A)
    loss = - mean of term over the masked tokens of the whole batch (the token-level mean
    of the DAPO recipe the section cites); 0 if nothing is masked.
    Also returns d loss / d logp_new [S, T]: -A * rho / N where the unclipped branch is the
    minimum (A >= 0 and rho <= 1 + eps_high, or A < 0 and rho >= 1 - eps_low), else 0; the
    two branches coincide inside the clip range, so the choice at equality does not matter.
    float64 throughout; returns (float, float64 [S, T]).
    """
    ln = np.asarray(logp_new, dtype=np.float64)
    lo = np.asarray(logp_old, dtype=np.float64)
    mk = np.asarray(completion_mask) != 0
    adv = np.asarray(advantages, dtype=np.float64)
    assert ln.shape == lo.shape == mk.shape and adv.shape == (ln.shape[0],)
    n = int(mk.sum())
    grad = np.zeros(ln.shape, dtype=np.float64)
    if n == 0:
        return 0.0, grad
    total = 0.0
    for s in range(ln.shape[0]):
        a = adv[s]
        for t in np.nonzero(mk[s])[0]:
            rho = math.exp(ln[s, t] - lo[s, t])
            clipped = min(max(rho, 1.0 - eps_low), 1.0 + eps_high)
            total += min(rho * a, clipped * a)
            active = (rho <= 1.0 + eps_high) if a >= 0 else (rho >= 1.0 - eps_low)
            if active:
                grad[s, t] = -a * rho / n
    return -total / n, grad


# --------------------------------------------------------------------------- #
# Training-set assembly (Sec. 3.2; Algorithm 1 "Assemble training set")
# --------------------------------------------------------------------------- #
STREAM_EXTERNAL, STREAM_LOCAL = 1, 2   # word 3 of the Philox counter (0 is the token sampler's)


def subset_keys(seed: int, stream: int, n_groups: int) -> np.ndarray:
    """uint32[n_groups]: the random key of each datapoint, word 0 of the Philox block with counter
    (g, 0, 0, stream) under the seed's key."""
    ctr = np.zeros((n_groups, 4), dtype=np.uint32)
    ctr[:, 0] = np.arange(n_groups, dtype=np.uint32)
    ctr[:, 3] = np.uint32(stream)
    key = np.array([seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF], dtype=np.uint32)
    return philox4x32_10(ctr, key)[:, 0]


def uniform_subset(eligible: np.ndarray, k: int, seed: int, stream: int) -> np.ndarray:
    """Indices of a uniformly random subset of min(k, #eligible) of the eligible datapoints, in the
    order drawn: every eligible datapoint gets an independent random key, the k smallest
    (key, index) pairs are the sample (a uniform subset because the keys are exchangeable)."""
    elig = np.nonzero(np.asarray(eligible))[0]
    keys = subset_keys(seed, stream, len(eligible))
    order = sorted(elig.tolist(), key=lambda g: (int(keys[g]), g))
    return np.asarray(order[:max(0, k)], dtype=np.int64)


def assemble_training_set(local_tokens: np.ndarray, local_rewards: np.ndarray, ext_tokens: np.ndarray,
                          ext_rewards: np.ndarray, group: int, n_local: int, n_ext: int, seed: int):
    """The training set T^n of one round: n_local datapoints (a question's whole rollout of `group`
    answers) drawn uniformly from the node's own, followed by n_ext drawn uniformly from those
    swarm datapoints whose advantage is not identically zero (all `group` rewards equal means zero
    advantage: discarded first, as in the paper's experiments).  Fewer are returned when the pool
    runs out.  Returns (tokens int32 [(n_local + n_ext) * group, T], rewards float32 [...],
    source int32 [n_local + n_ext], counts (taken local, taken external)); source g >= 0 is local
    datapoint g, external datapoint g is n_local_pool + g; unfilled slots hold zeros and source -1."""
    lt, et = np.asarray(local_tokens, np.int32), np.asarray(ext_tokens, np.int32)
    lr, er = np.asarray(local_rewards, np.float32), np.asarray(ext_rewards, np.float32)
    T = lt.shape[1] if lt.size else et.shape[1]
    pl, pe = lt.shape[0] // group, et.shape[0] // group
    take_l = uniform_subset(np.ones(pl, bool), n_local, seed, STREAM_LOCAL)
    live = np.array([not np.all(er[g * group:(g + 1) * group] == er[g * group]) for g in range(pe)], dtype=bool)
    take_e = uniform_subset(live, n_ext, seed, STREAM_EXTERNAL)
    n = n_local + n_ext
    tokens = np.zeros((n * group, T), np.int32)
    rewards = np.zeros(n * group, np.float32)
    source = np.full(n, -1, np.int32)
    for slot, g in enumerate(take_l):
        tokens[slot * group:(slot + 1) * group] = lt[g * group:(g + 1) * group]
        rewards[slot * group:(slot + 1) * group] = lr[g * group:(g + 1) * group]
        source[slot] = g
    for i, g in enumerate(take_e):
        slot = n_local + i
        tokens[slot * group:(slot + 1) * group] = et[g * group:(g + 1) * group]
        rewards[slot * group:(slot + 1) * group] = er[g * group:(g + 1) * group]
        source[slot] = pl + g
    return tokens, rewards, source, (len(take_l), len(take_e))
