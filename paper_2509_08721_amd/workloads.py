"""Seeded synthetic inputs for the SAPO node loop (rollout generation + scoring).

This module only *makes inputs*: model shapes, random weights, prompt token ids,
rewards and completion masks.  It holds none of the method's arithmetic (no
forward pass, no sampling, no log-probs, no advantages) so that both the CPU
oracle's tests and the HIP path's tests can draw identical bytes from it.

The workloads mirror one node-round of the paper's controlled experiment
(Sec. 4.1 / Sec. 5: 8 questions x 8 completions per agent per round, a
0.5B-parameter decoder-only LM, binary verifier rewards, and the 4 local /
4 external training-set mix of Sec. 5).  The paper's prompts come from a
procedurally generated reasoning dataset and its weights from a public
checkpoint; neither is available here, so prompts are Zipf-distributed token
ids and weights are Gaussian.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional

import numpy as np


# --------------------------------------------------------------------------- #
# bf16 <-> fp32 bit conversions (storage format helpers, round-to-nearest-even)
# --------------------------------------------------------------------------- #
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 array of bf16 bit patterns (RNE; inputs are finite)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> fp32 array with the same values."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- #
# Model shapes
# --------------------------------------------------------------------------- #
@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    rms_eps: float = 1e-6
    rope_theta: float = 1e4
    tied_embeddings: bool = True
    dtype: str = "f32"          # "f32" or "bf16": storage type of weights and KV cache
    kv_page_tokens: int = 16
    max_seq: int = 2048

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    def matmul_params_per_layer(self) -> int:
        d, q, kv, f = self.d_model, self.q_dim, self.kv_dim, self.d_ff
        return d * q + 2 * d * kv + q * d + 3 * d * f

    def weight_bytes_per_decode_step(self) -> int:
        """Bytes of weights every decode step has to stream (matrices + gains + LM head)."""
        elt = 4 if self.dtype == "f32" else 2
        n = self.n_layers * self.matmul_params_per_layer() + self.vocab * self.d_model
        if not self.tied_embeddings:
            pass  # the embedding itself is only gathered, never streamed
        n += (2 * self.n_layers + 1) * self.d_model
        return n * elt

    def kv_bytes_per_token(self) -> int:
        elt = 4 if self.dtype == "f32" else 2
        return 2 * self.kv_dim * self.n_layers * elt


TINY = ModelShape(n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ff=172,
                  vocab=512, rms_eps=1e-6, rope_theta=1e4, tied_embeddings=True, dtype="f32",
                  max_seq=256)
HALF_B = ModelShape(n_layers=24, d_model=896, n_q_heads=14, n_kv_heads=2, head_dim=64, d_ff=4864,
                    vocab=151936, rms_eps=1e-6, rope_theta=1e6, tied_embeddings=True, dtype="bf16",
                    max_seq=2048)
# Small bf16 shapes that satisfy the tile alignment of the MFMA kernels (tests only).
MINI_BF16 = ModelShape(n_layers=2, d_model=128, n_q_heads=4, n_kv_heads=2, head_dim=64, d_ff=256,
                       vocab=1024, rms_eps=1e-6, rope_theta=1e4, tied_embeddings=True, dtype="bf16",
                       max_seq=512)
MINI_BF16_HD128 = ModelShape(n_layers=2, d_model=256, n_q_heads=6, n_kv_heads=1, head_dim=128, d_ff=320,
                             vocab=640, rms_eps=1e-6, rope_theta=1e6, tied_embeddings=False, dtype="bf16",
                             max_seq=512)
ONE_HALF_B = ModelShape(n_layers=28, d_model=1536, n_q_heads=12, n_kv_heads=2, head_dim=128,
                        d_ff=8960, vocab=151936, rms_eps=1e-6, rope_theta=1e6,
                        tied_embeddings=True, dtype="bf16", max_seq=2048)


# --------------------------------------------------------------------------- #
# Workloads (the five configurations)
# --------------------------------------------------------------------------- #
@dataclass(frozen=True)
class Workload:
    name: str
    shape: ModelShape
    weight_seed: int
    # rollout part (None of it used when n_new == 0)
    n_prompts: int = 0
    group: int = 8              # completions per prompt (L^n in the paper)
    prompt_len: int = 0
    n_new: int = 0
    temperature: float = 1.0
    prompt_dist: str = "zipf"   # "zipf" (exponent 1.1) or "uniform"
    prompt_seed: int = 0
    rollout_seed: int = 0
    # scoring part
    score_seqs: int = 0
    score_len: int = 0
    score_masked: int = 0       # completion mask covers the last score_masked positions
    reward_p: float = 0.5
    reward_seed: int = 0
    external_weight_seed: Optional[int] = None   # weights of the "other node" (config 4)
    # answers of different lengths: rollouts end at stop_token, whose LM-head row is scaled by 2^stop_boost
    # (boost_token) so that lengths spread between a few tokens and n_new
    stop_token: int = -1
    stop_boost: int = 0

    @property
    def n_seqs(self) -> int:
        return self.n_prompts * self.group


WORKLOADS: Dict[str, Workload] = {
    # 1: tiny fp32 decoder, 2 prompts x 4 completions, 16 + 16 tokens, then score all 8.
    "tiny": Workload("tiny", TINY, weight_seed=101, n_prompts=2, group=4, prompt_len=16, n_new=16,
                     temperature=1.0, prompt_dist="uniform", prompt_seed=102, rollout_seed=103,
                     score_seqs=8, score_len=32, score_masked=16, reward_p=0.5, reward_seed=104),
    # 2: one node-round of the paper's experiment on a 0.5B-class decoder.
    "halfb_rollout": Workload("halfb_rollout", HALF_B, weight_seed=201, n_prompts=8, group=8,
                              prompt_len=128, n_new=256, temperature=1.0, prompt_seed=202,
                              rollout_seed=203, score_seqs=64, score_len=384, score_masked=256,
                              reward_p=0.3, reward_seed=204),
    # 3: long generation, KV-cache bound, temperature 0.7.
    "halfb_long": Workload("halfb_long", HALF_B, weight_seed=201, n_prompts=8, group=8,
                           prompt_len=512, n_new=1024, temperature=0.7, prompt_seed=302,
                           rollout_seed=303),
    # 4: scoring of a half local / half external batch (the 4/4 mix of Sec. 5).
    "halfb_score_mixed": Workload("halfb_score_mixed", HALF_B, weight_seed=201, n_prompts=4,
                                  group=8, prompt_len=256, n_new=512, temperature=1.0,
                                  prompt_seed=402, rollout_seed=403, score_seqs=64, score_len=768,
                                  score_masked=512, reward_p=0.3, reward_seed=404,
                                  external_weight_seed=411),
    # 5: 1.5B-class decoder, 32 prompts x 8, then score all 256.
    "onehalfb": Workload("onehalfb", ONE_HALF_B, weight_seed=501, n_prompts=32, group=8,
                         prompt_len=256, n_new=512, temperature=1.0, prompt_seed=502,
                         rollout_seed=503, score_seqs=256, score_len=768, score_masked=512,
                         reward_p=0.3, reward_seed=504),
    # not one of the five: the shape of the paper's pass@1 judge (Sec. 5, the demo's evaluation):
    # one question, one completion - decode at batch 1, bound by latency, not by bandwidth.
    # not one of the five: the local policy update (Algorithm 1's PolicyGradient step) on the training set of
    # one node-round of configuration 2 (64 sequences of 128 + 256 tokens, completions masked).
    "halfb_update": Workload("halfb_update", HALF_B, weight_seed=201, n_prompts=8, group=8, prompt_len=128,
                             n_new=0, prompt_seed=202, score_seqs=64, score_len=384, score_masked=256,
                             reward_p=0.3, reward_seed=204),
    # the same for configuration 5 (1.5B-class decoder, 256 sequences of 256 + 512 tokens): the activations of the
    # whole set would not fit one GPU, the update runs in micro-batches
    "onehalfb_update": Workload("onehalfb_update", ONE_HALF_B, weight_seed=501, n_prompts=32, group=8, prompt_len=256,
                                n_new=0, prompt_seed=502, score_seqs=256, score_len=768, score_masked=512,
                                reward_p=0.3, reward_seed=504),
    # not one of the five: configuration 5's rollouts with answers of different lengths (a stop token), where
    # ended sequences leave the decode batch
    "onehalfb_stop": Workload("onehalfb_stop", ONE_HALF_B, weight_seed=501, n_prompts=32, group=8, prompt_len=256,
                              n_new=512, temperature=1.0, prompt_seed=502, rollout_seed=503, stop_token=1000,
                              stop_boost=4),
    # not one of the five: one whole round of Algorithm 1 for one node on configuration 2's shapes - rollouts for 8
    # questions, a training set of 4 own + 4 swarm datapoints (the best mix of Sec. 5), scoring, the policy update,
    # the updated policy in place for the next round
    "halfb_round": Workload("halfb_round", HALF_B, weight_seed=201, n_prompts=8, group=8, prompt_len=128, n_new=256,
                            temperature=1.0, prompt_seed=202, rollout_seed=203, score_seqs=64, score_len=384,
                            score_masked=256, reward_p=0.3, reward_seed=204, external_weight_seed=211),
    "halfb_pass1": Workload("halfb_pass1", HALF_B, weight_seed=201, n_prompts=1, group=1,
                            prompt_len=128, n_new=256, temperature=1.0, prompt_seed=602,
                            rollout_seed=603),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (smaller cases for tests)."""
    return replace(w, **kw)


# --------------------------------------------------------------------------- #
# Weights
# --------------------------------------------------------------------------- #
LAYER_TENSORS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


def layer_tensor_shapes(s: ModelShape) -> Dict[str, tuple]:
    d, q, kv, f = s.d_model, s.q_dim, s.kv_dim, s.d_ff
    return {"attn_norm": (d,), "wq": (q, d), "wk": (kv, d), "wv": (kv, d), "wo": (d, q),
            "ffn_norm": (d,), "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f)}


def boost_token(weights: dict, shape: ModelShape, token: int, log2_scale: int) -> dict:
    """A copy of `weights` whose LM-head row of `token` (the embedding row when the head is tied) is multiplied by
    2^log2_scale, exactly in either storage type: the token's logit then swings that much more from position to
    position, so a stop token placed there ends sequences after a spread of lengths (random heads of the
    workloads' scale would emit any given token about once in `vocab` steps)."""
    out = dict(weights)
    key = "embed" if weights.get("lm_head") is None else "lm_head"
    m = np.array(weights[key], copy=True)
    if m.dtype == np.uint16:     # bf16 bit patterns: the exponent field starts at bit 7
        row = m[token].astype(np.int32)
        expo = (row >> 7) & 0xFF
        assert np.all((expo == 0) | ((expo + log2_scale > 0) & (expo + log2_scale < 255)))
        m[token] = np.where(expo == 0, row, row + (log2_scale << 7)).astype(np.uint16)
    else:
        m[token] = m[token] * np.float32(2.0 ** log2_scale)
    out[key] = m
    return out


def make_weights(shape: ModelShape, seed: int, std: float = 0.02) -> dict:
    """Random model weights.

    Every matrix (embedding included) is N(0, std^2); every RMSNorm gain is 1.
    Matrices are row-major [out_features, in_features] (y = x W^T).
    For dtype "f32" arrays are float32; for "bf16" they are uint16 bf16 bit
    patterns (each fp32 draw rounded to nearest-even once).  Gains are always
    float32.  Tensor i draws from its own generator default_rng([seed, i]).
    """
    def mat(idx: int, shp: tuple) -> np.ndarray:
        rng = np.random.default_rng([seed, idx])
        x = rng.standard_normal(shp, dtype=np.float32) * np.float32(std)
        return x if shape.dtype == "f32" else f32_to_bf16_bits(x)

    shapes = layer_tensor_shapes(shape)
    w = {"embed": mat(0, (shape.vocab, shape.d_model)), "layers": []}
    idx = 1
    for _ in range(shape.n_layers):
        lw = {}
        for name in LAYER_TENSORS:
            if name.endswith("norm"):
                lw[name] = np.ones(shapes[name], dtype=np.float32)
            else:
                lw[name] = mat(idx, shapes[name])
            idx += 1
        w["layers"].append(lw)
    w["final_norm"] = np.ones((shape.d_model,), dtype=np.float32)
    w["lm_head"] = None if shape.tied_embeddings else mat(idx, (shape.vocab, shape.d_model))
    return w


def add_qkv_bias(weights: dict, shape: ModelShape, seed: int, std: float = 0.1) -> dict:
    """A copy of the weights with float32 biases bq [q], bk [kv], bv [kv] on the three attention
    projections of every layer (N(0, std^2), generator default_rng([seed, 7, layer]))."""
    out = dict(weights)
    out["layers"] = []
    for l, lw in enumerate(weights["layers"]):
        rng = np.random.default_rng([seed, 7, l])
        lw = dict(lw)
        lw["bq"] = (rng.standard_normal(shape.q_dim) * std).astype(np.float32)
        lw["bk"] = (rng.standard_normal(shape.kv_dim) * std).astype(np.float32)
        lw["bv"] = (rng.standard_normal(shape.kv_dim) * std).astype(np.float32)
        out["layers"].append(lw)
    return out


def perturb_norm_gains(weights: dict, seed: int, spread: float = 0.25) -> dict:
    """Same weights but with non-trivial RMSNorm gains 1 + U(-spread, spread) (test helper:
    all-ones gains would hide a missing or misplaced gain multiply)."""
    rng = np.random.default_rng([seed, 9999])
    out = {"embed": weights["embed"], "lm_head": weights["lm_head"], "layers": []}
    for lw in weights["layers"]:
        nl = dict(lw)
        for name in ("attn_norm", "ffn_norm"):
            nl[name] = (1.0 + rng.uniform(-spread, spread, lw[name].shape)).astype(np.float32)
        out["layers"].append(nl)
    out["final_norm"] = (1.0 + rng.uniform(-spread, spread, weights["final_norm"].shape)).astype(np.float32)
    return out


def weights_as_f32(shape: ModelShape, weights: dict) -> dict:
    """The same values as float32 arrays whatever the storage type (exact for bf16)."""
    def cv(a):
        if a is None:
            return None
        return bf16_bits_to_f32(a) if a.dtype == np.uint16 else a
    return {"embed": cv(weights["embed"]),
            "layers": [{k: cv(v) for k, v in lw.items()} for lw in weights["layers"]],
            "final_norm": weights["final_norm"], "lm_head": cv(weights["lm_head"])}


# --------------------------------------------------------------------------- #
# Prompts, rewards, masks
# --------------------------------------------------------------------------- #
def zipf_token_ids(n: int, vocab: int, exponent: float, rng: np.random.Generator) -> np.ndarray:
    """n token ids with P(id = r-1) proportional to r^-exponent over the finite ranks 1..vocab
    (inverse CDF on the normalised table)."""
    ranks = np.arange(1, vocab + 1, dtype=np.float64)
    cdf = np.cumsum(ranks ** (-exponent))
    cdf /= cdf[-1]
    u = rng.random(n)
    ids = np.searchsorted(cdf, u, side="left")
    return np.minimum(ids, vocab - 1).astype(np.int32)


def make_prompts(w: Workload) -> np.ndarray:
    """int32 [n_prompts, prompt_len] prompt token ids."""
    rng = np.random.default_rng([w.prompt_seed, 1])
    n = w.n_prompts * w.prompt_len
    if w.prompt_dist == "uniform":
        ids = rng.integers(0, w.shape.vocab, size=n, dtype=np.int64).astype(np.int32)
    else:
        ids = zipf_token_ids(n, w.shape.vocab, 1.1, rng)
    return ids.reshape(w.n_prompts, w.prompt_len)


def make_rewards(n_seqs: int, p: float, seed: int) -> np.ndarray:
    """float32 [n_seqs] verifier-style rewards: 1 with probability p, else 0 (Sec. 4.3)."""
    rng = np.random.default_rng([seed, 2])
    return (rng.random(n_seqs) < p).astype(np.float32)


def make_completion_mask(n_seqs: int, seq_len: int, n_last: int) -> np.ndarray:
    """uint8 [n_seqs, seq_len]: 1 on the last n_last positions of every sequence."""
    m = np.zeros((n_seqs, seq_len), dtype=np.uint8)
    if n_last > 0:
        m[:, seq_len - n_last:] = 1
    return m


def make_random_tokens(n_seqs: int, seq_len: int, vocab: int, seed: int, dist: str = "zipf") -> np.ndarray:
    """int32 [n_seqs, seq_len] token ids for scoring-only inputs (stand-in for rollouts
    produced elsewhere, e.g. by another node's policy)."""
    rng = np.random.default_rng([seed, 3])
    if dist == "uniform":
        return rng.integers(0, vocab, size=(n_seqs, seq_len), dtype=np.int64).astype(np.int32)
    return zipf_token_ids(n_seqs * seq_len, vocab, 1.1, rng).reshape(n_seqs, seq_len)
