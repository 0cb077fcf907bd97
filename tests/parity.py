"""Helpers shared by the GPU parity tests (not collected by pytest)."""
from __future__ import annotations

import numpy as np

from oracle import sapo_oracle as O


def gpu_available() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def teacher_forced_token_check(model: O.Model, prompts, group, gpu_tokens, temperature, seed, seqs, steps=None,
                               delta=1e-3):
    """Per-step token parity: feed the GPU's own prefix to the oracle, recompute the perturbed
    scores y = z/T + g and compare the GPU's token with the oracle's argmax.

    Returns (n_checked, n_exact, near_ties, failures) where near_ties/failures are lists of
    (s, t, v_oracle, v_gpu, gap); a step is a stated near-tie when the top perturbed score
    exceeds the GPU token's score by at most delta.
    """
    gpu_tokens = np.asarray(gpu_tokens)
    Lp = prompts.shape[1]
    N = gpu_tokens.shape[1]
    n = exact = 0
    near, bad = [], []
    worst_lp = 0.0
    for s in seqs:
        seq = np.concatenate([prompts[s // group], gpu_tokens[s]])
        ts = list(range(N)) if steps is None else list(steps)
        z = O.forward_logits(model, seq[: Lp + max(ts)], at=[Lp - 1 + t for t in ts])
        for i, t in enumerate(ts):
            y = O.perturbed_scores(z[i], temperature, seed, s, t)
            v_star, v_gpu = int(np.argmax(y)), int(gpu_tokens[s, t])
            n += 1
            if v_star == v_gpu:
                exact += 1
                continue
            gap = float(y[v_star]) - float(y[v_gpu])
            (near if gap <= delta else bad).append((s, t, v_star, v_gpu, gap))
    return n, exact, near, bad


def oracle_logprobs_for(model: O.Model, prompts, group, gpu_tokens, seqs):
    """Oracle log softmax(z)[token] along the GPU's own sequences: dict s -> float64 [N]."""
    Lp = prompts.shape[1]
    N = gpu_tokens.shape[1]
    out = {}
    for s in seqs:
        seq = np.concatenate([prompts[s // group], gpu_tokens[s]])
        z = O.forward_logits(model, seq[:-1], at=range(Lp - 1, Lp + N - 1))
        lp = O.log_softmax(z)
        out[s] = lp[np.arange(N), gpu_tokens[s]]
    return out
