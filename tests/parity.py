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


def check_rollout_steps(model: O.Model, prompts, group, gpu_tokens, gpu_logprobs, temperature, seed, seq_steps,
                        delta):
    """One oracle forward per checked sequence, used for tokens and log-probs alike.

    seq_steps: dict sequence -> list of steps (None = every step).  The oracle runs on the GPU's own
    prefix (teacher-forced), recomputes the perturbed scores and the log-prob of the GPU's token.
    Returns dict(n, exact, near, bad, max_lp_err, max_gap) with near/bad lists of
    (s, t, v_oracle, v_gpu, gap)."""
    gpu_tokens = np.asarray(gpu_tokens)
    Lp, N = prompts.shape[1], gpu_tokens.shape[1]
    out = dict(n=0, exact=0, near=[], bad=[], max_lp_err=0.0, max_gap=0.0)
    for s, steps in seq_steps.items():
        ts = list(range(N)) if steps is None else sorted(steps)
        seq = np.concatenate([prompts[s // group], gpu_tokens[s]])
        z = O.forward_logits(model, seq[: Lp + ts[-1]], at=[Lp - 1 + t for t in ts])
        lp = O.log_softmax(z)
        for i, t in enumerate(ts):
            v_gpu = int(gpu_tokens[s, t])
            out["max_lp_err"] = max(out["max_lp_err"], abs(float(lp[i, v_gpu]) - float(gpu_logprobs[s, t])))
            y = O.perturbed_scores(z[i], temperature, seed, s, t)
            v_star = int(np.argmax(y))
            out["n"] += 1
            if v_star == v_gpu:
                out["exact"] += 1
                continue
            gap = float(y[v_star]) - float(y[v_gpu])
            out["max_gap"] = max(out["max_gap"], gap)
            (out["near"] if gap <= delta else out["bad"]).append((s, t, v_star, v_gpu, gap))
    return out
