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


# ----------------------------------------------------------------------------------------------
# Full-size sample checks: one oracle forward per sequence serves tokens, log-probs and logits.
# ----------------------------------------------------------------------------------------------
class SampleStats:
    """What a sample of (sequence, step) pairs showed.  `flips` holds (s, t, v_oracle, v_gpu, gap, eps) for every step
    whose token is not the oracle's argmax; eps is the measured max-abs logit error at that position."""

    def __init__(self):
        self.n = 0
        self.exact = 0
        self.flips = []
        self.max_eps = 0.0
        self.max_lp_err = 0.0
        self.sum_eps = 0.0

    def merge(self, other):
        self.n += other.n
        self.exact += other.exact
        self.flips += other.flips
        self.max_eps = max(self.max_eps, other.max_eps)
        self.max_lp_err = max(self.max_lp_err, other.max_lp_err)
        self.sum_eps += other.sum_eps
        return self

    def above(self, delta):
        return [f for f in self.flips if f[4] > delta]

    def summary(self):
        return ("%d steps, %d exact, %d flips (%d above 1e-3, largest gap %.2e), logits: max eps %.2e mean of max %.2e, max |dlogp| %.2e"
                % (self.n, self.exact, len(self.flips), len(self.above(1e-3)), max([f[4] for f in self.flips], default=0.0),
                   self.max_eps, self.sum_eps / max(1, self.n), self.max_lp_err))


def prompt_cache(model: O.Model, prompt):
    """The oracle's K/V of a prompt (shared by the prompt's sibling sequences) and nothing else."""
    cache = [[None, None] for _ in range(model.n_layers)]
    O.hidden_states(model, np.asarray(prompt), cache)
    return cache


def check_sequence(model: O.Model, seq, Lp, steps, s, *, device_logits, gpu_tokens=None, gpu_logprobs=(),
                   temperature=1.0, seed=0, cache=None, chunk=256) -> SampleStats:
    """Teacher-forced check of generated-token indices `steps` of one sequence (seq = prompt + completion, s = its
    index in the batch, which keys the noise).

    The oracle runs the sequence once (full recompute, or the completion on top of the prompt's K/V when `cache`
    is given: the two are pinned equal) and yields the logits z_t after tokens 0 .. Lp + t - 1.  Against them:
      * device_logits(positions) -> float32 [n, V]: the device's teacher-forced logits at sequence positions
        Lp - 1 + t (eps = max-abs difference per position);
      * gpu_tokens[t] (optional): the token the device chose at step t against the argmax of the oracle's perturbed
        scores z / T + g;
      * gpu_logprobs: rows (indexed by t) of the device's log softmax(z)[token], e.g. the rollout's and the scoring
        pass's, each against the oracle's for the token in seq."""
    st = SampleStats()
    seq = np.asarray(seq)
    steps = sorted(int(t) for t in steps)
    last = Lp + steps[-1]                       # tokens consumed for the deepest checked step
    if cache is None:
        x = O.hidden_states(model, seq[:last])
        row0 = 0
    else:
        # the prompt's last position is needed for step 0: run it again on a cache cut by one position
        own = [[k[:Lp - 1].copy(), v[:Lp - 1].copy()] for k, v in cache]
        x = O.hidden_states(model, seq[Lp - 1:last], own)
        row0 = Lp - 1
    for c0 in range(0, len(steps), chunk):
        ts = steps[c0:c0 + chunk]
        pos = [Lp - 1 + t for t in ts]
        z = O.logits_from_hidden(model, x[[p - row0 for p in pos]])
        zd = np.asarray(device_logits(pos), dtype=np.float64)
        eps = np.max(np.abs(zd - z), axis=1)
        lp = O.log_softmax(z)
        for i, t in enumerate(ts):
            tok = int(seq[Lp + t])
            st.n += 1
            st.max_eps = max(st.max_eps, float(eps[i]))
            st.sum_eps += float(eps[i])
            for row in (gpu_logprobs or ()):
                st.max_lp_err = max(st.max_lp_err, abs(float(lp[i, tok]) - float(row[t])))
            if gpu_tokens is None:
                st.exact += 1
                continue
            assert int(gpu_tokens[t]) == tok
            y = O.perturbed_scores(z[i], temperature, seed, s, t)
            v_star = int(np.argmax(y))
            if v_star == tok:
                st.exact += 1
            else:
                st.flips.append((s, t, v_star, tok, float(y[v_star]) - float(y[tok]), float(eps[i])))
    return st


def measured_logit_eps(sapo, gw, model: O.Model, seq, first_pos: int) -> float:
    """Largest abs difference between the device's teacher-forced logits (sapo_debug_logits, the sequence as a batch of
    one) and the oracle's over positions first_pos .. len(seq) - 2 of one sequence: the logit error a near-tie band is
    widened by."""
    import torch
    seq = np.asarray(seq, dtype=np.int32)
    pos = list(range(first_pos, len(seq) - 1))
    zd = sapo.sapo_debug_logits(gw, torch.from_numpy(seq[None, :].copy()).cuda(), [(0, p) for p in pos]).cpu().numpy()
    z = O.forward_logits(model, seq[:-1], at=pos)
    return float(np.max(np.abs(zd.astype(np.float64) - z)))
