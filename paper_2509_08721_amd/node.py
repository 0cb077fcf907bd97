"""One SAPO node's round (Algorithm 1) as calls into libsapo: generate rollouts, assemble the training
set from own and swarm rollouts, score it, update the policy, continue with the updated policy.

Glue only: every step runs in the library's kernels; rewards come from the caller (the node's reward
model, Sec. 3.1) and the exchange of rollouts with the swarm is the caller's business (Sec. 3.2)."""
from __future__ import annotations

from typing import Optional

from . import sapo


class Node:
    """A node n of the swarm: its policy pi^n (a weights handle for generation and scoring) and the
    trainer that improves it."""

    def __init__(self, shape, weights: dict, group: int, lr: float = 1e-3, eps_low: float = 0.2, eps_high: float = 0.28,
                 matmul_pieces: int = 3):
        self.shape, self.group = shape, group
        self.eps_low, self.eps_high = eps_low, eps_high
        self.policy = sapo.sapo_weights_create(shape, weights)
        self.trainer = sapo.sapo_trainer_create(shape, weights, lr=lr)
        sapo.sapo_trainer_set_matmul_pieces(self.trainer, matmul_pieces)
        self.rounds = 0
        self._export_buffers = None
        self._rollout_buffers = {}

    def rollouts(self, prompts, max_new: int, temperature: float, seed: int):
        """prompts int32 [P, Lp] (device).  Returns (sequences int32 [P * G, Lp + max_new]: each prompt followed by
        one of its G completions, log-probs of the completion tokens float32 [P * G, max_new])."""
        torch = sapo._torch()
        # the same workspace and output buffers for every call of a shape: the policy handle then replays the decode
        # step it captured the first time (sapo_weights_update leaves that capture valid)
        P, Lp = int(prompts.shape[0]), int(prompts.shape[1])
        key = (P, Lp, max_new)
        if key not in self._rollout_buffers:
            nbytes = sapo.sapo_rollout_workspace_bytes(self.policy, P, Lp, self.group, max_new)
            self._rollout_buffers[key] = (torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda"),
                                          torch.empty((P * self.group, max_new), dtype=torch.int32, device="cuda"),
                                          torch.empty((P * self.group, max_new), dtype=torch.float32, device="cuda"))
        ws, out_tok, out_lp = self._rollout_buffers[key]
        comp, lps = sapo.sapo_rollout_generate(self.policy, prompts, self.group, max_new, temperature, seed, workspace=ws,
                                               out_tokens=out_tok, out_logprobs=out_lp)
        return torch.cat([prompts.repeat_interleave(self.group, dim=0), comp], dim=1).contiguous(), lps.clone()

    def training_set(self, own_sequences, own_rewards, swarm_sequences, swarm_rewards, n_own: int, n_swarm: int, seed: int):
        """I^n datapoints of the node's own and J^n sampled from the swarm's, those with zero advantage discarded
        (a datapoint is a question's G sequences).  Returns (sequences, rewards) of the datapoints actually taken."""
        torch = sapo._torch()
        tok, rew, _, cnt = sapo.sapo_assemble_training_set(own_sequences, own_rewards, swarm_sequences, swarm_rewards,
                                                           self.group, n_own, n_swarm, seed)
        # the node's own datapoints fill slots 0 .. n_own - 1 and the swarm's start at slot n_own whatever the own pool
        # held, so with fewer own datapoints than asked for the slots in between are empty: take both runs, not a prefix
        taken_own, taken_swarm = (int(c) for c in cnt.cpu().tolist())
        G = self.group
        rows = torch.cat([torch.arange(0, taken_own * G, device=tok.device),
                          torch.arange(n_own * G, (n_own + taken_swarm) * G, device=tok.device)])
        return tok[rows].contiguous(), rew[rows].contiguous()

    def update(self, sequences, rewards, n_completion: int, workspace=None):
        """One PolicyGradient step on the training set: score it under the current policy (old log-probs, group-relative
        advantages), take the step, continue with the updated policy.  Returns the loss before the step (float32 [1])."""
        torch = sapo._torch()
        S, T = int(sequences.shape[0]), int(sequences.shape[1])
        mask = torch.zeros((S, T), dtype=torch.uint8, device="cuda")
        mask[:, T - n_completion:] = 1
        logp_old, adv = sapo.sapo_score_logprobs(self.policy, sequences, mask, rewards, self.group)
        loss, _ = sapo.sapo_policy_update(self.trainer, sequences, mask, logp_old, adv, self.eps_low, self.eps_high,
                                          want_logp=False, workspace=workspace)
        # the updated masters go into the policy handle in place: no allocation, and the decode step the handle
        # captured for its rollout calls stays valid
        self._export_buffers = sapo.sapo_trainer_export_into(self.trainer, self.policy, self._export_buffers)
        self.rounds += 1
        return loss

    def close(self):
        self.policy.close()
        self.trainer.close()
