#!/usr/bin/env python3
"""Benchmark of the SAPO node hot path on one MI355X.

One step = one pass of the whole path over one batch: rollout generation
(sapo_rollout_generate: prefill of the unique prompts, then autoregressive decode of all
completions) followed by the scoring pass over the generated batch (sapo_score_logprobs:
teacher-forced log-probs on the completion positions + group-relative advantages).
The default workload is one node-round of the paper's experiment (8 questions x 8
completions, Sec. 4.1 / Sec. 5) on the 0.5B-class decoder with synthetic weights and prompts.
Other workloads (--workload): halfb_round (one whole round of Algorithm 1 for one node), halfb_long (rollout only, long generation), halfb_score_mixed
(scoring only, half local / half external rollouts; the batch is prepared untimed), onehalfb
(1.5B-class decoder, rollout + scoring), tiny, halfb_pass1 (one sequence: the latency of a
decode step at batch 1), halfb_update / onehalfb_update (the local policy update on configuration 2's / 5's training set:
trained tokens/s; --pieces 1 for bf16 GEMM operands).

The default invocation also times, a few steps each, the other full-size configurations (halfb_long, halfb_score_mixed,
onehalfb) and reports them under "other_configs" of the same line; the headline fields stay those of the default workload.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
from dataclasses import replace
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
MFMA_16BIT_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 / fp16 MFMA, published


def algorithmic_bytes_rollout(shape, P, G, Lp, N):
    """Decode bytes of one rollout call: (N-1) weight passes + KV reads + KV writes.
    KV reads count a prompt's K/V once per group per step ("shared") or once per sequence."""
    S = P * G
    W = shape.weight_bytes_per_decode_step()
    kvb = shape.kv_bytes_per_token()
    tri = sum(range(1, N))
    shared = kvb * (P * (N - 1) * Lp + S * tri)
    unshared = kvb * S * sum(Lp + t for t in range(1, N))
    write = kvb * (P * Lp + S * (N - 1))
    return {"weights": (N - 1) * W, "kv_read_shared": shared, "kv_read_unshared": unshared, "kv_write": write}


def algorithmic_flops_score(shape, S, T, Tm):
    layers = 2 * shape.n_layers * shape.matmul_params_per_layer() * S * T
    lm = 2 * shape.vocab * shape.d_model * S * Tm
    attn = 2 * T * T * shape.q_dim * shape.n_layers * S
    return {"layers": layers, "lm_head": lm, "attention": attn, "total": layers + lm + attn}


def per_launch_work(shape, plan, kernel, launches):
    """Algorithmic bytes (HBM-bound kernels) or flops (MFMA-bound kernels) one launch of a kernel
    processes in one step of this workload, averaged over the launches of the step."""
    L, d, V = shape.n_layers, shape.d_model, shape.vocab
    S, N, Lp, P = plan["S"], plan["N"], plan["Lp"], plan["P"]
    T, Tm, Ss = plan["T"], plan["Tm"], plan["S_score"]
    dec_steps = max(N - 1, 0) if plan["rollout"] else 0
    big_tokens = (P * Lp if plan["rollout"] else 0) + (Ss * T if plan["score"] else 0)
    ffn_params = 3.0 * d * shape.d_ff
    if kernel == "k_gemm_skinny":       # the projection GEMMs of a decode layer that run on the register-direct kernel
        params = shape.matmul_params_per_layer() - (ffn_params if plan["ffn_big"] else 0.0)
        return "hbm", 2.0 * params * L * dec_steps / launches
    if kernel == "k_decode_layers":     # every layer of a decode step in one launch: the layers' matrices + the cached K/V
        kv = 2 * shape.kv_dim * 2 * L * S * sum(Lp + t for t in range(1, N))
        return "hbm", (2.0 * shape.matmul_params_per_layer() * L * dec_steps + kv) / launches
    if kernel == "k_gemm_big_decode":   # gate/up and down projections of a decode layer on the token-parallel kernel
        return "hbm", 2.0 * ffn_params * L * dec_steps / launches
    if kernel == "k_lmhead_sample":     # LM head of one decode step: the whole [V, d] matrix
        return "hbm", 2.0 * V * d
    if kernel == "k_decode_attention":  # K and V of every cached token of every sequence, one layer
        kv_layer = 2 * shape.kv_dim * 2
        tot = kv_layer * S * sum(Lp + t for t in range(1, N)) * L
        return "hbm", tot / launches
    if kernel == "k_decode_attention_shared":   # the same with a prompt's full page pairs read once per group of siblings
        kv_layer = 2 * shape.kv_dim * 2
        shared_tokens = (Lp // 32) * 32
        tot = kv_layer * L * sum(P * shared_tokens + S * (Lp + t - shared_tokens) for t in range(1, N))
        return "hbm", tot / launches
    if kernel == "k_gemm_big":          # projection GEMMs of prefill + scoring (+ LM head where logits are materialised)
        fl = 2.0 * L * shape.matmul_params_per_layer() * big_tokens
        if plan["rollout"] and not plan["fused_lm"]:
            fl += 2.0 * V * d * S * N
        return "mfma", fl / launches
    if kernel == "k_lmhead_score":
        return "mfma", 2.0 * V * d * Ss * Tm / launches
    if kernel in ("k_attention", "k_flash_attention"):
        fl = 2.0 * shape.q_dim * L * ((Ss * T * T if plan["score"] else 0) + (P * Lp * Lp if plan["rollout"] else 0))
        return "mfma", fl / launches
    return None, 0.0


FP32_MFMA_PEAK_TFLOPS = 157.3


def update_flops(shape, S, T, Tm):
    """(GEMM flops, attention flops) of one policy update: every projection three times (forward, d input, d weight),
    the LM head three times on the rows that predict a masked token (Tm per sequence); attention's seven products
    (scores twice, P V, dP, dQ, dK, dV) over the causal half of T x T."""
    M = S * T
    per_layer = shape.matmul_params_per_layer()
    proj = 2 * M * 3 * per_layer * shape.n_layers
    head = 2 * S * Tm * 3 * shape.vocab * shape.d_model
    attn = 2 * 7 * S * shape.n_q_heads * (T * (T + 1) // 2) * shape.head_dim * shape.n_layers
    return proj + head, attn


def bench_stop(args, wl):
    """Rollouts with a stop token (answers of different lengths): generated tokens/s with ended sequences leaving
    the decode batch, and the same call with every sequence kept in the batch to the end."""
    import torch
    from paper_2509_08721_amd import sapo, workloads as W
    shape = wl.shape
    torch.cuda.set_device(0)
    t0 = time.time()
    weights = W.boost_token(W.make_weights(shape, wl.weight_seed), shape, wl.stop_token, wl.stop_boost)
    gw = sapo.sapo_weights_create(shape, weights)
    P, G, Lp, N = wl.n_prompts, wl.group, wl.prompt_len, wl.n_new
    S = P * G
    prompts_np = W.make_prompts(wl)
    prompts = torch.from_numpy(prompts_np).cuda()
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    torch.cuda.set_stream(side)
    ws = torch.empty(sapo.sapo_rollout_workspace_bytes(gw, P, Lp, G, N) + 256, dtype=torch.uint8, device="cuda")
    bufs = (torch.empty((S, N), dtype=torch.int32, device="cuda"), torch.empty((S, N), dtype=torch.float32, device="cuda"),
            torch.empty((S,), dtype=torch.int32, device="cuda"))
    setup_s = time.time() - t0
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]

    def timed(compact):
        if not compact:
            os.environ["SAPO_NO_COMPACT"] = "1"
        try:
            ms, last = [], None
            for i in range(args.warmup + args.steps):
                ev[0].record()
                last = sapo.sapo_rollout_generate_stop(gw, prompts, G, N, wl.temperature, wl.rollout_seed + i, wl.stop_token,
                                                       workspace=ws, out=bufs)
                ev[1].record()
                torch.cuda.synchronize()
                if i >= args.warmup:
                    ms.append((ev[0].elapsed_time(ev[1]), int(last[2].sum().item())))
            return ms, last, sapo.sapo_rollout_last_stats(gw)
        finally:
            os.environ.pop("SAPO_NO_COMPACT", None)

    ms_c, last_c, stats_c = timed(True)
    ms_n, last_n, stats_n = timed(False)
    rate = lambda runs: float(np.median([tok / (m * 1e-3) for m, tok in runs]))
    lens = last_c[2].cpu().numpy().astype(np.int64)
    # algorithmic bytes of the last timed call: one pass over the weights per decode step that some sequence still
    # needs, K/V of every running sequence's own tokens, a prompt's K/V once per group with a running sibling
    Wb, kvb = shape.weight_bytes_per_decode_step(), shape.kv_bytes_per_token()
    steps_needed = int(lens.max()) - 1
    t_idx = np.arange(1, steps_needed + 1)
    running = lens[None, :] > t_idx[:, None]                              # [steps, S]
    groups_running = running.reshape(len(t_idx), P, G).any(axis=2).sum(axis=1)
    kv_read = kvb * float((running * t_idx[:, None]).sum() + (groups_running * Lp).sum())
    kv_write = kvb * float(P * Lp + running.sum())
    alg_bytes = steps_needed * Wb + kv_read + kv_write
    ms_last = ms_c[-1][0]
    gbs = alg_bytes / (ms_last * 1e-3) / 1e9
    out = {"metric": "generated tokens/s of rollouts with a stop token (%s, 1 GPU)" % wl.name,
           "value": round(rate(ms_c), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(float(np.median([m for m, _ in ms_c])), 3), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f16", "data": "synthetic",
           "config": {"workload": wl.name, "layers": shape.n_layers, "d_model": shape.d_model, "vocab": shape.vocab,
                      "prompts": P, "completions_per_prompt": G, "prompt_len": Lp, "max_new": N,
                      "stop_token": wl.stop_token, "stop_row_scale": 2 ** wl.stop_boost,
                      "lengths": {"mean": round(float(lens.mean()), 1), "min": int(lens.min()), "max": int(lens.max()),
                                  "quartiles": [int(x) for x in np.percentile(lens, [25, 50, 75])],
                                  "at_max_new": int((lens == N).sum())}},
           "generated_tokens": int(lens.sum()),
           "batch_compacted": {"tokens_per_s": round(rate(ms_c), 1), "ms": round(float(np.median([m for m, _ in ms_c])), 3), **stats_c},
           "batch_kept_whole": {"tokens_per_s": round(rate(ms_n), 1), "ms": round(float(np.median([m for m, _ in ms_n])), 3), **stats_n},
           "roofline": {"kernel": "the decode steps of the call (all kernels)", "bound": "hbm", "achieved": round(gbs, 1),
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None,
                        "algorithmic_bytes": alg_bytes},
           "cpu_baseline": None, "setup_s": round(setup_s, 1)}
    if not args.no_cpu_baseline:
        from oracle import sapo_oracle as O
        m = O.Model(shape, weights)
        t1 = time.perf_counter()
        O.rollout_generate_stop(m, prompts_np[:1, :32], 1, 4, wl.temperature, wl.rollout_seed, wl.stop_token)
        dtc = time.perf_counter() - t1
        out["cpu_baseline"] = {"value": round(4 / dtc, 3), "unit": "tokens/s", "cores": len(os.sched_getaffinity(0)),
                               "kind": "oracle", "sample": "numpy fp64 oracle: 1 sequence, 32-token prompt, 4 new tokens in %.1f s" % dtc}
    print(json.dumps(out))


def bench_round(args, wl):
    """One node's round of Algorithm 1, every step in the library: rollouts -> (rewards: an input) -> training set of
    own and swarm datapoints -> scoring -> policy update -> updated policy in place.  The swarm's rollouts are
    generated beforehand by a second set of weights (they arrive over the network in the paper's setting)."""
    import torch
    from paper_2509_08721_amd import sapo, workloads as W
    from paper_2509_08721_amd.node import Node
    shape = wl.shape
    torch.cuda.set_device(0)
    t0 = time.time()
    P, G, Lp, N = wl.n_prompts, wl.group, wl.prompt_len, wl.n_new
    S, T = P * G, Lp + N
    n_own, n_swarm = P // 2, P // 2
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    torch.cuda.set_stream(side)
    node = Node(shape, W.make_weights(shape, wl.weight_seed), G, matmul_pieces=args.pieces)
    other = Node(shape, W.make_weights(shape, wl.external_weight_seed), G)
    prompts = torch.from_numpy(W.make_prompts(wl)).cuda()
    ext_prompts = torch.from_numpy(W.make_prompts(replace(wl, prompt_seed=wl.prompt_seed + 1))).cuda()
    ext_seq, _ = other.rollouts(ext_prompts, N, wl.temperature, wl.rollout_seed + 1000)
    ext_rew = torch.from_numpy(W.make_rewards(S, wl.reward_p, wl.reward_seed + 1)).cuda()
    torch.cuda.synchronize()
    other.close()
    ws = torch.empty(sapo.sapo_trainer_workspace_bytes(node.trainer, (n_own + n_swarm) * G, T) + 256, dtype=torch.uint8,
                     device="cuda")
    setup_s = time.time() - t0
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    rows = []
    for i in range(args.warmup + args.steps):
        own_rew = torch.from_numpy(W.make_rewards(S, wl.reward_p, wl.reward_seed + 10 * i)).cuda()   # the reward model's verdicts
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ev[0].record()
        own_seq, _ = node.rollouts(prompts, N, wl.temperature, wl.rollout_seed + i)
        ev[1].record()
        seqs, rew = node.training_set(own_seq, own_rew, ext_seq, ext_rew, n_own, n_swarm, 77 + i)
        ev[2].record()
        loss = node.update(seqs, rew, N, workspace=ws)
        ev[3].record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t1) * 1e3
        if i >= args.warmup:
            rows.append((wall, ev[0].elapsed_time(ev[1]), ev[1].elapsed_time(ev[2]), ev[2].elapsed_time(ev[3]),
                         int(seqs.shape[0]), float(loss.cpu()[0])))
    med = lambda k: float(np.median([r[k] for r in rows]))
    n_train = int(np.median([r[4] for r in rows]))
    tokens = S * N + n_train * T
    out = {"metric": "tokens/s (generated + trained) of one node-round of Algorithm 1 (%s, 1 GPU)" % wl.name,
           "value": round(tokens / (med(0) * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(med(0), 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": {3: "f32", 2: "bf16x2", 1: "bf16"}[args.pieces] + " update, f16 rollouts and scoring", "data": "synthetic",
           "config": {"workload": wl.name, "layers": shape.n_layers, "d_model": shape.d_model, "vocab": shape.vocab,
                      "prompts": P, "completions_per_prompt": G, "prompt_len": Lp, "new_tokens": N,
                      "own_datapoints": n_own, "swarm_datapoints": n_swarm, "training_sequences": n_train,
                      "update_matmul_pieces": args.pieces, "rewards": "Bernoulli(%.1f) stand-in for the verifier" % wl.reward_p},
           "phases_ms": {"rollouts": round(med(1), 3), "training_set": round(med(2), 3),
                         "scoring + update + new policy in place": round(med(3), 3)},
           "rounds_per_s": round(1e3 / med(0), 3), "losses": [round(r[5], 6) for r in rows],
           "roofline": None, "cpu_baseline": None, "setup_s": round(setup_s, 1)}
    node.close()
    print(json.dumps(out))


def bench_update(args, wl):
    """The local policy update on one training set: trained tokens/s of sapo_policy_update."""
    import torch
    from paper_2509_08721_amd import sapo, workloads as W
    shape = wl.shape
    torch.cuda.set_device(0)
    t0 = time.time()
    weights = W.make_weights(shape, wl.weight_seed)
    S, T, Tm, G = wl.score_seqs, wl.score_len, wl.score_masked, wl.group
    # the training set: Zipf prompts repeated G times + random completions; old log-probs and advantages from
    # the scoring call under the same weights (what a node holds when it reaches the update)
    prompts = W.make_prompts(wl)
    rng = np.random.default_rng([wl.prompt_seed, 7])
    comp = rng.integers(0, shape.vocab, size=(S, T - wl.prompt_len)).astype(np.int32)
    tokens_np = np.concatenate([np.repeat(prompts, G, axis=0), comp], axis=1)
    mask_np = W.make_completion_mask(S, T, Tm)
    tokens, mask = torch.from_numpy(tokens_np).cuda(), torch.from_numpy(mask_np).cuda()
    rewards = torch.from_numpy(W.make_rewards(S, wl.reward_p, wl.reward_seed)).cuda()
    gw = sapo.sapo_weights_create(shape, weights)
    logp_old, adv = sapo.sapo_score_logprobs(gw, tokens, mask, rewards, G)
    torch.cuda.synchronize()
    gw.close()
    tr = sapo.sapo_trainer_create(shape, weights)
    sapo.sapo_trainer_set_matmul_pieces(tr, args.pieces)
    # the whole set at once if its activations fit the free memory, else the largest micro-batch (halving) that does
    s_micro = S
    free_b = torch.cuda.mem_get_info()[0]
    while s_micro > 1 and sapo.sapo_trainer_workspace_bytes_for(tr, S, T, s_micro) > 0.9 * free_b:
        s_micro = (s_micro + 1) // 2
    nbytes = sapo.sapo_trainer_workspace_bytes_for(tr, S, T, s_micro)
    ws = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
    setup_s = time.time() - t0
    losses = []
    for _ in range(args.warmup):
        loss, _ = sapo.sapo_policy_update(tr, tokens, mask, logp_old, adv, want_logp=False, workspace=ws)
        losses.append(loss)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        loss, _ = sapo.sapo_policy_update(tr, tokens, mask, logp_old, adv, want_logp=False, workspace=ws)
        losses.append(loss)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t1) / args.steps
    flops, attn_flops = update_flops(shape, S, T, Tm)
    kernels, roofline = {}, None
    if not args.no_kernel_profile:
        sapo.sapo_profile_start()
        sapo.sapo_policy_update(tr, tokens, mask, logp_old, adv, want_logp=False, workspace=ws)
        prof = sapo.sapo_profile_stop()
        for name, (ms, cnt) in sorted(prof.items(), key=lambda kv: -kv[1][0]):
            kernels[name] = {"launches": cnt, "total_ms": round(ms, 3), "avg_us": round(ms * 1e3 / cnt, 3)}
        if "k_gemm" in kernels:
            # The GEMMs multiply fp32 values as three bf16 pieces each: one algorithmic multiply-add is six bf16
            # MFMA multiply-adds.  `achieved` counts the algorithmic flops (what an fp32 GEMM would count) against
            # the bf16 MFMA peak, the contraction's own type; `executed_*` counts what the matrix cores ran.
            k = kernels["k_gemm"]
            n_products = {3: 6, 2: 3, 1: 1}[args.pieces]
            ach = flops / (k["total_ms"] * 1e-3) / 1e12
            k.update(bound="mfma", work_per_launch=flops / k["launches"], achieved=round(ach, 2), unit="TFLOP/s",
                     frac=round(ach / MFMA_16BIT_PEAK_TFLOPS, 4))
            roofline = {"kernel": "k_gemm_x3 (the projection and LM-head GEMMs of the update)", "bound": "mfma", "achieved": k["achieved"],
                        "peak": MFMA_16BIT_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": k["frac"], "traffic": None,
                        "avg_us": k["avg_us"], "launches": k["launches"], "work_per_launch": k["work_per_launch"],
                        "executed_TFLOPs": round(n_products * ach, 1),
                        "executed_frac": round(n_products * ach / MFMA_16BIT_PEAK_TFLOPS, 4),
                        "vs_fp32_mfma_peak": round(ach / FP32_MFMA_PEAK_TFLOPS, 4)}
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import sapo_update_oracle as U
        ncores = len(os.sched_getaffinity(0))
        big = shape.d_model >= 512
        s_n, t_n = (1, T) if big else (S, T)
        params = U.parameter_list(shape, weights)
        t2 = time.perf_counter()
        U.loss_and_gradients(shape, params, tokens_np[:s_n, :t_n], W.make_completion_mask(s_n, t_n, 2 * t_n // 3),
                             np.full((s_n, t_n), -10.0, dtype=np.float32), np.ones(s_n, dtype=np.float32))
        dtc = time.perf_counter() - t2
        cpu = {"value": round(s_n * t_n / dtc, 2), "unit": "tokens/s", "cores": ncores, "kind": "oracle",
               "sample": "torch fp64 autograd oracle: loss and gradient of %d sequence(s) x %d tokens in %.1f s "
                         "(no optimiser step)" % (s_n, t_n, dtc)}
    out = {"metric": "trained tokens/s of one policy update (forward + clipped surrogate + backward + Adam)",
           "value": round(S * T / dt, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(dt * 1e3, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": {3: "f32", 2: "bf16x2", 1: "bf16"}[args.pieces], "data": "synthetic",
           "config": {"workload": wl.name,
                      "arithmetic": {3: "fp32 (GEMM products as 6 bf16 x bf16 partial products, fp32 accumulation)",
                                     2: "fp32 with GEMM operands of 16 significant bits (2 bf16 pieces, 3 partial products), "
                                        "fp32 accumulation",
                                     1: "fp32 with bf16 GEMM operands (1 piece), fp32 accumulation"}[args.pieces],
                      "layers": shape.n_layers, "d_model": shape.d_model, "vocab": shape.vocab,
                      "seqs": S, "seq_len": T, "masked": Tm, "sequences_per_micro_batch": s_micro,
                      "optimizer": "Adam lr 1e-3 (defaults)",
                      "weights": "fp32 masters of the bf16 model"},
           "update_flops": flops + attn_flops, "achieved_TFLOPs": round((flops + attn_flops) / dt / 1e12, 2),
           "workspace_GB": round(nbytes / 2 ** 30, 2), "loss_first": round(float(losses[0].cpu()[0]), 6),
           "loss_last": round(float(losses[-1].cpu()[0]), 6),
           "roofline": roofline, "cpu_baseline": cpu, "kernels": kernels, "setup_s": round(setup_s, 1)}
    print(json.dumps(out))


def run_workload(args, workload, n_steps, n_warmup, cpu_baseline, probes):
    """Time one workload (rollout and / or scoring) and return its record."""
    import torch
    from paper_2509_08721_amd import sapo, workloads as W

    wl = W.WORKLOADS[workload]
    if args.layers > 0:
        wl = replace(wl, shape=replace(wl.shape, n_layers=args.layers))
    if args.new_tokens > 0:
        wl = replace(wl, n_new=args.new_tokens)
    shape = wl.shape
    torch.cuda.set_device(0)
    t0 = time.time()
    weights = W.make_weights(shape, wl.weight_seed)
    gw = sapo.sapo_weights_create(shape, weights)
    G = wl.group
    do_rollout = wl.n_new > 0 and workload != "halfb_score_mixed"
    do_score = wl.score_seqs > 0
    side = torch.cuda.Stream()      # a non-default stream: the library replays a captured decode step on it
    torch.cuda.synchronize()
    torch.cuda.set_stream(side)

    if do_rollout:
        P, Lp, N = wl.n_prompts, wl.prompt_len, wl.n_new
        S = P * G
        prompts_np = W.make_prompts(wl)
        T, Tm, S_score = (Lp + N, N, S) if do_score else (0, 0, 0)
        seq_src = None
    else:
        # scoring only (Sec. 5's 4 local / 4 external mix): half the groups are rolled out by the local
        # weights, half by an independently seeded copy; this preparation is input generation, untimed
        S_score, T, Tm = wl.score_seqs, wl.score_len, wl.score_masked
        P, Lp, N = S_score // G, T - Tm, Tm
        S = S_score
        prompts_np = W.make_prompts(W.scaled(wl, n_prompts=P, prompt_len=Lp))
        if args.layers > 0:
            # counter run: traffic does not depend on token values, and the preparation rollouts would only add launches
            seq_src = torch.from_numpy(W.make_random_tokens(S_score, T, shape.vocab, wl.rollout_seed)).cuda()
        else:
            other = sapo.sapo_weights_create(shape, W.make_weights(shape, wl.external_weight_seed))
            half = P // 2
            t_loc, _ = sapo.sapo_rollout_generate(gw, torch.from_numpy(prompts_np[:half]).cuda(), G, N, 1.0, wl.rollout_seed)
            t_ext, _ = sapo.sapo_rollout_generate(other, torch.from_numpy(prompts_np[half:]).cuda(), G, N, 1.0,
                                                  wl.rollout_seed + 1)
            torch.cuda.synchronize()
            del other
            seq_src = torch.cat([torch.from_numpy(np.repeat(prompts_np, G, axis=0)).cuda(),
                                 torch.cat([t_loc, t_ext], dim=0)], dim=1).contiguous()
    prompts = torch.from_numpy(prompts_np).cuda()
    plan = {"S": S, "N": N, "Lp": Lp, "P": P, "T": T, "Tm": Tm, "S_score": S_score, "rollout": do_rollout,
            "score": do_score, "fused_lm": S <= 64 and shape.d_model <= 1024,
            "ffn_big": 64 < S <= 256 and bool(gw.uses_mfma)}

    if do_rollout:
        ws_r = torch.empty(sapo.sapo_rollout_workspace_bytes(gw, P, Lp, G, N) + 256, dtype=torch.uint8, device="cuda")
        out_tok = torch.empty((S, N), dtype=torch.int32, device="cuda")
        out_lp = torch.empty((S, N), dtype=torch.float32, device="cuda")
        prompt_rep = prompts.repeat_interleave(G, dim=0)
    if do_score:
        rewards = torch.from_numpy(W.make_rewards(S_score, wl.reward_p, wl.reward_seed)).cuda()
        mask = torch.from_numpy(W.make_completion_mask(S_score, T, Tm)).cuda()
        ws_s = torch.empty(sapo.sapo_score_workspace_bytes(gw, S_score, T) + 256, dtype=torch.uint8, device="cuda")
        sc_lp = torch.empty((S_score, T), dtype=torch.float32, device="cuda")
        sc_adv = torch.empty((S_score,), dtype=torch.float32, device="cuda")
    setup_s = time.time() - t0

    if args.copy_probe and probes:
        a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]

    def step(i):
        ev[0].record()
        if do_rollout:
            sapo.sapo_rollout_generate(gw, prompts, G, N, wl.temperature, wl.rollout_seed + i, workspace=ws_r,
                                       out_tokens=out_tok, out_logprobs=out_lp)
        ev[1].record()
        if do_score:
            seqs = seq_src if seq_src is not None else torch.cat([prompt_rep, out_tok], dim=1).contiguous()
            sapo.sapo_score_logprobs(gw, seqs, mask, rewards, G, workspace=ws_s, out_logprobs=sc_lp,
                                     out_advantages=sc_adv)
        ev[2].record()

    for i in range(n_warmup):
        step(i)
    torch.cuda.synchronize()
    roll_ms, score_ms = [], []
    t_start = time.perf_counter()
    for i in range(n_steps):
        step(100 + i)
        torch.cuda.synchronize()
        roll_ms.append(ev[0].elapsed_time(ev[1]))
        score_ms.append(ev[1].elapsed_time(ev[2]))
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_start) * 1e3 / max(1, n_steps)
    r_ms, s_ms = float(np.median(roll_ms)), float(np.median(score_ms))
    step_ms = r_ms + s_ms

    # sanity: finite outputs; decode with the cache reproduces the teacher-forced log-probs
    lp_gap = None
    if do_score:
        assert torch.isfinite(sc_lp).all()
    if do_rollout and do_score:
        lp_gap = float((sc_lp[:, Lp:] - out_lp).abs().max().item())
        assert lp_gap < 4e-2, lp_gap

    # prefill alone (max_new = 1: the prompts' forward and the first sampled token), for a decode-only rate
    prefill_ms = None
    if do_rollout and N > 1:
        t1 = torch.empty((S, 1), dtype=torch.int32, device="cuda")
        l1 = torch.empty((S, 1), dtype=torch.float32, device="cuda")
        pm = []
        for i in range(3):
            ev[0].record()
            sapo.sapo_rollout_generate(gw, prompts, G, 1, wl.temperature, wl.rollout_seed, workspace=ws_r,
                                       out_tokens=t1, out_logprobs=l1)
            ev[1].record()
            torch.cuda.synchronize()
            pm.append(ev[0].elapsed_time(ev[1]))
        prefill_ms = float(np.median(pm))

    # the update's clipped surrogate on this batch (Sec. 4.2), outside the timed step: a few small kernels
    surrogate = None
    if do_score and probes:
        lp_old = sc_lp + 0.05 * torch.randn_like(sc_lp)
        ws_l = torch.empty(sapo.sapo_surrogate_workspace_bytes() + 256, dtype=torch.uint8, device="cuda")
        lm = []
        for i in range(5):
            ev[0].record()
            sapo.sapo_clipped_surrogate(sc_lp, lp_old, mask, sc_adv, workspace=ws_l)
            ev[1].record()
            torch.cuda.synchronize()
            lm.append(ev[0].elapsed_time(ev[1]))
        l_ms = float(np.median(lm))
        l_bytes = S_score * T * (4 + 4 + 1 + 4 + 1) + S_score * Tm * (4 + 4)   # mask twice, logp pair twice where set, gradient out
        surrogate = {"ms": round(l_ms, 4), "algorithmic_bytes": l_bytes, "GBs": round(l_bytes / (l_ms * 1e-3) / 1e9, 2),
                     "note": "three dependent launches on under 2 MB: launch-latency-bound, not a roofline case"}

    gen_tokens = S * N if do_rollout else 0
    scored_tokens = S_score * T if do_score else 0
    out = {
        "metric": "rollout tokens/s + scored tokens/s (0.5B GQA, 1 GPU)" if shape.d_model == 896 else
                  "rollout tokens/s + scored tokens/s (%s, 1 GPU)" % wl.name,
        "value": round((gen_tokens + scored_tokens) / (step_ms * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": n_steps, "warmup": n_warmup,
        "ms_per_step": round(step_ms, 3), "wall_ms_per_step": round(wall_ms, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if shape.dtype == "f32" else "f16", "data": "synthetic",
        "config": {"workload": wl.name if not (args.layers or args.new_tokens) else wl.name + " (cut down for a counter run: NOT a result)", "layers": shape.n_layers, "d_model": shape.d_model,
                   "heads": "%dq/%dkv x %d" % (shape.n_q_heads, shape.n_kv_heads, shape.head_dim),
                   "d_ff": shape.d_ff, "vocab": shape.vocab,
                   "weights": "fp32" if shape.dtype == "f32" else "bf16 values, MFMA operands in IEEE half, fp32 accumulation",
                   "prompts": P, "completions_per_prompt": G, "prompt_len": Lp, "new_tokens": N,
                   "temperature": wl.temperature, "timed": ("rollout+" if do_rollout else "") + ("score" if do_score else ""),
                   "score_seqs": S_score, "score_len": T, "score_masked": Tm, "mfma_path": bool(gw.uses_mfma)},
    }
    if do_rollout:
        ab = algorithmic_bytes_rollout(shape, P, G, Lp, N)
        bytes_shared = ab["weights"] + ab["kv_read_shared"] + ab["kv_write"]
        bytes_unshared = ab["weights"] + ab["kv_read_unshared"] + ab["kv_write"]
        roll_gbs = bytes_shared / (r_ms * 1e-3) / 1e9
        if prefill_ms is not None and r_ms > prefill_ms:
            out.update({"prefill_ms": round(prefill_ms, 3),
                        "decode_only_tokens_per_s": round(S * (N - 1) / ((r_ms - prefill_ms) * 1e-3), 1)})
        out.update({"rollout_tokens_per_s": round(gen_tokens / (r_ms * 1e-3), 1), "rollout_ms": round(r_ms, 3),
                    "rollout_hbm": {"algorithmic_bytes_shared": bytes_shared, "algorithmic_bytes_unshared": bytes_unshared,
                                    "achieved_GBs": round(roll_gbs, 1), "peak_GBs": HBM_PEAK_GBS,
                                    "frac": round(roll_gbs / HBM_PEAK_GBS, 4)}})
    if do_score:
        fl = algorithmic_flops_score(shape, S_score, T, Tm)
        score_tflops = fl["total"] / (s_ms * 1e-3) / 1e12
        out.update({"scored_tokens_per_s": round(scored_tokens / (s_ms * 1e-3), 1), "score_ms": round(s_ms, 3),
                    "masked_tokens_per_s": round(S_score * Tm / (s_ms * 1e-3), 1),
                    "score_mfma": {"algorithmic_flops": fl["total"], "achieved_TFLOPs": round(score_tflops, 2),
                                   "peak_TFLOPs": MFMA_16BIT_PEAK_TFLOPS,
                                   "frac": round(score_tflops / MFMA_16BIT_PEAK_TFLOPS, 4)}})
    if lp_gap is not None:
        out["rollout_vs_score_logprob_max_abs"] = round(lp_gap, 6)

    # per-kernel durations: one extra step in which every launch carries two HIP events (on the launch
    # stream) that take the kernel's own start and end timestamps
    kernels = {}
    roofline = None
    if not args.no_kernel_profile:
        sapo.sapo_profile_start()
        step(999)
        prof = sapo.sapo_profile_stop()
        for name, (ms, cnt) in sorted(prof.items(), key=lambda kv: -kv[1][0]):
            bound, work = per_launch_work(shape, plan, name, cnt)
            avg_us = ms * 1e3 / cnt
            ent = {"launches": cnt, "total_ms": round(ms, 3), "avg_us": round(avg_us, 3)}
            if bound == "hbm":
                ach = work / (avg_us * 1e-6) / 1e9
                ent.update(bound="hbm", work_per_launch=work, achieved=round(ach, 1), unit="GB/s",
                           frac=round(ach / HBM_PEAK_GBS, 4))
            elif bound == "mfma":
                ach = work / (avg_us * 1e-6) / 1e12
                ent.update(bound="mfma", work_per_launch=work, achieved=round(ach, 2), unit="TFLOP/s",
                           frac=round(ach / MFMA_16BIT_PEAK_TFLOPS, 4))
            kernels[name] = ent
        dom = next((n for n in kernels if "bound" in kernels[n]), None)
        if dom:
            k = kernels[dom]
            from paper_2509_08721_amd import traffic as TR
            cut = bool(args.layers or args.new_tokens)
            roofline = {"kernel": dom, "bound": k["bound"], "achieved": k["achieved"],
                        "peak": HBM_PEAK_GBS if k["bound"] == "hbm" else MFMA_16BIT_PEAK_TFLOPS, "unit": k["unit"],
                        "frac": k["frac"], "traffic": None if cut else TR.lookup(wl.name, dom), "avg_us": k["avg_us"], "launches": k["launches"],
                        "work_per_launch": k["work_per_launch"]}

    # CPU baseline: the oracle as it stands, on a bounded slice of the same workload
    cpu = None
    if cpu_baseline:
        from oracle import sapo_oracle as O
        ncores = len(os.sched_getaffinity(0))
        m = O.Model(shape, weights)
        big = shape.d_model >= 512
        parts, cpu_step_s = [], 0.0
        res = {}
        if do_rollout and big:
            # one group of G sequences, 16 decode steps each at the starting context, timed apart from the prompt's
            # forward: the call is timed whole, the prompt's forward alone is timed again and taken off
            n_n = 16
            t1 = time.perf_counter()
            O.rollout_generate(m, prompts_np[:1], G, n_n + 1, wl.temperature, wl.rollout_seed)
            dt_all = time.perf_counter() - t1
            t1 = time.perf_counter()
            O.hidden_states(m, prompts_np[0], [[None, None] for _ in range(m.n_layers)])
            dt_prompt = time.perf_counter() - t1
            dec_rate = G * n_n / max(dt_all - dt_prompt, 1e-9)
            res["decode_tokens_per_s"] = round(dec_rate, 3)
            res["prompt_forward_s"] = round(dt_prompt, 3)
            cpu_roll_s = P * dt_prompt + gen_tokens / dec_rate          # every prompt once, every token one decode step
            res["rollout_tokens_per_s"] = round(gen_tokens / cpu_roll_s, 3)
            cpu_step_s += cpu_roll_s
            parts.append("decode of one group of %d sequences x %d steps after a %d-token prompt in %.1f s "
                         "(+ %.1f s for the prompt's forward, timed apart)" % (G, n_n, Lp, dt_all - dt_prompt, dt_prompt))
        elif do_rollout:
            t1 = time.perf_counter()
            O.rollout_generate(m, prompts_np, G, N, wl.temperature, wl.rollout_seed)
            dt = time.perf_counter() - t1
            res["rollout_tokens_per_s"] = round(gen_tokens / dt, 3)
            cpu_step_s += dt
            parts.append("the whole rollout call in %.1f s" % dt)
        if do_score:
            s_n = 2 if big else S_score
            seq_np = (seq_src if seq_src is not None else torch.cat([prompt_rep, out_tok], dim=1))[:s_n].cpu().numpy()
            t1 = time.perf_counter()
            O.score_logprobs(m, seq_np, W.make_completion_mask(s_n, T, Tm))
            dt = time.perf_counter() - t1
            res["scored_tokens_per_s"] = round(s_n * T / dt, 2)
            cpu_step_s += scored_tokens / (s_n * T / dt)
            parts.append("scoring of %d sequence(s) x %d tokens in %.1f s" % (s_n, T, dt))
        cpu = {"value": round((gen_tokens + scored_tokens) / cpu_step_s, 2), "unit": "tokens/s", "cores": ncores,
               "kind": "oracle",
               "sample": "numpy fp64 oracle: " + ", ".join(parts) + "; whole-step rate extrapolated from the slice rates"}
        cpu.update(res)

    # context for the HBM fractions: what a kernel that only reads reaches on this machine (not a denominator)
    read_probe = None
    if probes and not (args.layers or args.new_tokens):
        read_probe = {"GBs": round(sapo.sapo_debug_read_probe(), 1), "bytes": 1 << 31,
                      "note": "streaming read of 2 GiB, 16-byte non-temporal loads; the roofline fractions use the published 8000 GB/s"}
    # context for the MFMA fractions: what a kernel that only issues MFMAs on registers sustains (not a denominator)
    mfma_probe = None
    if probes and not (args.layers or args.new_tokens):
        tf = sapo.sapo_debug_mfma_probe()
        mfma_probe = {"TFLOPs": round(tf, 1), "frac_of_peak": round(tf / MFMA_16BIT_PEAK_TFLOPS, 3),
                      "note": "32x32x16 half MFMAs on registers only, two waves per SIMD, N(0,1) operands; the roofline "
                              "fractions use the published 2500 TFLOP/s"}
    props = torch.cuda.get_device_properties(0)
    device = {"name": props.name, "memory_GB": round(props.total_memory / 2 ** 30), **sapo.sapo_device_info()}
    out.update({"roofline": roofline, "cpu_baseline": cpu, "kernels": kernels, "surrogate_loss": surrogate,
                "hbm_read_probe": read_probe, "mfma_probe": mfma_probe, "device": device, "setup_s": round(setup_s, 1)})
    gw.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="halfb_rollout")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-profile", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="default workload only: do not also time the long-generation, mixed-scoring and 1.5B-class workloads")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 1 GiB device copy (a kernel of known traffic, for scaling profiler byte counters)")
    ap.add_argument("--layers", type=int, default=0,
                    help="counter runs only: same kernels and shapes with this many layers (fewer launches); "
                         "the printed line is then not a benchmark result")
    ap.add_argument("--new-tokens", type=int, default=0, help="counter runs only: generate this many tokens")
    ap.add_argument("--pieces", type=int, default=3, choices=(1, 2, 3),
                    help="*_update workloads only: 3 = fp32-accurate matrix products (default), 2 = operands of 16 "
                         "significant bits, 1 = bf16 operands")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on ONE GPU (no sharding, no collectives); --gpus %d is not "
              "supported. Sequences are independent, so N GPUs would each take P/N prompts." % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2509_08721_amd import sapo, workloads as W

    wl = W.WORKLOADS[args.workload]
    if args.workload.endswith("_update"):
        return bench_update(args, wl)
    if wl.stop_token >= 0:
        return bench_stop(args, wl)
    if args.workload.endswith("_round"):
        return bench_round(args, wl)
    out = run_workload(args, args.workload, args.steps, args.warmup, cpu_baseline=not args.no_cpu_baseline,
                       probes=True)
    default_run = args.workload == "halfb_rollout" and not (args.layers or args.new_tokens or args.no_other_configs)
    if default_run:
        # the other full-size configurations, a few steps each, in the same line: the long-generation rollout, the
        # swarm-mixed scoring batch the scoring target is stated on, and the 1.5B-class decoder
        other = {}
        for name in ("halfb_long", "halfb_score_mixed", "onehalfb"):
            r = run_workload(args, name, 3, 1, cpu_baseline=False, probes=False)
            keep = {k: r[k] for k in ("value", "ms_per_step", "rollout_tokens_per_s", "rollout_ms", "decode_only_tokens_per_s",
                                      "rollout_hbm", "scored_tokens_per_s", "score_ms", "score_mfma", "roofline",
                                      "rollout_vs_score_logprob_max_abs") if k in r}
            keep["steps"], keep["warmup"] = 3, 1
            keep["config"] = {k: r["config"][k] for k in ("workload", "prompts", "completions_per_prompt", "prompt_len",
                                                          "new_tokens", "temperature", "timed", "score_seqs", "score_len",
                                                          "score_masked")}
            keep["kernels"] = {k: {f: v[f] for f in ("launches", "avg_us", "frac") if f in v} for k, v in r["kernels"].items()
                               if "frac" in v}
            other[name] = keep
        out["other_configs"] = other
    print(json.dumps(out))



if __name__ == "__main__":
    main()
