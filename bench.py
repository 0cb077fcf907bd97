#!/usr/bin/env python3
"""Benchmark of the SAPO node hot path on one MI355X.

One step = one pass of the whole path over one batch: rollout generation
(sapo_rollout_generate: prefill of the unique prompts, then autoregressive decode of all
completions) followed by the scoring pass over the generated batch (sapo_score_logprobs:
teacher-forced log-probs on the completion positions + group-relative advantages).
The default workload is one node-round of the paper's experiment (8 questions x 8
completions, Sec. 4.1 / Sec. 5) on the 0.5B-class decoder with synthetic weights and prompts.

Prints ONE JSON line (see README / DESIGN for the fields).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published


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


def per_launch_work(shape, wl, kernel, launches):
    """Algorithmic bytes (HBM-bound kernels) or flops (MFMA-bound kernels) one launch of a kernel
    processes on this workload, averaged over the launches of one step."""
    S, N, Lp, P = wl.n_seqs, wl.n_new, wl.prompt_len, wl.n_prompts
    L, d, V = shape.n_layers, shape.d_model, shape.vocab
    T, Tm = wl.score_len, wl.score_masked
    if kernel == "k_gemm_skinny":       # the four projection GEMMs of a decode layer
        return "hbm", 2.0 * shape.matmul_params_per_layer() * L * (N - 1) / launches
    if kernel == "k_lmhead_sample":     # LM head of one decode step: the whole [V, d] matrix
        return "hbm", 2.0 * V * d
    if kernel == "k_decode_attention":  # K and V of every cached token of every sequence, one layer
        kv_layer = 2 * shape.kv_dim * 2
        tot = kv_layer * S * sum(Lp + t for t in range(1, N)) * L
        return "hbm", tot / launches
    if kernel == "k_gemm_big":          # projection GEMMs of prefill + scoring
        fl = 2.0 * L * shape.matmul_params_per_layer() * (P * Lp + S * T)
        return "mfma", fl / launches
    if kernel == "k_lmhead_score":
        return "mfma", 2.0 * V * d * S * Tm / launches
    if kernel in ("k_attention", "k_flash_attention"):
        fl = 2.0 * shape.q_dim * L * (S * T * T + P * Lp * Lp)
        return "mfma", fl / launches
    return None, 0.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="halfb_rollout")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-profile", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus %d is not "
              "supported. Sequences are independent, so N GPUs would each take P/N prompts." % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2509_08721_amd import sapo, workloads as W

    wl = W.WORKLOADS[args.workload]
    shape = wl.shape
    torch.cuda.set_device(0)
    t0 = time.time()
    weights = W.make_weights(shape, wl.weight_seed)
    gw = sapo.sapo_weights_create(shape, weights)
    prompts_np = W.make_prompts(wl)
    prompts = torch.from_numpy(prompts_np).cuda()
    S, N, Lp, G, P = wl.n_seqs, wl.n_new, wl.prompt_len, wl.group, wl.n_prompts
    T, Tm = Lp + N, N
    rewards = torch.from_numpy(W.make_rewards(S, wl.reward_p, wl.reward_seed)).cuda()
    mask = torch.from_numpy(W.make_completion_mask(S, T, Tm)).cuda()
    ws_r = torch.empty(sapo.sapo_rollout_workspace_bytes(gw, P, Lp, G, N) + 256, dtype=torch.uint8, device="cuda")
    ws_s = torch.empty(sapo.sapo_score_workspace_bytes(gw, S, T) + 256, dtype=torch.uint8, device="cuda")
    out_tok = torch.empty((S, N), dtype=torch.int32, device="cuda")
    out_lp = torch.empty((S, N), dtype=torch.float32, device="cuda")
    sc_lp = torch.empty((S, T), dtype=torch.float32, device="cuda")
    sc_adv = torch.empty((S,), dtype=torch.float32, device="cuda")
    prompt_rep = prompts.repeat_interleave(G, dim=0)
    setup_s = time.time() - t0

    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    side = torch.cuda.Stream()      # a non-default stream: the library replays a captured decode step on it
    torch.cuda.synchronize()
    torch.cuda.set_stream(side)

    def step(i):
        ev[0].record()
        sapo.sapo_rollout_generate(gw, prompts, G, N, wl.temperature, wl.rollout_seed + i, workspace=ws_r,
                                   out_tokens=out_tok, out_logprobs=out_lp)
        ev[1].record()
        seqs = torch.cat([prompt_rep, out_tok], dim=1).contiguous()
        sapo.sapo_score_logprobs(gw, seqs, mask, rewards, G, workspace=ws_s, out_logprobs=sc_lp,
                                 out_advantages=sc_adv)
        ev[2].record()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    roll_ms, score_ms = [], []
    t_start = time.perf_counter()
    for i in range(args.steps):
        step(100 + i)
        torch.cuda.synchronize()
        roll_ms.append(ev[0].elapsed_time(ev[1]))
        score_ms.append(ev[1].elapsed_time(ev[2]))
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_start) * 1e3 / max(1, args.steps)
    r_ms, s_ms = float(np.median(roll_ms)), float(np.median(score_ms))

    # sanity: the path produced finite log-probs and self-consistent outputs
    lp_gap = float((sc_lp[:, Lp:] - out_lp).abs().max().item())
    assert torch.isfinite(sc_lp).all() and lp_gap < 5e-2, lp_gap

    gen_tokens, scored_tokens = S * N, S * T
    ab = algorithmic_bytes_rollout(shape, P, G, Lp, N)
    bytes_shared = ab["weights"] + ab["kv_read_shared"] + ab["kv_write"]
    bytes_unshared = ab["weights"] + ab["kv_read_unshared"] + ab["kv_write"]
    fl = algorithmic_flops_score(shape, S, T, Tm)
    roll_gbs = bytes_shared / (r_ms * 1e-3) / 1e9
    score_tflops = fl["total"] / (s_ms * 1e-3) / 1e12

    # per-kernel durations with HIP events (one extra, untimed-for-throughput step)
    kernels = {}
    roofline = None
    if not args.no_kernel_profile:
        # every launch carries two HIP events (on the launch stream) that take the kernel's own
        # start and end timestamps
        sapo.sapo_profile_start()
        step(999)
        prof = sapo.sapo_profile_stop()
        for name, (ms, cnt) in sorted(prof.items(), key=lambda kv: -kv[1][0]):
            bound, work = per_launch_work(shape, wl, name, cnt)
            avg_us = ms * 1e3 / cnt
            ent = {"launches": cnt, "total_ms": round(ms, 3), "avg_us": round(avg_us, 3)}
            if bound == "hbm":
                ach = work / (avg_us * 1e-6) / 1e9
                ent.update(bound="hbm", work_per_launch=work, achieved=round(ach, 1), unit="GB/s",
                           frac=round(ach / HBM_PEAK_GBS, 4))
            elif bound == "mfma":
                ach = work / (avg_us * 1e-6) / 1e12
                ent.update(bound="mfma", work_per_launch=work, achieved=round(ach, 2), unit="TFLOP/s",
                           frac=round(ach / MFMA_BF16_PEAK_TFLOPS, 4))
            kernels[name] = ent
        dom = next((n for n in kernels if "bound" in kernels[n]), None)
        if dom:
            k = kernels[dom]
            roofline = {"kernel": dom, "bound": k["bound"], "achieved": k["achieved"],
                        "peak": HBM_PEAK_GBS if k["bound"] == "hbm" else MFMA_BF16_PEAK_TFLOPS, "unit": k["unit"],
                        "frac": k["frac"], "traffic": None, "avg_us": k["avg_us"], "launches": k["launches"],
                        "work_per_launch": k["work_per_launch"]}

    # CPU baseline: the oracle as it stands, on a bounded slice of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import sapo_oracle as O
        ncores = len(os.sched_getaffinity(0))
        m = O.Model(shape, weights)
        big = shape.d_model >= 512
        p_n, g_n, n_n = (1, 2, 6) if big else (P, G, N)
        s_n = 1 if big else S
        t1 = time.perf_counter()
        O.rollout_generate(m, prompts_np[:p_n], g_n, n_n, wl.temperature, wl.rollout_seed)
        t2 = time.perf_counter()
        seq_np = np.concatenate([np.repeat(prompts_np, G, axis=0), out_tok.cpu().numpy()], axis=1)[:s_n]
        O.score_logprobs(m, seq_np, W.make_completion_mask(s_n, T, Tm))
        t3 = time.perf_counter()
        cpu_roll = p_n * g_n * n_n / (t2 - t1)
        cpu_score = s_n * T / (t3 - t2)
        cpu_step_s = gen_tokens / cpu_roll + scored_tokens / cpu_score
        cpu = {"value": round((gen_tokens + scored_tokens) / cpu_step_s, 2), "unit": "tokens/s", "cores": ncores,
               "kind": "oracle",
               "sample": "numpy fp64 oracle: rollout of %d prompt(s) x %d completions x %d new tokens (prompt %d) in "
                         "%.1f s, scoring of %d sequence(s) x %d tokens in %.1f s; whole-step rate extrapolated from "
                         "the two slice rates" % (p_n, g_n, n_n, Lp, t2 - t1, s_n, T, t3 - t2),
               "rollout_tokens_per_s": round(cpu_roll, 3), "scored_tokens_per_s": round(cpu_score, 2)}

    step_ms = r_ms + s_ms
    out = {
        "metric": "rollout tokens/s + scored tokens/s (0.5B GQA, 1 GPU)" if "halfb" in wl.name else
                  "rollout tokens/s + scored tokens/s (%s, 1 GPU)" % wl.name,
        "value": round((gen_tokens + scored_tokens) / (step_ms * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(step_ms, 3), "wall_ms_per_step": round(wall_ms, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if shape.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "layers": shape.n_layers, "d_model": shape.d_model,
                   "heads": "%dq/%dkv x %d" % (shape.n_q_heads, shape.n_kv_heads, shape.head_dim),
                   "d_ff": shape.d_ff, "vocab": shape.vocab, "prompts": P, "completions_per_prompt": G,
                   "prompt_len": Lp, "new_tokens": N, "temperature": wl.temperature,
                   "score_seqs": S, "score_len": T, "score_masked": Tm, "mfma_path": bool(gw.uses_mfma)},
        "rollout_tokens_per_s": round(gen_tokens / (r_ms * 1e-3), 1), "rollout_ms": round(r_ms, 3),
        "scored_tokens_per_s": round(scored_tokens / (s_ms * 1e-3), 1), "score_ms": round(s_ms, 3),
        "rollout_hbm": {"algorithmic_bytes_shared": bytes_shared, "algorithmic_bytes_unshared": bytes_unshared,
                        "achieved_GBs": round(roll_gbs, 1), "peak_GBs": HBM_PEAK_GBS,
                        "frac": round(roll_gbs / HBM_PEAK_GBS, 4)},
        "score_mfma": {"algorithmic_flops": fl["total"], "achieved_TFLOPs": round(score_tflops, 2),
                       "peak_TFLOPs": MFMA_BF16_PEAK_TFLOPS, "frac": round(score_tflops / MFMA_BF16_PEAK_TFLOPS, 4)},
        "rollout_vs_score_logprob_max_abs": round(lp_gap, 6),
        "roofline": roofline, "cpu_baseline": cpu, "kernels": kernels,
        "setup_s": round(setup_s, 1),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
