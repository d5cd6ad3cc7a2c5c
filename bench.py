#!/usr/bin/env python3
"""Benchmark of the RPO suffix-rollout hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C1]

One "step" is one pass of the whole path over one synthetic batch: cut + pack,
shared-prefix prefill, KV fork, the sample / decode loop, teacher-forced suffix
log-probs and group advantages.  Prints ONE JSON line (rank 0 is the only rank:
this build runs on a single GPU).
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

PEAK = {"hbm": (8000.0, "GB/s"), "mfma": (2500.0, "TFLOP/s")}
KERNEL_BOUND = {"gemm256": "mfma", "gemm256x128": "mfma", "gemm128": "mfma", "gemm64": "mfma",
                "attn_decode": "hbm", "sample": "hbm"}


def build_case(workload: str, n_groups: int | None, max_rows: int):
    import torch
    from paper_2601_19404_amd import binding as rpo
    from paper_2601_19404_amd import rollout, synth
    cfg = synth.CONFIGS[workload]
    mc = cfg.model
    w = synth.make_weights(mc, seed=1234, device="cuda")
    model = rpo.rpo_model_create(mc, w)
    wl = synth.make_workload(cfg, n_groups=n_groups)
    order = rollout.order_by_suffix_length(wl.m)
    prompts = [wl.prompts[i] for i in order]
    cached = [wl.cached[i] for i in order]
    m = wl.m[order]
    rewards = wl.rewards[order]
    ng, G = len(prompts), cfg.G
    max_prefix = cfg.prompt_len + cfg.traj_len - int(m.min())
    max_suffix = int(m.max())
    max_rows = max(max_rows, max_prefix, ng * G, max_suffix)
    page = 64 if mc.dtype == "bf16" else 16
    batch = rpo.rpo_batch_create(model, ng, G, max_prefix, max_suffix, page, max_rows)
    seq_ids = (torch.arange(ng * G, dtype=torch.int64)).cuda()
    idx, cu_s = rollout.suffix_index(m, G, max_suffix)
    state = dict(cfg=cfg, model=model, batch=batch, prompts=prompts, cached=cached, m=m, G=G, ng=ng,
                 rewards_dev=torch.from_numpy(rewards).cuda(), seq_ids=seq_ids,
                 idx_dev=torch.from_numpy(idx).cuda(), cu_s=cu_s,
                 lp_out=torch.empty(max(int(cu_s[-1]), 1), dtype=torch.float32, device="cuda"),
                 adv_out=torch.empty(ng, G, dtype=torch.float32, device="cuda"), weights=w,
                 page=page, max_prefix=max_prefix, max_suffix=max_suffix)
    return state


def one_step(st, seed: int):
    from paper_2601_19404_amd import binding as rpo
    from paper_2601_19404_amd import rollout
    res = rollout.suffix_rollout(st["batch"], st["prompts"], st["cached"], st["m"], st["cfg"].temperature,
                                 seed, st["seq_ids"])
    packed, cu_s = rollout.pack_suffixes(res.tokens, st["m"], st["G"], st["idx_dev"])
    rpo.rpo_suffix_logprobs(st["batch"], packed, cu_s, st["cfg"].temperature, st["lp_out"])
    rpo.grpo_advantages(st["rewards_dev"], st["ng"], st["G"], 0, 0.0, st["adv_out"])
    return res


def cpu_baseline(st, budget_tokens: int = 6, prefix_cap: int = 256, n_rollouts: int = 3):
    """The fp64 oracle on the host cores, on a bounded slice of the same workload: group 0,
    its prefix cut to the last `prefix_cap` tokens, `n_rollouts` rollouts, `budget_tokens`
    regenerated tokens each."""
    import torch
    from oracle import rollout as orollout
    from oracle import transformer as T
    from paper_2601_19404_amd import synth
    mc = st["cfg"].model
    w_np = synth.weights_to_numpy(st["weights"])
    shape = T.Shape(mc.n_layers, mc.d_model, mc.n_q_heads, mc.n_kv_heads, mc.head_dim, mc.d_ffn,
                    mc.vocab, mc.rope_base, mc.rms_eps)
    prompt = np.asarray(st["prompts"][0])
    cached = np.asarray(st["cached"][0])
    mk = int(st["m"][0])
    keep = len(cached) - mk
    if len(prompt) + keep > prefix_cap:          # bounded sample: keep the tail of the prefix
        drop = len(prompt) + keep - prefix_cap
        cached_s = cached[drop:] if drop <= keep else cached
        prompt_s = prompt if drop <= keep else prompt[:1]
    else:
        cached_s, prompt_s = cached, prompt
    n_tok = min(budget_tokens, mk)
    t0 = time.perf_counter()
    out = orollout.suffix_rollout(shape, w_np, prompt_s, cached_s, mk, n_rollouts, st["cfg"].temperature,
                                  3, np.arange(n_rollouts), n_tokens=n_tok)
    dt = time.perf_counter() - t0
    gen = n_rollouts * n_tok
    return dict(value=gen / dt, unit="tokens/s", cores=int(torch.get_num_threads()), kind="oracle",
                sample=(f"group 0 of {st['cfg'].name}, prefix cut to its last {len(out['prefix'])} tokens, "
                        f"{n_rollouts} rollouts x {n_tok} regenerated tokens, {dt:.1f} s of fp64 numpy"),
                seconds=dt)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="C1", choices=["C0", "C1", "C2", "C3"])
    ap.add_argument("--groups", type=int, default=None, help="override the number of groups (debugging)")
    ap.add_argument("--max-rows", type=int, default=16384)
    ap.add_argument("--profile-kernel", default="gemm256",
                    help="kernel whose launches are timed with HIP events for the roofline object")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2601_19404_amd import binding as rpo
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    rpo.lib()
    st = build_case(args.workload, args.groups, args.max_rows)
    cfg = st["cfg"]
    for i in range(args.warmup):
        one_step(st, seed=100 + i)
    torch.cuda.synchronize()

    kid = rpo.KERNEL_IDS[args.profile_kernel]
    rpo.rpo_profile_start(kid)
    t0 = time.perf_counter()
    for i in range(args.steps):
        res = one_step(st, seed=200 + i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    launches, k_ms, k_flops, k_bytes = rpo.rpo_profile_stop()

    n_gen = res.n_generated
    value = n_gen * args.steps / dt
    bound = KERNEL_BOUND.get(args.profile_kernel, "hbm")
    peak, unit = PEAK[bound]
    if launches and k_ms > 0:
        work = k_flops / 1e12 if bound == "mfma" else k_bytes / 1e9
        achieved = work / (k_ms / 1e3)
    else:
        achieved = 0.0
    roofline = dict(bound=bound, achieved=achieved, peak=peak, unit=unit, frac=achieved / peak, traffic=None,
                    kernel=args.profile_kernel, launches=launches,
                    avg_launch_us=(k_ms * 1e3 / launches) if launches else None,
                    share_of_step_time=(k_ms / 1e3) / dt)
    out = dict(metric="suffix-rollout tokens/sec at 1.5B shape; decode HBM GB/s vs peak",
               value=value, unit="tokens/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=dt * 1e3 / args.steps, higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype=cfg.model.dtype, data="synthetic",
               config=dict(workload=cfg.name, model_shape=cfg.model.name, n_groups=st["ng"], G=st["G"],
                           prompt_len=cfg.prompt_len, traj_len=cfg.traj_len,
                           suffix_len_range=[int(st["m"].min()), int(st["m"].max())],
                           generated_tokens_per_step=int(n_gen), page_tokens=st["page"],
                           temperature=cfg.temperature),
               roofline=roofline)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(st)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
