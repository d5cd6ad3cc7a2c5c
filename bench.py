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

PEAK = {"hbm": (8000.0, "GB/s"), "mfma": (2500.0, "TFLOP/s"), "alu": (157.3, "TFLOP/s")}
HBM_BPS, MFMA_FLOPS = 8.0e12, 2.5e15
# HBM-side bytes of ONE launch of the dominant kernel (the gate/up projection of a full prefill chunk),
# quoted from rocprofv3 --pmc runs of that launch alone (FETCH_SIZE, WRITE_SIZE scaled by what the
# same counters read for a plain copy of known size): a stored figure, not something this run
# measures -- the counters cannot be read from inside the timed run.  Source and command:
# profiles/gemm_hbm_traffic_pmc.txt.
DOMINANT_TRAFFIC = dict(launch="gate/up projection of a full chunk, M=32768 N=17920 K=1536, SwiGLU epilogue",
                        read_bytes=2680.2e6, write_bytes=587.6e6, algorithmic_bytes=155.7e6 + 587.2e6,
                        source="profiles/gemm_hbm_traffic_pmc.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)")
KERNEL_BOUND = {"gemm256": "mfma", "gemm256_swiglu": "mfma", "gemm256x192": "mfma", "gemm256x160": "mfma",
                "gemm128": "mfma", "gemm64": "mfma", "gemm32": "mfma", "gemm64x64": "mfma",
                "gemm_generic": "alu", "attn_chunk": "mfma", "attn_decode": "hbm", "sample": "hbm"}


def _model_sizes(mc):
    es = 2 if mc.dtype == "bf16" else 4
    proj = dict(qkv=mc.qkv_rows * mc.d_model, o=mc.d_model * mc.n_q_heads * mc.head_dim,
                gate_up=2 * mc.d_ffn * mc.d_model, down=mc.d_model * mc.d_ffn)
    io = dict(qkv=(mc.d_model, mc.qkv_rows), o=(mc.n_q_heads * mc.head_dim, mc.d_model),
              gate_up=(mc.d_model, mc.d_ffn), down=(mc.d_ffn, mc.d_model))
    return es, proj, io


def step_roofline(st) -> dict:
    """Lower bound of one pass at the published peaks: the sum over kernel classes k of
    max(algorithmic bytes_k / 8 TB/s, algorithmic flops_k / 2.5 PFLOP/s), per phase (ms)."""
    cfg, mc, m, G = st["cfg"], st["cfg"].model, st["m"], st["G"]
    es, proj, io = _model_sizes(mc)
    L, V, d, dh, Hq = mc.n_layers, mc.vocab, mc.d_model, mc.head_dim, mc.n_q_heads
    kv_tok = 2 * mc.n_kv_heads * dh * es                      # one layer

    def gemm_t(rows, params, k_in, n_out, out_es=None):
        byt = params * es + rows * (k_in * es + n_out * (es if out_es is None else out_es))
        return max(byt / HBM_BPS, 2.0 * rows * params / MFMA_FLOPS)

    def layers_t(rows):
        return L * sum(gemm_t(rows, proj[k], *io[k]) for k in proj)

    S = np.asarray([cfg.prompt_len + cfg.traj_len - int(mk) for mk in m], np.float64)
    # prefill: projections on every prefix row, causal attention, LM head on the last row of each group
    pre = layers_t(float(S.sum()))
    attn_fl = 4.0 * dh * Hq * L * float((S * (S + 1) / 2).sum())
    attn_by = L * float(S.sum()) * (kv_tok + 2 * Hq * dh * es)
    pre += max(attn_fl / MFMA_FLOPS, attn_by / HBM_BPS) + gemm_t(len(m), V * d, d, V, 4)
    # decode: per step the projections on the live rows, the shared-prefix attention, LM head, sampler
    dec = 0.0
    for j in range(1, int(m.max())):
        live = m > j
        n = int(live.sum()) * G
        if n == 0:
            break
        dec += layers_t(n) + gemm_t(n, V * d, d, V, 4)
        a_by = L * kv_tok * (float(S[live].sum()) + n * (j + 1))
        a_fl = 4.0 * dh * Hq * L * G * float((S[live] + j + 1).sum())
        dec += max(a_by / HBM_BPS, a_fl / MFMA_FLOPS) + n * V * 4 / HBM_BPS
    # first draw of every rollout reads the group's prefill logits row
    dec += len(m) * G * V * 4 / HBM_BPS
    # log-prob pass: rows 0..m-2 of every suffix through the layers, LM head on m rows per rollout
    fr = np.maximum(m.astype(np.float64) - 1, 0)
    lp = layers_t(float(fr.sum()) * G)
    lp_fl = 4.0 * dh * Hq * L * G * float((fr * S + fr * (fr + 1) / 2).sum())
    lp += lp_fl / MFMA_FLOPS + gemm_t(float(m.sum()) * G, V * d, d, 0)
    return {"prefill+fork": pre * 1e3, "decode": dec * 1e3, "logprobs+advantages": lp * 1e3,
            "total": (pre + dec + lp) * 1e3}


def algorithmic_decode_bytes(st) -> float:
    """HBM bytes the decode loop must move: per step the layer and
    LM-head weights once, the shared prefix KV once per live GROUP, each live rollout's private
    KV, the new token's KV write, and the logits written by the LM head and read by the sampler."""
    cfg = st["cfg"]
    mc = cfg.model
    es = 2 if mc.dtype == "bf16" else 4
    per_layer = (mc.qkv_rows * mc.d_model + mc.d_model * mc.n_q_heads * mc.head_dim +
                 2 * mc.d_ffn * mc.d_model + mc.d_model * mc.d_ffn)
    w_bytes = (per_layer * mc.n_layers + mc.vocab * mc.d_model) * es
    kv_tok = 2 * mc.n_kv_heads * mc.head_dim * es * mc.n_layers
    m, G = st["m"], st["G"]
    total = 0.0
    for j in range(1, int(m.max())):
        live = m > j
        n_live = int(live.sum())
        if n_live == 0:
            break
        prefix = sum(cfg.prompt_len + cfg.traj_len - int(mk) for mk in m[live])
        total += w_bytes + prefix * kv_tok + n_live * G * (j + 1) * kv_tok + n_live * G * mc.vocab * 4 * 2
    return total


def build_case(workload: str, n_groups: int | None, max_rows: int, G: int | None = None,
               temperature: float | None = None, trunc_max: int | None = None, epochs: int = 0):
    import dataclasses
    import torch
    from paper_2601_19404_amd import binding as rpo
    from paper_2601_19404_amd import rollout, synth
    cfg = synth.CONFIGS[workload]
    # the paper's own sampling settings (Sec. 4.1, Fig. 3): G in {6, 8, 16}, temperature 0.7,
    # m ~ U{0..L} with L in {300, 500, 800}
    if G is not None:
        cfg = dataclasses.replace(cfg, G=G)
    if temperature is not None:
        cfg = dataclasses.replace(cfg, temperature=temperature)
    if trunc_max is not None:
        cfg = dataclasses.replace(cfg, m_lo=0, m_hi=trunc_max)
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
    max_suffix = max(int(m.max()), 1)
    if epochs:      # every epoch draws its own cuts: size the batch for the whole range
        max_prefix = cfg.prompt_len + cfg.traj_len - cfg.m_lo
        max_suffix = max(cfg.m_hi, 1)
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
    if epochs:
        from paper_2601_19404_amd import cache
        state["pool"] = cache.DeviceCachePool(wl.prompts, wl.cached)
    return state


def one_step(st, seed: int, marks=None):
    import torch
    from paper_2601_19404_amd import binding as rpo
    from paper_2601_19404_amd import rollout
    res = rollout.suffix_rollout(st["batch"], st["prompts"], st["cached"], st["m"], st["cfg"].temperature,
                                 seed, st["seq_ids"], marks=marks)
    packed, cu_s = rollout.pack_suffixes(res.tokens, st["m"], st["G"], st["idx_dev"])
    rpo.rpo_suffix_logprobs(st["batch"], packed, cu_s, st["cfg"].temperature, st["lp_out"])
    rpo.grpo_advantages(st["rewards_dev"], st["ng"], st["G"], 0, 0.0, st["adv_out"])
    if marks is not None:
        ev = torch.cuda.Event(enable_timing=True)
        ev.record()
        marks.append(("logprobs+advantages", ev, time.perf_counter()))
    return res


def one_epoch_step(st, seed: int, epoch: int):
    """One pass of Algorithm 1's inner loop with the experience cache on the device: draw the cuts,
    cut + pack from the pool, rollout, suffix log-probs, advantages, epsilon-greedy cache update
    (Sec. 3.3).  The next epoch conditions on what this one wrote.  Returns tokens generated."""
    import torch
    from paper_2601_19404_amd import binding as rpo
    from paper_2601_19404_amd import rollout
    cfg, ng, G = st["cfg"], st["ng"], st["G"]
    rng = np.random.Generator(np.random.PCG64(7000 + epoch))
    m_q = rng.integers(cfg.m_lo, cfg.m_hi + 1, size=ng, dtype=np.int32)
    order = rollout.order_by_suffix_length(m_q)
    m = m_q[order]
    toks, cu = st["pool"].cut_pack(m, order)
    res = rollout.suffix_rollout(st["batch"], None, None, m, cfg.temperature, seed, st["seq_ids"], prefix=(toks, cu))
    packed, cu_s = rollout.pack_suffixes(res.tokens, m, G)
    rpo.rpo_suffix_logprobs(st["batch"], packed, cu_s, cfg.temperature, st["lp_out"][:max(int(cu_s[-1]), 1)])
    rewards = torch.from_numpy((rng.random((ng, G)) < cfg.reward_p).astype(np.float32)).cuda()
    rpo.grpo_advantages(rewards, ng, G, 0, 0.0, st["adv_out"])
    st["pool"].update(m, order, res.tokens, rewards, rng.random(ng).astype(np.float32),
                      rng.integers(0, G, size=ng), 0.1)
    return res.n_generated


def run_epochs(args):
    """--epochs N: N consecutive passes per step, each reading the cache the previous one updated."""
    import torch
    st = build_case(args.workload, args.groups, args.max_rows, args.G, args.temperature, args.trunc_max,
                    epochs=args.epochs)
    cfg = st["cfg"]
    st["lp_out"] = torch.empty(st["ng"] * st["G"] * st["max_suffix"], dtype=torch.float32, device="cuda")
    before = st["pool"].answers.clone()
    for i in range(args.warmup):
        one_epoch_step(st, 100 + i, i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n_gen = 0
    for i in range(args.steps):
        for e in range(args.epochs):
            n_gen += one_epoch_step(st, 200 + i * args.epochs + e, args.warmup + i * args.epochs + e)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    changed = float((st["pool"].answers != before).float().mean().item())
    out = dict(metric="suffix-rollout tokens/sec at 1.5B shape; decode HBM GB/s vs peak", value=n_gen / dt,
               unit="tokens/s", n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=dt * 1e3 / args.steps,
               higher_is_better=True, scaling="weak", vs_baseline=None, dtype=cfg.model.dtype, data="synthetic",
               config=dict(workload=cfg.name, model_shape=cfg.model.name, n_groups=st["ng"], G=st["G"],
                           epochs_per_step=args.epochs, cuts="redrawn every epoch", cache="device pool, "
                           "epsilon-greedy update (eps 0.1) after every epoch",
                           step="per epoch: cut+pack from the device pool, prefill, fork, sample/decode loop, "
                                "suffix log-probs, advantages, cache update"),
               generated_tokens=int(n_gen), cache_tokens_replaced_frac=round(changed, 4),
               roofline=None, cpu_baseline=None)
    print(json.dumps(out), flush=True)


def run_c4(args):
    """Config C4: teacher-forced log-prob + advantage pass at the 7B shape, every sequence
    re-prefilled on its own (a G = 1 batch: no prefix sharing), LM head on the suffix rows only."""
    import torch
    from paper_2601_19404_amd import binding as rpo
    from paper_2601_19404_amd import synth
    cfg = synth.CONFIGS["C4"]
    mc = cfg.model
    w = synth.make_weights(mc, seed=1234, device="cuda")
    model = rpo.rpo_model_create(mc, w)
    ng = cfg.n_groups if args.groups is None else args.groups
    G, T = cfg.G, cfg.traj_len
    wl = synth.make_workload(cfg, n_groups=ng)
    n_seq = ng * G
    rt = np.random.Generator(np.random.PCG64(1))
    toks = rt.integers(0, mc.vocab, size=(n_seq, T), dtype=np.int32)
    m_seq = np.repeat(wl.m, G)
    order = np.argsort(-m_seq, kind="stable")
    toks, m_seq = toks[order], m_seq[order]
    pre = np.concatenate([toks[i, :T - m_seq[i]] for i in range(n_seq)])
    suf = np.concatenate([toks[i, T - m_seq[i]:] for i in range(n_seq)])
    cu_p = np.concatenate([[0], np.cumsum(T - m_seq)]).astype(np.int32)
    cu_s = np.concatenate([[0], np.cumsum(m_seq)]).astype(np.int32)
    max_prefix, max_suffix = int((T - m_seq).max()), int(m_seq.max())
    batch = rpo.rpo_batch_create(model, n_seq, 1, max_prefix, max_suffix, 64, max(args.max_rows, max_prefix))
    pre_d, suf_d = torch.from_numpy(pre).cuda(), torch.from_numpy(suf).cuda()
    last = torch.empty(n_seq, mc.vocab, dtype=torch.float32, device="cuda")
    lp = torch.empty(int(cu_s[-1]), dtype=torch.float32, device="cuda")
    rewards = torch.from_numpy(wl.rewards).cuda()
    adv = torch.empty(ng, G, dtype=torch.float32, device="cuda")

    def step():
        rpo.rpo_prefill_prefix(batch, pre_d, cu_p, last)
        rpo.rpo_kv_fork(batch)
        rpo.rpo_suffix_logprobs(batch, suf_d, cu_s, cfg.temperature, lp)
        rpo.grpo_advantages(rewards, ng, G, 0, 0.0, adv)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    per_layer = (mc.qkv_rows * mc.d_model + mc.d_model * mc.n_q_heads * mc.head_dim +
                 3 * mc.d_ffn * mc.d_model)
    rows = n_seq * T - n_seq            # the last token of a sequence is never pushed through the layers
    flops = (2.0 * per_layer * mc.n_layers * rows
             + 4.0 * mc.head_dim * mc.n_q_heads * mc.n_layers * n_seq * T * T / 2
             + 2.0 * mc.vocab * mc.d_model * float(cu_s[-1]))
    out = dict(metric="teacher-forced suffix log-prob + advantage pass, sequence tokens/sec at the 7B shape",
               value=n_seq * T / dt, unit="tokens/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=dt * 1e3, higher_is_better=True, scaling="weak", vs_baseline=None, dtype=mc.dtype,
               data="synthetic",
               config=dict(workload=cfg.name, model_shape=mc.name, sequences=n_seq, seq_len=T,
                           suffix_tokens_scored=int(cu_s[-1]), mode="full re-prefill (G = 1 batch)"),
               roofline=dict(bound="mfma", achieved=flops / dt / 1e12, peak=2500.0, unit="TFLOP/s",
                             frac=flops / dt / 1e12 / 2500.0, traffic=None, kernel="whole pass",
                             counted_PFLOP=flops / 1e15))
    print(json.dumps(out), flush=True)


def cpu_baseline(st, budget_tokens: int = 6, prefix_cap: int = 256, n_rollouts: int = 3):
    """The fp64 oracle on the host cores, on a bounded slice of the same workload: group 0,
    its prefix cut to the last `prefix_cap` tokens, `n_rollouts` rollouts, `budget_tokens`
    regenerated tokens each."""
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
    try:
        from threadpoolctl import threadpool_info
        blas = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
    except Exception:
        blas = None
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count()
    return dict(value=gen / dt, unit="tokens/s", cores=int(cores), blas_threads=blas, kind="oracle",
                sample=(f"group 0 of {st['cfg'].name}, prefix cut to its last {len(out['prefix'])} tokens, "
                        f"{n_rollouts} rollouts x {n_tok} regenerated tokens, {dt:.1f} s of fp64 numpy"),
                seconds=dt)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="C1", choices=["C0", "C1", "C2", "C3", "C4"])
    ap.add_argument("--groups", type=int, default=None, help="override the number of groups (debugging)")
    ap.add_argument("--max-rows", type=int, default=32768,
                    help="rows pushed through the layers at once (prefill and log-prob chunks of whole sequences)")
    ap.add_argument("--G", type=int, default=None, help="rollouts per group (paper: 6, 8, 16)")
    ap.add_argument("--temperature", type=float, default=None, help="sampling temperature (paper: 0.7)")
    ap.add_argument("--trunc-max", type=int, default=None,
                    help="draw m ~ U{0..L} as in Eq. 3 (paper: L = 300, 500, 800) instead of the 5-10 %% cut")
    ap.add_argument("--profile-kernel", default="gemm256_swiglu",
                    help="kernel whose launches are ALL timed with HIP events for the roofline object "
                         "(default: the instantiation that leads the kernel table of a step by time)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--epochs", type=int, default=0,
                    help="N > 0: a step is N consecutive passes with the experience cache on the device, cuts "
                         "redrawn per pass and the epsilon-greedy cache update after each (Sec. 3.3, Algorithm 1)")
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
    if args.workload == "C4":
        run_c4(args)
        return
    if args.epochs > 0:
        run_epochs(args)
        return
    st = build_case(args.workload, args.groups, args.max_rows, args.G, args.temperature, args.trunc_max)
    cfg = st["cfg"]
    for i in range(args.warmup):
        one_step(st, seed=100 + i)
    torch.cuda.synchronize()

    # HIP events (recorded by the library on the launch stream) around EVERY launch of the dominant
    # kernel, and around every 5th decode-attention launch (5 is coprime to the 28 launches per
    # step, so all layers are sampled evenly) and every sampler launch: a few thousand event pairs
    # per step, under 1 % of its time.
    timed = {args.profile_kernel: 1}
    for name, every in (("attn_decode", 5), ("sample", 1)):
        timed.setdefault(name, every)
    for name, every in timed.items():
        rpo.rpo_profile_start(rpo.KERNEL_IDS[name], every)
    t0 = time.perf_counter()
    all_marks = []
    for i in range(args.steps):
        marks = []
        res = one_step(st, seed=200 + i, marks=marks)
        all_marks.append(marks)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    phases, enqueue = {}, {}
    for marks in all_marks:
        for (_, e0, c0), (name, e1, c1) in zip(marks[:-1], marks[1:]):
            phases[name] = phases.get(name, 0.0) + e0.elapsed_time(e1) / args.steps
            enqueue[name] = enqueue.get(name, 0.0) + (c1 - c0) * 1e3 / args.steps

    def kernel_report(name):
        launches, k_ms, k_flops, k_bytes = rpo.rpo_profile_stop(rpo.KERNEL_IDS[name])
        bound = KERNEL_BOUND.get(name, "hbm")
        peak, unit = PEAK[bound]
        work = k_bytes / 1e9 if bound == "hbm" else k_flops / 1e12
        achieved = work / (k_ms / 1e3) if launches and k_ms > 0 else 0.0
        every = timed[name]
        return dict(bound=bound, achieved=achieved, peak=peak, unit=unit, frac=achieved / peak,
                    kernel=name, launches_timed=launches, timed_every_nth_launch=every,
                    avg_launch_us=(k_ms * 1e3 / launches) if launches else None,
                    share_of_step_time=(k_ms * every / 1e3) / dt)

    roofline = kernel_report(args.profile_kernel)
    others = {name: kernel_report(name) for name in timed if name != args.profile_kernel}
    roofline["traffic"] = None
    if args.profile_kernel == "gemm256_swiglu" and args.workload == "C1":
        roofline["traffic"] = DOMINANT_TRAFFIC["read_bytes"] + DOMINANT_TRAFFIC["write_bytes"]
        roofline["traffic_of"] = DOMINANT_TRAFFIC
    roofline["other_kernels"] = others

    n_gen = res.n_generated
    value = n_gen * args.steps / dt
    rollout_ms = phases.get("prefill+fork", float("nan")) + phases.get("decode", float("nan"))
    dec_bytes = algorithmic_decode_bytes(st)
    dec_s = phases.get("decode", float("nan")) / 1e3
    bound_ms = step_roofline(st)
    out = dict(metric="suffix-rollout tokens/sec at 1.5B shape; decode HBM GB/s vs peak",
               value=value, unit="tokens/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=dt * 1e3 / args.steps, higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype=cfg.model.dtype, data="synthetic",
               config=dict(workload=cfg.name, model_shape=cfg.model.name, n_groups=st["ng"], G=st["G"],
                           prompt_len=cfg.prompt_len, traj_len=cfg.traj_len,
                           suffix_len_range=[int(st["m"].min()), int(st["m"].max())],
                           generated_tokens_per_step=int(n_gen), page_tokens=st["page"],
                           temperature=cfg.temperature, mean_suffix_len=float(st["m"].mean()),
                           step="cut+pack, prefill, fork, sample/decode loop, suffix log-probs, advantages"),
               phase_ms_per_step={k: round(v, 2) for k, v in phases.items()},
               host_enqueue_ms_per_step={k: round(v, 2) for k, v in enqueue.items()},
               # the rollout alone (prefill + fork + decode loop + sampling), without the log-prob pass
               rollout_tokens_per_s=n_gen / (rollout_ms / 1e3),
               decode_tokens_per_s=(n_gen - st["ng"] * st["G"]) / dec_s,
               decode_hbm=dict(algorithmic_GB_per_step=round(dec_bytes / 1e9, 2),
                               achieved_GBps=dec_bytes / 1e9 / dec_s, peak_GBps=8000.0,
                               frac=dec_bytes / 1e9 / dec_s / 8000.0),
               step_roofline_ms={k: round(v, 2) for k, v in bound_ms.items()},
               frac_of_step_roofline={k: round(bound_ms[k] / v, 3) for k, v in
                                      list(phases.items()) + [("total", dt * 1e3 / args.steps)] if k in bound_ms},
               roofline=roofline)
    # what this GPU sustains on a plain copy and on an MFMA issue loop, measured now (outside the
    # timed region): context for the fractions above, which are against the published peaks
    try:
        copy_gbps, mfma_tflops = rpo.rpo_probe_peaks()
        out["practical_peaks"] = dict(copy_GBps=round(copy_gbps, 1), mfma_bf16_TFLOPs=round(mfma_tflops, 1),
                                      note="plain copy (read + write) and bf16 32x32x16 MFMA issue loop, "
                                           "measured by rpo_probe_peaks in this run")
        practical = mfma_tflops if roofline["bound"] == "mfma" else copy_gbps if roofline["bound"] == "hbm" else 0.0
        roofline["frac_of_practical"] = roofline["achieved"] / practical if practical > 0 else None
    except rpo.RpoError as e:  # the probe is informational
        out["practical_peaks"] = dict(error=str(e))
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(st)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
