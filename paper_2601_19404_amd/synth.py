"""Seeded synthetic inputs: model shapes, random-init weights, prompts, cached
trajectories, cut points and rewards.

This module holds none of the method's arithmetic.  It is the only code the
HIP path's tests and the fp64 oracle's tests have in common: both are handed
the arrays made here.  The paper trains DeepSeek-R1-Distill-Qwen 1.5B / 7B on
open-rs questions (Sec. 4.1); neither weights nor data are available, so
random-init models of the same shapes and uniform random token ids stand in
for them.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch


@dataclass(frozen=True)
class ModelCfg:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str                    # "f32" or "bf16"
    rope_base: float = 1.0e4
    rms_eps: float = 1.0e-6

    @property
    def qkv_rows(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim


@dataclass(frozen=True)
class WorkloadCfg:
    name: str
    model: ModelCfg
    n_groups: int                 # prompts (one sampling group each)
    G: int                        # rollouts per group
    prompt_len: int               # P
    traj_len: int                 # Ta, cached answer length (prompt excluded)
    m_lo: int                     # regenerated-suffix length drawn uniformly
    m_hi: int                     # from {m_lo .. m_hi}, one draw per group
    temperature: float = 1.0
    reward_p: float = 0.5


TINY = ModelCfg("tiny", 2, 128, 4, 2, 32, 256, 512, "f32")
QWEN_1P5B = ModelCfg("1.5B-shape", 28, 1536, 12, 2, 128, 8960, 151936, "bf16")
QWEN_7B = ModelCfg("7B-shape", 28, 3584, 28, 4, 128, 18944, 152064, "bf16")

# C0..C4 of the benchmark description.  m = Ta - c; "cut uniformly in the last
# 5-10 %" -> m in {ceil(.05 Ta) .. floor(.10 Ta)}; the tiny case keeps
# c in {48..56} of 64.
C0 = WorkloadCfg("C0-tiny-suffix", TINY, 2, 4, 16, 64, 8, 16)
C1 = WorkloadCfg("C1-1.5B-suffix", QWEN_1P5B, 64, 8, 128, 2048, 103, 204)
C2 = WorkloadCfg("C2-1.5B-fullpath", QWEN_1P5B, 64, 8, 128, 2048, 2048, 2048)
C3 = WorkloadCfg("C3-7B-suffix", QWEN_7B, 32, 8, 256, 4096, 205, 409)
C4 = WorkloadCfg("C4-7B-logprob", QWEN_7B, 32, 8, 0, 4096, 205, 409, reward_p=0.3)
CONFIGS = {c.name.split("-")[0]: c for c in (C0, C1, C2, C3, C4)}


def torch_dtype(cfg: ModelCfg) -> torch.dtype:
    return torch.float32 if cfg.dtype == "f32" else torch.bfloat16


def make_weights(cfg: ModelCfg, seed: int = 1234, device: str = "cpu",
                 n_layers: int | None = None) -> dict:
    """N(0, 0.02) matrices and embedding, unit norm gains, stored in cfg.dtype
    (bf16 values are the rounded ones: what the GPU multiplies is what the
    oracle reads).  Layout: see include/rpo.h (rpo_weights)."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    dt = torch_dtype(cfg)

    def mat(rows, cols):
        return (torch.randn(rows, cols, generator=g, device=device,
                            dtype=torch.float32) * 0.02).to(dt)

    def ones(n):
        return torch.ones(n, device=device, dtype=dt)

    nl = cfg.n_layers if n_layers is None else n_layers
    w = dict(embed=mat(cfg.vocab, cfg.d_model), lm_head=mat(cfg.vocab, cfg.d_model),
             final_norm=ones(cfg.d_model), layers=[])
    for _ in range(nl):
        w["layers"].append(dict(
            attn_norm=ones(cfg.d_model),
            wqkv=mat(cfg.qkv_rows, cfg.d_model),
            wo=mat(cfg.d_model, cfg.n_q_heads * cfg.head_dim),
            ffn_norm=ones(cfg.d_model),
            w_gate_up=mat(2 * cfg.d_ffn, cfg.d_model),
            w_down=mat(cfg.d_model, cfg.d_ffn)))
    return w


def perturb_gains(w: dict, seed: int = 99) -> dict:
    """Make the norm gains differ from 1 (same dtype) so a dropped or misplaced
    gain shows up in parity tests."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)

    def jig(t):
        r = 1.0 + 0.25 * torch.randn(t.shape, generator=g, dtype=torch.float32)
        return r.to(t.dtype).to(t.device)

    w["final_norm"] = jig(w["final_norm"])
    for lw in w["layers"]:
        lw["attn_norm"] = jig(lw["attn_norm"])
        lw["ffn_norm"] = jig(lw["ffn_norm"])
    return w


def weights_to_numpy(w: dict) -> dict:
    """Same values as float32 numpy arrays on the host (bf16 -> f32 is exact)."""
    def cv(t):
        return t.detach().to("cpu", torch.float32).numpy()
    return dict(embed=cv(w["embed"]), lm_head=cv(w["lm_head"]),
                final_norm=cv(w["final_norm"]),
                layers=[{k: cv(v) for k, v in lw.items()} for lw in w["layers"]])


@dataclass
class Workload:
    cfg: WorkloadCfg
    prompts: np.ndarray           # int32 [n_groups, P]
    cached: np.ndarray            # int32 [n_groups, Ta]
    m: np.ndarray                 # int32 [n_groups]
    rewards: np.ndarray           # float32 [n_groups, G]
    seq_ids: np.ndarray           # uint64 [n_groups * G]
    sample_seed: int = 3


def make_workload(cfg: WorkloadCfg, n_groups: int | None = None, token_seed: int = 1,
                  cut_seed: int = 2, sample_seed: int = 3, reward_seed: int = 4) -> Workload:
    ng = cfg.n_groups if n_groups is None else n_groups
    v = cfg.model.vocab
    rt = np.random.Generator(np.random.PCG64(token_seed))
    prompts = rt.integers(0, v, size=(ng, cfg.prompt_len), dtype=np.int32)
    cached = rt.integers(0, v, size=(ng, cfg.traj_len), dtype=np.int32)
    rc = np.random.Generator(np.random.PCG64(cut_seed))
    m = rc.integers(cfg.m_lo, cfg.m_hi + 1, size=ng, dtype=np.int32)
    rr = np.random.Generator(np.random.PCG64(reward_seed))
    rewards = (rr.random(size=(ng, cfg.G)) < cfg.reward_p).astype(np.float32)
    seq_ids = np.arange(ng * cfg.G, dtype=np.uint64)
    return Workload(cfg, prompts, cached, m, rewards, seq_ids, sample_seed)
