"""Helpers shared by the GPU parity tests: the same seeded arrays go to librpo
(as device tensors) and to the fp64 oracle (as numpy arrays)."""
import numpy as np
import torch

from oracle import sampler as osampler
from oracle import transformer as T
from paper_2601_19404_amd import synth


def oracle_shape(cfg: synth.ModelCfg, n_layers=None, storage="f64") -> T.Shape:
    """storage="model": the precision the model stores its activations / KV in (bf16 models
    quantise them, fp32 models are compared with the exact fp64 forward)."""
    if storage == "model":
        storage = "bf16" if cfg.dtype == "bf16" else "f64"
    return T.Shape(cfg.n_layers if n_layers is None else n_layers, cfg.d_model, cfg.n_q_heads,
                   cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn, cfg.vocab, cfg.rope_base, cfg.rms_eps,
                   storage)


def to_device(w: dict) -> dict:
    mv = lambda t: t.cuda().contiguous()
    return dict(embed=mv(w["embed"]), lm_head=mv(w["lm_head"]), final_norm=mv(w["final_norm"]),
                layers=[{k: mv(v) for k, v in lw.items()} for lw in w["layers"]])


def seq_ids_dev(n: int, base: int = 0) -> torch.Tensor:
    """uint64 Philox stream ids stored in an int64 device tensor."""
    return (torch.arange(n, dtype=torch.int64) + base).cuda()


def check_sampler_consistency(logits_f32: np.ndarray, temperature, seed, seq_ids, step, gpu_tokens,
                              row_map=None):
    """The oracle sampler fed the GPU's logits must return the GPU's tokens, bit for bit."""
    toks, lps = osampler.sample(logits_f32, temperature, seed, seq_ids, step, row_map=row_map)
    np.testing.assert_array_equal(toks, np.asarray(gpu_tokens))
    return lps
