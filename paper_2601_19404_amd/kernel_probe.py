"""Run ONE kernel of librpo alone, a few times, so that a profiler can read its counters:

    rocprofv3 --pmc FETCH_SIZE -d out -o p -- python3 -m paper_2601_19404_amd.kernel_probe copy
    rocprofv3 --pmc FETCH_SIZE -d out -o p -- python3 -m paper_2601_19404_amd.kernel_probe gemm 32768,17920,1536,3

`copy` moves 1 GiB device to device three times (a transfer of known size calibrates the
FETCH_SIZE / WRITE_SIZE counters); `gemm M,N,K,EPI` runs rpo_gemm_nt five times on bf16 N(0,1)
activations and N(0,0.02) weights (EPI as in rpo_gemm_nt: 0 store, 1 fp32 store, 2 fp32
accumulate, 3 fused SwiGLU); `attn` fills the KV pages of a ONE-layer model of the 1.5B widths
with the C1 workload's prefixes (64 groups x 8 rollouts, ~2000-token shared prefixes) plus 100
private tokens per rollout (written by a teacher-forced pass), then runs the shared-prefix decode
attention alone five times
(rpo_attn_decode; the dispatches named attn_decode_mfma_kernel are the ones to read).
Prints one JSON line naming what ran, with the algorithmic bytes of one launch where it applies.
"""
from __future__ import annotations

import json
import sys

import torch

from . import binding as rpo


def probe_copy() -> dict:
    a = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
    b = torch.empty_like(a)
    for _ in range(3):
        b.copy_(a)
    torch.cuda.synchronize()
    return {"copy_probe_bytes_each_way": a.numel() * 4}


def probe_gemm(M: int, N: int, K: int, epi: int, reps: int = 5) -> dict:
    a = torch.randn(M, K, device="cuda").to(torch.bfloat16)
    w = (torch.randn(N, K, device="cuda") * 0.02).to(torch.bfloat16)
    c = torch.zeros(M, N // 2 if epi == 3 else N, device="cuda",
                    dtype=torch.bfloat16 if epi in (0, 3) else torch.float32)
    ws = torch.empty(96 << 20, dtype=torch.uint8, device="cuda")
    for _ in range(reps):
        rpo.rpo_gemm_nt(a, w, c, epi, ws)
    torch.cuda.synchronize()
    return {"gemm_probe": [M, N, K, epi], "launches": reps}


def probe_attn(n_fill: int = 100, reps: int = 5) -> dict:
    import numpy as np

    from . import synth
    mc = synth.ModelCfg("attn-probe", 1, 1536, 12, 2, 128, 256, 512, "bf16")
    wl = synth.make_workload(synth.C1)
    lens = [int(synth.C1.prompt_len + synth.C1.traj_len - mk) for mk in wl.m]
    ng, G = len(lens), synth.C1.G
    B = ng * G
    model = rpo.rpo_model_create(mc, synth.make_weights(mc, seed=1, device="cuda"))
    batch = rpo.rpo_batch_create(model, ng, G, max(lens), n_fill + 1, 64, 32768)
    rng = np.random.default_rng(0)
    toks = torch.from_numpy(rng.integers(0, mc.vocab, size=sum(lens)).astype(np.int32)).cuda()
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    rpo.rpo_prefill_prefix(batch, toks, cu, torch.empty(ng, mc.vocab, device="cuda"))
    rpo.rpo_kv_fork(batch)
    # private pages: a teacher-forced pass over n_fill + 1 random suffix tokens per rollout writes the
    # keys / values of the first n_fill of them
    suffix = torch.from_numpy(rng.integers(0, mc.vocab, size=B * (n_fill + 1)).astype(np.int32)).cuda()
    cu_s = (np.arange(B + 1) * (n_fill + 1)).astype(np.int32)
    rpo.rpo_suffix_logprobs(batch, suffix, cu_s, 1.0, torch.empty(B * (n_fill + 1), device="cuda"))
    q = torch.randn(B, mc.n_q_heads * mc.head_dim, device="cuda").to(torch.bfloat16)
    out = torch.empty_like(q)
    torch.cuda.synchronize()
    for _ in range(reps):
        rpo.rpo_attn_decode(batch, 0, q, B, n_fill, None, out)
    torch.cuda.synchronize()
    kv_tok = 2 * mc.n_kv_heads * mc.head_dim * 2
    shared = sum((n // 64) * 64 for n in lens)
    private = sum((n % 64) + n_fill for n in lens) * G
    return {"attn_probe": {"groups": ng, "G": G, "private_tokens": n_fill}, "launches": reps,
            "algorithmic_kv_bytes_per_launch": (shared + private) * kv_tok,
            "page_granular_kv_bytes_per_launch": (sum(n // 64 for n in lens)
                                                  + sum(-(-((n % 64) + n_fill) // 64) for n in lens) * G) * 64 * kv_tok}


def main(argv) -> int:
    if len(argv) < 1 or argv[0] not in ("copy", "gemm", "attn") or (argv[0] == "gemm" and len(argv) != 2):
        print(__doc__, file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("kernel_probe: no GPU visible", file=sys.stderr)
        return 3
    rpo.lib()
    if argv[0] == "copy":
        out = probe_copy()
    elif argv[0] == "attn":
        out = probe_attn()
    else:
        out = probe_gemm(*(int(v) for v in argv[1].split(",")))
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
