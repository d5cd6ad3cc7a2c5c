"""Run ONE kernel of librpo alone, a few times, so that a profiler can read its counters:

    rocprofv3 --pmc FETCH_SIZE -d out -o p -- python3 -m paper_2601_19404_amd.kernel_probe copy
    rocprofv3 --pmc FETCH_SIZE -d out -o p -- python3 -m paper_2601_19404_amd.kernel_probe gemm 32768,17920,1536,3

`copy` moves 1 GiB device to device three times (a transfer of known size calibrates the
FETCH_SIZE / WRITE_SIZE counters); `gemm M,N,K,EPI` runs rpo_gemm_nt five times on bf16 N(0,1)
activations and N(0,0.02) weights (EPI as in rpo_gemm_nt: 0 store, 1 fp32 store, 2 fp32
accumulate, 3 fused SwiGLU).  Prints one JSON line naming what ran.
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


def main(argv) -> int:
    if len(argv) < 1 or argv[0] not in ("copy", "gemm") or (argv[0] == "gemm" and len(argv) != 2):
        print(__doc__, file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("kernel_probe: no GPU visible", file=sys.stderr)
        return 3
    rpo.lib()
    if argv[0] == "copy":
        out = probe_copy()
    else:
        out = probe_gemm(*(int(v) for v in argv[1].split(",")))
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
