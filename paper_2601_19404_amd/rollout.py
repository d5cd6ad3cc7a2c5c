"""Host side of the suffix rollout (RPO Sec. 3.2, Eq. 3; Algorithm 1, rollout
lines): cut the cached answers, pack the prefixes, and drive
prefill -> fork -> {sample, decode}* through librpo.  Only integer bookkeeping
happens here; every arithmetic step runs in the library's kernels.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

from . import binding as rpo


def cut_and_pack(prompts, cached, m):
    """Per group: q_k || a_k[0:-m_k].  Returns (packed int32 tokens, cu_len[n+1])."""
    parts, cu = [], [0]
    for q, a, mk in zip(prompts, cached, m):
        keep = len(a) - int(mk)
        if keep < 0:
            raise ValueError("cut longer than the cached answer")
        parts.append(np.concatenate([np.asarray(q, np.int32), np.asarray(a[:keep], np.int32)]))
        cu.append(cu[-1] + len(parts[-1]))
    return np.concatenate(parts).astype(np.int32), np.asarray(cu, np.int32)


def order_by_suffix_length(m):
    """Permutation that sorts groups by decreasing m: finished groups then always sit at
    the tail of the row range and every decode step runs on a leading block of rows."""
    return np.argsort(-np.asarray(m), kind="stable")


COMPACT_LAG = 8   # decode steps the host may run ahead of the device in a compacted rollout


@dataclass
class RolloutResult:
    tokens: torch.Tensor          # int32 [B, max_m] sampled suffix tokens (row r = group * G + i)
    sample_logprobs: torch.Tensor  # fp32 [B, max_m] log-prob of each token as seen by the sampler
    m: np.ndarray                 # int32 [n_groups] suffix length per group (batch order)
    cu_len: np.ndarray
    n_generated: int
    logits: list | None = None    # per step: fp32 [rows, V] copies when keep_logits
    lengths: torch.Tensor | None = None   # int32 [B] tokens generated per rollout (with eos_id)
    row_of: list | None = None    # compacted rollouts: per decode step, int32 [rows] rollout -> logits row
    rows_computed: list | None = None     # compacted rollouts: logits rows each decode step computed


def suffix_rollout(batch: rpo.Batch, prompts, cached, m, temperature: float, seed: int,
                   seq_ids: torch.Tensor, keep_logits: bool | int = False, stream=None,
                   marks: list | None = None, eos_id: int | None = None, prefix=None,
                   compact: bool = False) -> RolloutResult:
    """Regenerate m_k tokens for each of the G rollouts of every group.

    Groups must be ordered by decreasing m (see order_by_suffix_length) so that the
    live rows are always a leading block.  seq_ids: uint64-valued int64 device tensor
    [B], the Philox stream id of each rollout row.  keep_logits: True keeps a copy of every
    step's logits (tests), an integer n only those of the first n steps.  marks: if a list,
    (name, torch.cuda.Event) pairs are appended at the phase boundaries (benchmark timing).
    eos_id: if given, a rollout that samples it stops there (its later tokens are eos_id padding,
    it appends no more K/V) and the per-rollout lengths are returned; m is then the cap.
    prefix: (packed prefix tokens on the device, cu_len host array) when the cut was already made
    on the device (DeviceCachePool.cut_pack); prompts / cached are then not read.
    compact (with eos_id): finished rollouts leave the decode batch (rpo_decode_step_compact) instead
    of being masked; kept logits are then in compacted row order, RolloutResult.row_of says which
    row of step j belongs to which rollout, RolloutResult.rows_computed how many rows each step ran."""
    cfg = batch.model.cfg
    G, ng = batch.G, batch.n_groups
    B = ng * G
    m = np.asarray(m, np.int32)
    if len(m) != ng or np.any(np.diff(m) > 0):
        raise ValueError("groups must be ordered by decreasing suffix length")
    V = cfg.vocab
    if prefix is not None:
        tokens_dev, cu = prefix
    else:
        toks_host, cu = cut_and_pack(prompts, cached, m)
        tokens_dev = torch.from_numpy(toks_host).cuda()
    max_m = int(m.max()) if ng else 0
    last_logits = torch.empty((ng, V), dtype=torch.float32, device="cuda")
    logits = torch.empty((B, V), dtype=torch.float32, device="cuda")
    # positions a rollout never reaches hold the end-of-sequence id when there is one, else 0
    out_tokens = torch.full((max_m, B), 0 if eos_id is None else int(eos_id), dtype=torch.int32, device="cuda")
    out_lp = torch.zeros((max_m, B), dtype=torch.float32, device="cuda")
    row_map = torch.arange(B, dtype=torch.int32, device="cuda") // G
    row_max = torch.empty(B, dtype=torch.float32, device="cuda")   # per-row logits maximum from the LM head
    active = lengths = None
    eos = -1
    if eos_id is not None:
        eos = int(eos_id)
        active = torch.ones(B, dtype=torch.uint8, device="cuda")
        lengths = torch.zeros(B, dtype=torch.int32, device="cuda")
    kept = [] if keep_logits else None
    n_keep = max_m if keep_logits is True else int(keep_logits)
    if compact and eos_id is None:
        raise ValueError("compact=True needs an end-of-sequence id")
    row_of = torch.empty(B, dtype=torch.int32, device="cuda") if compact else None
    kept_row_of, rows_computed = ([], []) if compact else (None, None)
    step_done = []

    import time

    def mark(name):
        if marks is not None:
            ev = torch.cuda.Event(enable_timing=True)
            ev.record(stream)
            marks.append((name, ev, time.perf_counter()))

    mark("start")
    rpo.rpo_prefill_prefix(batch, tokens_dev, cu, last_logits, stream)
    rpo.rpo_kv_fork(batch, stream)
    mark("prefill+fork")
    # rows alive at step j: groups with m > j, a leading block because m is non-increasing
    live_groups = [int(np.sum(m > j)) for j in range(max_m)]
    if max_m > 0:
        n0 = live_groups[0] * G
        rpo.rpo_sample(last_logits, ng, V, V, row_map, n0, temperature, seed, seq_ids, 0,
                       out_tokens[0], out_lp[0], stream, eos, active, lengths)
        if n_keep > 0:
            kept.append(last_logits.clone())
    for j in range(1, max_m):
        n = live_groups[j] * G
        if n == 0:
            break
        if compact:
            # the host learns the live-row count from the device without waiting; letting it run at
            # most LAG steps ahead keeps that report fresh
            if len(step_done) >= COMPACT_LAG:
                step_done[-COMPACT_LAG].synchronize()
            n_logit = rpo.rpo_decode_step_compact(batch, out_tokens[j - 1], n, active, logits, row_of, stream,
                                                  row_max)
            rows_computed.append(n_logit)
            if n_logit == 0:
                break
            rpo.rpo_sample(logits, n_logit, V, V, row_of, n, temperature, seed, seq_ids, j, out_tokens[j],
                           out_lp[j], stream, eos, active, lengths, row_max)
            ev = torch.cuda.Event()
            ev.record(stream)
            step_done.append(ev)
            if j < n_keep:
                kept.append(logits[:n_logit].clone())
                kept_row_of.append(row_of[:n].clone())
            continue
        rpo.rpo_decode_step(batch, out_tokens[j - 1], n, active, logits, stream, row_max)
        rpo.rpo_sample(logits, n, V, V, None, n, temperature, seed, seq_ids, j, out_tokens[j],
                       out_lp[j], stream, eos, active, lengths, row_max)
        if j < n_keep:
            kept.append(logits[:n].clone())
    mark("decode")
    return RolloutResult(out_tokens.t().contiguous(), out_lp.t().contiguous(), m, cu,
                         int(m.sum()) * G, kept, lengths, kept_row_of, rows_computed)


def suffix_index(m, G: int, max_m: int):
    """Flat positions, inside a [B, max_m] token matrix, of every rollout's m tokens in row
    order, and the cumulative suffix lengths cu_suffix[B+1] (host integers only)."""
    lens = np.repeat(np.asarray(m, np.int64), G)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    rows = np.repeat(np.arange(len(lens), dtype=np.int64), lens)
    cols = np.arange(int(cu[-1]), dtype=np.int64) - np.repeat(cu[:-1].astype(np.int64), lens)
    return rows * max_m + cols, cu


def pack_suffixes(tokens: torch.Tensor, m, G: int, index_dev: torch.Tensor | None = None):
    """tokens [B, max_m] + per-group m -> (packed int32 device tensor, cu_suffix[B+1])."""
    idx, cu = suffix_index(m, G, tokens.shape[1])
    if index_dev is None:
        index_dev = torch.from_numpy(idx).to(tokens.device)
    return tokens.reshape(-1)[index_dev].contiguous(), cu
