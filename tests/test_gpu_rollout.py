"""End-to-end GPU parity of the suffix rollout against the fp64 oracle.

The GPU samples its own tokens; the oracle then (a) recomputes, teacher-forced on
those tokens, every logits row the GPU sampled from and every suffix log-prob
(floating point: within the stated tolerance), and (b) is fed the GPU's logits and
must return the GPU's tokens (integers: bit-exact).

Tolerances against the exact fp64 forward: 1e-4 (fp32 model), 2e-2 (bf16 models) on
logits and log-probs.  A model with bf16 matrix operands and a bf16 KV cache quantises
those tensors; that alone moves the logits of a two-layer random-init stack by ~0.5 % of
their standard deviation rms, so over 1e6 logits of standard deviation 0.8 the maximum
sits at the 2e-2 mark for ANY bf16-operand implementation.  bf16 cases are therefore
judged three ways:
  * against the quantisation noise floor measured with the oracle itself: exact forward
    vs the forward that rounds the minimal set of tensors a bf16-operand model must round
    (projection operands, q and k after the rotation, the cached k and v -- each once;
    nothing before the rotation, no probabilities): GPU error <= FLOOR_RMS x floor rms and
    <= FLOOR_MAX x floor max on the same rows.  Whatever else the kernels round counts
    against them;
  * against that rounded forward directly, in units of one bf16 ulp of the logit scale
    (models of at most two layers, where two correct pipelines cannot drift apart);
  * against the absolute 2e-2 wherever the floor leaves room for it (decided by the floor
    itself, not by the case)."""
import numpy as np
import pytest
import torch

from oracle import advantages as oadv
from oracle import transformer as T
from paper_2601_19404_amd import synth
from tests import util

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
FLOOR_RMS, FLOOR_MAX = 1.25, 1.5     # allowed GPU error in units of the bf16 quantisation floor
ULP_RMS, ULP_MAX = 1.25, 6.0         # allowed distance to the rounded forward, in bf16 ulps of the logit scale


def bf16_ulp(x: float) -> float:
    """Spacing of bfloat16 numbers around |x| (8 significand bits)."""
    return float(2.0 ** (np.floor(np.log2(abs(x))) - 7))


@pytest.fixture(scope="module")
def rpo():
    from paper_2601_19404_amd import binding
    binding.lib()
    yield binding
    binding.rpo_set_kernel_path(0)


def run_case(rpo, mcfg, prompts, cached, m, G, temperature=1.0, seed=3, page=64, path=0,
             max_rows=None, weight_seed=1234, perturb=True, check_logprobs=True, n_layers=None,
             eos_from=None, oracle_rollouts=None, compact=False):
    """One batch through librpo, then element-by-element against the oracle.

    eos_from = (row, step): a first, unconstrained run picks the token that rollout `row` drew at
    `step`; the checked run then uses it as the end-of-sequence id, so that rollout (and any other
    that happens to draw the id) stops early and the `active` mask reaches every decode kernel.
    oracle_rollouts: which rollouts of each group the oracle recomputes (default: all G); the
    integer contract (oracle sampler on the GPU's logits) always covers every row and step.
    compact: the checked run drops finished rollouts from the decode batch (rpo_decode_step_compact)."""
    from paper_2601_19404_amd import rollout
    rpo.rpo_set_kernel_path(path)
    w = synth.make_weights(mcfg, seed=weight_seed, n_layers=n_layers)
    if perturb:
        w = synth.perturb_gains(w)
    w_np = synth.weights_to_numpy(w)
    shape = util.oracle_shape(mcfg, n_layers)
    shape_q = util.oracle_shape(mcfg, n_layers, storage="model")
    cfg = mcfg if n_layers is None else synth.ModelCfg(**{**mcfg.__dict__, "n_layers": n_layers})
    model = rpo.rpo_model_create(cfg, util.to_device(w))
    order = rollout.order_by_suffix_length(m)
    prompts = [prompts[i] for i in order]
    cached = [cached[i] for i in order]
    m = np.asarray(m)[order]
    ng = len(prompts)
    B = ng * G
    pref_lens = [len(p) + len(a) - int(mm) for p, a, mm in zip(prompts, cached, m)]
    max_prefix, max_suffix = max(pref_lens), max(int(m.max()), 1)
    if max_rows is None:
        max_rows = max(max_prefix, B, max_suffix)
    batch = rpo.rpo_batch_create(model, ng, G, max_prefix, max_suffix, page, max_rows)
    seq_ids = util.seq_ids_dev(B, base=1000)
    eos = None
    if eos_from is not None:
        free = rollout.suffix_rollout(batch, prompts, cached, m, temperature, seed, seq_ids)
        torch.cuda.synchronize()
        eos = int(free.tokens[eos_from[0], eos_from[1]].item())
    res = rollout.suffix_rollout(batch, prompts, cached, m, temperature, seed, seq_ids, keep_logits=True,
                                 eos_id=eos, compact=compact)
    torch.cuda.synchronize()
    toks = res.tokens.cpu().numpy()
    slp = res.sample_logprobs.cpu().numpy()
    kept = [k.cpu().numpy() for k in res.logits]
    row_of = [None] + [t.cpu().numpy() for t in res.row_of] if compact else None

    def logits_row(j, r):
        """The logits row rollout r drew its token j from."""
        if j == 0:
            return kept[0][r // G]
        return kept[j][row_of[j][r] if compact else r]

    sid = np.arange(1000, 1000 + B).astype(np.uint64)
    tol = TOL[mcfg.dtype]
    # tokens each rollout really generated (the end-of-sequence token counts)
    if eos is None:
        n_gen = np.repeat(m, G).astype(np.int64)
    else:
        n_gen = res.lengths.cpu().numpy().astype(np.int64)
        ft = free.tokens.cpu().numpy()
        for r in range(B):
            mg = int(m[r // G])
            hit = np.flatnonzero(ft[r, :mg] == eos)
            n = hit[0] + 1 if len(hit) else mg
            assert n_gen[r] == n, "a rollout stops right after it draws the end-of-sequence id"
            np.testing.assert_array_equal(toks[r, :n], ft[r, :n])      # same draws until the stop
            assert np.all(toks[r, n:mg] == eos)                        # padding after it
        assert n_gen[eos_from[0]] <= eos_from[1] + 1
        assert np.any(n_gen < np.repeat(m, G)) and np.any(n_gen == np.repeat(m, G))

    # (b) integer contract: oracle sampler on the GPU's logits, every live row of every step
    max_m = int(m.max())
    for j in range(max_m):
        n = int(np.sum(m > j)) * G
        if n == 0:
            break
        live = np.flatnonzero(n_gen[:n] > j)
        if len(live) == 0:
            continue
        z = np.stack([logits_row(j, r) for r in live])
        util.check_sampler_consistency(z, temperature, seed, sid[live], j, toks[live, j])
    if compact:
        # finished rollouts really left the batch: at some step fewer rows ran than rollouts were covered
        covered = [int(np.sum(m > j)) * G for j in range(1, 1 + len(res.rows_computed))]
        assert all(c <= n for c, n in zip(res.rows_computed, covered))
        assert any(c < n for c, n in zip(res.rows_computed, covered)), "no step ran on fewer rows"
        for j in range(1, len(row_of)):
            n = covered[j - 1]
            alive = n_gen[:n] > j
            assert np.all(row_of[j][:n][~alive] == -1)
            np.testing.assert_array_equal(row_of[j][:n][alive], np.arange(int(alive.sum())))

    # (a) floating point: oracle logits teacher-forced on the GPU's tokens
    which = range(G) if oracle_rollouts is None else oracle_rollouts
    worst, sq, cnt = 0.0, 0.0, 0
    slp_err = 0.0
    floor, err0, errq, ref_all = [], [], [], []
    for g in range(ng):
        prefix = np.concatenate([prompts[g], cached[g][:len(cached[g]) - int(m[g])]])
        for i in which:
            r = g * G + i
            mg = int(n_gen[r])
            if mg == 0:
                continue
            ref = T.teacher_forced_logits(shape, w_np, prefix, toks[r, :mg])
            got = np.stack([logits_row(j, r) for j in range(mg)]).astype(np.float64)
            if shape_q.storage != "f64" and i == which[0]:
                ref_q = T.teacher_forced_logits(shape_q, w_np, prefix, toks[r, :mg])
                floor.append((ref_q - ref).ravel())
                err0.append((got - ref).ravel())
                errq.append((got - ref_q).ravel())
                ref_all.append(ref.ravel())
            worst = max(worst, float(np.max(np.abs(got - ref))))
            sq += float(np.sum((got - ref) ** 2))
            cnt += got.size
            lp_ref = T.log_softmax(ref / temperature)[np.arange(mg), toks[r, :mg]]
            slp_err = max(slp_err, float(np.max(np.abs(slp[r, :mg] - lp_ref))))
    print(f"[{mcfg.name} path={path} G={G}] logits vs oracle: max {worst:.3e} rms {np.sqrt(sq / max(cnt, 1)):.3e} "
          f"over {cnt} values", flush=True)
    lp_tol = tol
    if floor:
        floor, err0, errq = np.concatenate(floor), np.concatenate(err0), np.concatenate(errq)
        f_rms, f_max = np.sqrt(np.mean(floor ** 2)), np.abs(floor).max()
        e_rms, e_max = np.sqrt(np.mean(err0 ** 2)), np.abs(err0).max()
        ulp = bf16_ulp(np.concatenate(ref_all).std())
        q_rms, q_max = np.sqrt(np.mean(errq ** 2)) / ulp, np.abs(errq).max() / ulp
        print(f"    bf16 floor rms {f_rms:.3e} max {f_max:.3e}; GPU on the same rows rms {e_rms:.3e} "
              f"max {e_max:.3e} (x{e_rms / f_rms:.2f}, x{e_max / f_max:.2f}); GPU vs rounded forward: "
              f"rms {q_rms:.2f} max {q_max:.2f} bf16 ulps of the logit scale ({ulp:.2e})", flush=True)
        assert e_rms <= FLOOR_RMS * f_rms and e_max <= FLOOR_MAX * f_max
        if shape.n_layers <= 2:
            assert q_rms <= ULP_RMS and q_max <= ULP_MAX
        lp_tol = max(tol, FLOOR_MAX * f_max)
        if FLOOR_MAX * f_max < tol:      # the floor leaves room for the absolute bound
            assert worst < tol, f"logits differ from the oracle by {worst}"
        else:
            assert np.sqrt(sq / max(cnt, 1)) < tol
    else:
        assert worst < tol, f"logits differ from the oracle by {worst}"
    assert slp_err < lp_tol, f"sampler log-probs differ from the oracle by {slp_err}"

    if check_logprobs:
        packed, cu_s = rollout.pack_suffixes(res.tokens, m, G)
        out = torch.full((max(int(cu_s[-1]), 1),), 7.0, dtype=torch.float32, device="cuda")
        rpo.rpo_suffix_logprobs(batch, packed, cu_s, temperature, out)
        torch.cuda.synchronize()
        out = out.cpu().numpy()
        for g in range(ng):
            prefix = np.concatenate([prompts[g], cached[g][:len(cached[g]) - int(m[g])]])
            for i in which:
                r = g * G + i
                mg = int(m[g])
                # teacher-forced over the whole (padded) suffix; compared where the rollout was live
                ref = T.suffix_logprobs(shape, w_np, prefix, toks[r, :mg], temperature)
                got = out[cu_s[r]:cu_s[r + 1]]
                assert got.shape == ref.shape
                if mg:
                    assert np.max(np.abs(got - ref)) < lp_tol, "suffix log-probs"
                    # one policy: ratio of Eq. 7 is 1 -> same value as the sampler reported
                    ng_r = int(n_gen[r])
                    assert np.max(np.abs(got[:ng_r] - slp[r, :ng_r])) < 2 * tol
    return worst, res


def tiny_workload(ng=2, seed=1):
    wl = synth.make_workload(synth.C0, n_groups=ng, token_seed=seed, cut_seed=seed + 1)
    return [wl.prompts[k] for k in range(ng)], [wl.cached[k] for k in range(ng)], wl.m


def test_c0_tiny_fp32_end_to_end(rpo):
    """The tiny benchmark configuration exactly: 2 prompts x G=4, prompt 16, answer 64 cut in [48, 56]."""
    p, a, m = tiny_workload()
    worst, res = run_case(rpo, synth.TINY, p, a, m, G=4, page=16)
    assert res.n_generated == int(m.sum()) * 4
    # rewards -> advantages, bit-exact
    wl = synth.make_workload(synth.C0)
    out = torch.empty(2, 4, dtype=torch.float32, device="cuda")
    rpo.grpo_advantages(torch.from_numpy(wl.rewards).cuda(), 2, 4, 0, 0.0, out)
    np.testing.assert_array_equal(out.cpu().numpy(), oadv.grpo_advantages(wl.rewards))


@pytest.mark.parametrize("page", [16, 32, 64])
def test_tiny_fp32_page_sizes_and_chunked_prefill(rpo, page):
    p, a, m = tiny_workload(ng=5, seed=11)
    # max_rows below the total prefix rows forces several prefill chunks
    run_case(rpo, synth.TINY, p, a, m, G=3, page=page, max_rows=150, temperature=0.7)


def test_tiny_fp32_edge_lengths(rpo):
    """Prefix lengths around page boundaries (no partial page to copy, prefix shorter than a
    page, one-token prefix) and a group that regenerates nothing (m = 0)."""
    rng = np.random.default_rng(7)
    v = synth.TINY.vocab
    prompts = [rng.integers(0, v, size=n).astype(np.int32) for n in (16, 16, 1, 5, 16)]
    cached = [rng.integers(0, v, size=n).astype(np.int32) for n in (32, 19, 6, 30, 20)]
    m = np.array([16, 3, 6, 9, 0])          # prefixes: 32 (= 2 pages), 32, 1, 26, 36
    run_case(rpo, synth.TINY, prompts, cached, m, G=2, page=16)


BF16_SMALL = synth.ModelCfg("bf16-small", 2, 768, 6, 1, 128, 1024, 2048, "bf16")
BF16_GQA7 = synth.ModelCfg("bf16-gqa7", 2, 896, 7, 1, 128, 512, 1024, "bf16")
BF16_2KV = synth.ModelCfg("bf16-2kv", 3, 1536, 12, 2, 128, 1024, 4096, "bf16")


def bf16_workload(mcfg, lens, ms, seed=0):
    rng = np.random.default_rng(seed)
    prompts = [rng.integers(0, mcfg.vocab, size=8).astype(np.int32) for _ in lens]
    cached = [rng.integers(0, mcfg.vocab, size=n).astype(np.int32) for n in lens]
    return prompts, cached, np.asarray(ms)


@pytest.mark.parametrize("path", [1, 0])
def test_bf16_small_generic_and_mfma(rpo, path):
    """Same case through the generic kernels (path 1) and the MFMA kernels (path 0): prefixes
    spanning several 64-token pages with ragged tails, G = 8 rollouts sharing them."""
    p, a, m = bf16_workload(BF16_SMALL, lens=(200, 333, 130), ms=(9, 12, 5))
    run_case(rpo, BF16_SMALL, p, a, m, G=8, path=path)


def test_bf16_gqa7_mfma(rpo):
    """7 query heads per KV head (the 7B shape's ratio): 8 x 7 = 56 query rows per shared page."""
    p, a, m = bf16_workload(BF16_GQA7, lens=(190, 64, 70), ms=(6, 8, 3), seed=1)
    run_case(rpo, BF16_GQA7, p, a, m, G=8)


def test_bf16_two_kv_heads_many_rollouts_mfma(rpo):
    """12 q / 2 kv heads (the 1.5B shape's ratio) and G = 16: two column tiles per group;
    prefix of exactly 4 pages, a prefix shorter than one page, chunked prefill."""
    p, a, m = bf16_workload(BF16_2KV, lens=(256 - 8 + 7, 40, 150), ms=(7, 10, 4), seed=2)
    run_case(rpo, BF16_2KV, p, a, m, G=16, max_rows=300)


def test_bf16_many_rows_wide_rotary_tile(rpo):
    """528 rollouts x 16 heads: more 32-row tiles than CUs, so the QKV projection of a decode step
    takes its 64-row tiles (rotation and KV page write in the epilogue), with a ragged last tile."""
    ng = 33
    lens = tuple(20 + (5 * k) % 23 for k in range(ng))
    p, a, m = bf16_workload(BF16_2KV, lens=lens, ms=(2,) * ng, seed=5)
    run_case(rpo, BF16_2KV, p, a, m, G=16)


def long_suffix_workload(mcfg, prompt_len, lens, ms, seed):
    rng = np.random.default_rng(seed)
    prompts = [rng.integers(0, mcfg.vocab, size=prompt_len).astype(np.int32) for _ in lens]
    cached = [rng.integers(0, mcfg.vocab, size=n).astype(np.int32) for n in lens]
    return prompts, cached, np.asarray(ms)


@pytest.mark.parametrize("G", [8, 6])
def test_bf16_long_suffix_across_private_pages(rpo, G):
    """What a full-size rollout does, on a two-layer model: 150-200 regenerated tokens per rollout,
    so every rollout walks through 3-4 private pages (each page boundary crossed while decoding) on
    top of 4-6 shared prefix pages; the paper's sampling settings (Sec. 4.1: temperature 0.7, group
    size 6 next to 8, i.e. 36 and 48 query columns per shared page); one group that regenerates
    nothing (m = 0) in the same batch.  Every logits row of every step against the fp64 oracle."""
    p, a, m = long_suffix_workload(BF16_SMALL, 24, lens=(520, 470, 600, 300), ms=(197, 171, 150, 0), seed=31)
    run_case(rpo, BF16_SMALL, p, a, m, G=G, temperature=0.7, oracle_rollouts=(0, G - 1, 3))


def test_bf16_long_suffix_with_end_of_sequence(rpo):
    """The same walk through private pages with an end-of-sequence id: rollouts stop at different
    steps, so the `active` mask reaches the shared-prefix attention, the rotary / KV-append
    epilogue and the sampler on the MFMA path; live rows against the oracle, stopped rows padded."""
    p, a, m = long_suffix_workload(BF16_SMALL, 24, lens=(500, 450, 380), ms=(180, 160, 140), seed=32)
    run_case(rpo, BF16_SMALL, p, a, m, G=8, temperature=0.7, eos_from=(9, 70), oracle_rollouts=(0, 1, 5))


@pytest.mark.parametrize("mcfg,page", [(BF16_SMALL, 64), (synth.TINY, 16)])
def test_end_of_sequence_with_batch_compaction(rpo, mcfg, page):
    """Variable-length rollouts with finished rollouts REMOVED from the decode batch
    (rpo_decode_step_compact): the rows of a step are the live rollouts in order, the projections
    run on them only, and every live row still matches the oracle (MFMA kernels and, on the fp32
    model, the generic ones)."""
    p, a, m = long_suffix_workload(mcfg, 24, lens=(200, 170, 140), ms=(90, 80, 70), seed=35)
    run_case(rpo, mcfg, p, a, m, G=8, temperature=0.7, page=page, eos_from=(9, 20), oracle_rollouts=(0, 1, 5),
             compact=True)


def test_bf16_prompt_only_prefix_decoded_past_two_pages(rpo):
    """The full-path baseline's shape: nothing of the cached answer is kept (c = 0), the shared
    prefix is the 128-token prompt (exactly two pages, no partial page to fork) and 140 tokens are
    decoded from it."""
    mcfg = BF16_GQA7
    rng = np.random.default_rng(33)
    prompts = [rng.integers(0, mcfg.vocab, size=128).astype(np.int32) for _ in range(2)]
    cached = [rng.integers(0, mcfg.vocab, size=140).astype(np.int32) for _ in range(2)]
    run_case(rpo, mcfg, prompts, cached, np.asarray([140, 140]), G=8, oracle_rollouts=(0, 6))


def test_bf16_wide_gqa_private_pieces(rpo):
    """32 query heads on one KV head: the private-page piece of a rollout spans two 16-column
    query tiles (heads 16..31 once fell out of it)."""
    mcfg = synth.ModelCfg("bf16-gqa32", 2, 1024, 32, 1, 128, 512, 1024, "bf16")
    p, a, m = bf16_workload(mcfg, lens=(150, 70), ms=(9, 6), seed=34)
    run_case(rpo, mcfg, p, a, m, G=2)


def test_logprob_pass_c4_shape_several_chunks(rpo):
    """The log-prob benchmark's call pattern on a two-layer model: every sequence re-prefilled on its
    own (a G = 1 batch), suffix = the last m tokens with m drawn per group of 4 sequences, and
    max_rows small enough that both the prefill and the log-prob pass run in several chunks of
    whole sequences."""
    mcfg = BF16_SMALL
    rng = np.random.default_rng(41)
    w = synth.perturb_gains(synth.make_weights(mcfg, seed=78))
    w_np = synth.weights_to_numpy(w)
    shape, shape_q = util.oracle_shape(mcfg), util.oracle_shape(mcfg, storage="model")
    model = rpo.rpo_model_create(mcfg, util.to_device(w))
    T_len, ms = 640, np.repeat([300, 251, 205], 4)          # descending, 4 sequences per group
    seqs = rng.integers(0, mcfg.vocab, size=(len(ms), T_len)).astype(np.int32)
    pre = [seqs[i, :T_len - ms[i]] for i in range(len(ms))]
    suf = [seqs[i, T_len - ms[i]:] for i in range(len(ms))]
    cu_p = np.concatenate([[0], np.cumsum([len(x) for x in pre])]).astype(np.int32)
    cu_s = np.concatenate([[0], np.cumsum(ms)]).astype(np.int32)
    batch = rpo.rpo_batch_create(model, len(ms), 1, int(max(np.diff(cu_p))), int(ms.max()), 64, 700)
    last = torch.empty(len(ms), mcfg.vocab, device="cuda")
    rpo.rpo_prefill_prefix(batch, torch.from_numpy(np.concatenate(pre)).cuda(), cu_p, last)
    rpo.rpo_kv_fork(batch)
    out = torch.full((int(cu_s[-1]),), 9.0, dtype=torch.float32, device="cuda")
    rpo.rpo_suffix_logprobs(batch, torch.from_numpy(np.concatenate(suf)).cuda(), cu_s, 1.0, out)
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    worst, floor_max = 0.0, 0.0
    for k in range(len(ms)):
        ref = T.suffix_logprobs(shape, w_np, pre[k], suf[k], 1.0)
        if k % 4 == 0:
            floor_max = max(floor_max, float(np.max(np.abs(T.suffix_logprobs(shape_q, w_np, pre[k], suf[k], 1.0) - ref))))
        worst = max(worst, float(np.max(np.abs(out[cu_s[k]:cu_s[k + 1]] - ref))))
    print(f"C4-shaped log-prob pass vs oracle: max {worst:.3e} (bf16 floor max {floor_max:.3e})", flush=True)
    assert worst < max(TOL["bf16"], FLOOR_MAX * floor_max)


def test_7b_shape_two_layers(rpo):
    """The 7B configuration's widths (d 3584, 28 q / 4 kv heads, F 18944, V 152064) on two layers:
    the projections take the tile shapes they take in the 7B benchmark (K = 3584 narrow tiles,
    K = 18944 split along K, 7 query heads per KV head, fused log-sum-exp over 594 column tiles)."""
    mcfg = synth.QWEN_7B
    rng = np.random.default_rng(12)
    prompts = [rng.integers(0, mcfg.vocab, size=8).astype(np.int32) for _ in range(2)]
    cached = [rng.integers(0, mcfg.vocab, size=n).astype(np.int32) for n in (150, 90)]
    run_case(rpo, mcfg, prompts, cached, np.asarray([5, 4]), G=4, n_layers=2)


BF16_WIDE_VOCAB = synth.ModelCfg("bf16-wide-vocab", 2, 768, 6, 1, 128, 1024, 33000, "bf16")


def test_bf16_wide_vocab_fused_logprobs(rpo):
    """A vocabulary wide enough (129 column tiles, the last one ragged) and enough scored rows that
    the log-prob pass takes its log-sum-exp inside the LM-head epilogue; checked against the oracle
    like every other case, and against the unfused path (register-staged GEMM, logits in memory)."""
    from paper_2601_19404_amd import rollout
    p, a, m = bf16_workload(BF16_WIDE_VOCAB, lens=(70, 100, 130), ms=(12, 9, 11), seed=4)
    _, res = run_case(rpo, BF16_WIDE_VOCAB, p, a, m, G=4)
    order = rollout.order_by_suffix_length(m)
    prompts = [p[i] for i in order]
    cached = [a[i] for i in order]
    ms = np.asarray(m)[order]
    outs = []
    for path in (0, 2):
        rpo.rpo_set_kernel_path(path)
        w = synth.perturb_gains(synth.make_weights(BF16_WIDE_VOCAB, seed=1234))
        model = rpo.rpo_model_create(BF16_WIDE_VOCAB, util.to_device(w))
        toks, cu = rollout.cut_and_pack(prompts, cached, ms)
        batch = rpo.rpo_batch_create(model, 3, 4, int(max(np.diff(cu))), int(ms.max()), 64, 256)
        last = torch.empty(3, BF16_WIDE_VOCAB.vocab, device="cuda")
        rpo.rpo_prefill_prefix(batch, torch.from_numpy(toks).cuda(), cu, last)
        rpo.rpo_kv_fork(batch)
        packed, cu_s = rollout.pack_suffixes(res.tokens, ms, 4)
        packed = packed.clone()
        packed[5] = -3                                   # a target outside the vocabulary scores NaN
        out = torch.zeros(int(cu_s[-1]), dtype=torch.float32, device="cuda")
        rpo.rpo_suffix_logprobs(batch, packed, cu_s, 1.0, out)
        torch.cuda.synchronize()
        outs.append(out.cpu().numpy())
    rpo.rpo_set_kernel_path(0)
    assert np.isnan(outs[0][5]) and np.isnan(outs[1][5])
    ok = np.ones(len(outs[0]), bool)
    ok[5] = False
    ok[6] = False    # the row after the bad token was fed an out-of-range embedding id
    assert np.max(np.abs(outs[0][ok] - outs[1][ok])) < 2e-2


def test_logprob_pass_full_reprefill_on_a_g1_batch(rpo):
    """The log-prob pass that re-prefills every sequence on its own (no sharing: a batch created
    with G = 1, the way the 7B log-prob benchmark calls it) against the oracle, and against the
    same sequences scored through shared prefixes (G = 3 rollouts per prefix)."""
    mcfg = BF16_SMALL
    rng = np.random.default_rng(21)
    w = synth.perturb_gains(synth.make_weights(mcfg, seed=77))
    w_np = synth.weights_to_numpy(w)
    shape, shape_q = util.oracle_shape(mcfg), util.oracle_shape(mcfg, storage="model")
    model = rpo.rpo_model_create(mcfg, util.to_device(w))
    G, pre_lens, ms = 3, (150, 64, 97), (11, 7, 4)          # suffix lengths in descending order
    prefixes = [rng.integers(0, mcfg.vocab, size=n).astype(np.int32) for n in pre_lens]
    suffixes = [[rng.integers(0, mcfg.vocab, size=m).astype(np.int32) for _ in range(G)] for m in ms]
    temp = 1.3

    def score(n_groups, g_per, prefix_list, suffix_list):
        cu_p = np.concatenate([[0], np.cumsum([len(x) for x in prefix_list])]).astype(np.int32)
        cu_s = np.concatenate([[0], np.cumsum([len(x) for x in suffix_list])]).astype(np.int32)
        batch = rpo.rpo_batch_create(model, n_groups, g_per, int(max(np.diff(cu_p))), max(ms), 64, 512)
        last = torch.empty(n_groups, mcfg.vocab, device="cuda")
        rpo.rpo_prefill_prefix(batch, torch.from_numpy(np.concatenate(prefix_list)).cuda(), cu_p, last)
        rpo.rpo_kv_fork(batch)
        out = torch.full((int(cu_s[-1]),), 9.0, dtype=torch.float32, device="cuda")
        rpo.rpo_suffix_logprobs(batch, torch.from_numpy(np.concatenate(suffix_list)).cuda(), cu_s, temp, out)
        torch.cuda.synchronize()
        return out.cpu().numpy(), cu_s

    flat_suffixes = [sfx for grp in suffixes for sfx in grp]
    shared, cu_s = score(len(prefixes), G, prefixes, flat_suffixes)
    own, cu_s1 = score(len(prefixes) * G, 1, [prefixes[k // G] for k in range(len(prefixes) * G)], flat_suffixes)
    np.testing.assert_array_equal(cu_s, cu_s1)
    worst, floor_max = 0.0, 0.0
    for k, sfx in enumerate(flat_suffixes):
        ref = T.suffix_logprobs(shape, w_np, prefixes[k // G], sfx, temp)
        ref_q = T.suffix_logprobs(shape_q, w_np, prefixes[k // G], sfx, temp)
        floor_max = max(floor_max, float(np.max(np.abs(ref_q - ref))))
        for got in (shared, own):
            worst = max(worst, float(np.max(np.abs(got[cu_s[k]:cu_s[k + 1]] - ref))))
    tol = max(TOL["bf16"], FLOOR_MAX * floor_max)
    print(f"log-probs vs oracle: max {worst:.3e} (bf16 storage floor max {floor_max:.3e})", flush=True)
    assert worst < tol
    assert np.max(np.abs(shared - own)) < tol            # two routes to the same numbers


@pytest.mark.parametrize("mcfg,rows_per_group", [(BF16_WIDE_VOCAB, 32), (BF16_SMALL, 4)])
def test_decode_row_max_output(rpo, mcfg, rows_per_group):
    """rpo_decode_step's row maxima equal the maxima of the logits it returns, bit for bit: from the
    LM-head epilogue (wide vocabulary, 96 rows) and from the plain kernel (small problem)."""
    from paper_2601_19404_amd import rollout
    rpo.rpo_set_kernel_path(0)
    model = rpo.rpo_model_create(mcfg, util.to_device(synth.make_weights(mcfg, seed=9)))
    p, a, m = bf16_workload(mcfg, lens=(70, 100, 130), ms=(4, 4, 4), seed=6)
    G, ng, V = rows_per_group, 3, mcfg.vocab
    toks, cu = rollout.cut_and_pack(p, a, m)
    batch = rpo.rpo_batch_create(model, ng, G, int(max(np.diff(cu))), 8, 64, 256)
    last = torch.empty(ng, V, device="cuda")
    rpo.rpo_prefill_prefix(batch, torch.from_numpy(toks).cuda(), cu, last)
    rpo.rpo_kv_fork(batch)
    B = ng * G
    step_tok = (torch.arange(B, dtype=torch.int32, device="cuda") * 7 + 3) % V
    for n in (B, B - G):
        logits = torch.full((B, V), float("nan"), device="cuda")
        ref = torch.empty_like(logits)
        rmax = torch.full((B,), float("nan"), device="cuda")
        rpo.rpo_decode_step(batch, step_tok, n, None, logits, row_max_out_dev=rmax)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(rmax[:n].cpu().numpy(), logits[:n].max(dim=1).values.cpu().numpy())
        assert np.all(np.isfinite(logits[:n].cpu().numpy()))


def test_decode_active_mask_and_row_prefix(rpo):
    """Rows masked out by `active` must not disturb the live ones; a shorter leading block works."""
    from paper_2601_19404_amd import rollout
    rpo.rpo_set_kernel_path(0)
    mcfg = BF16_SMALL
    w = synth.make_weights(mcfg, seed=5)
    model = rpo.rpo_model_create(mcfg, util.to_device(w))
    p, a, m = bf16_workload(mcfg, lens=(100, 90), ms=(4, 4), seed=3)
    G, ng, V = 4, 2, mcfg.vocab
    toks, cu = rollout.cut_and_pack(p, a, m)
    outs = []
    for mask in (None, [1, 1, 0, 1, 1, 1, 1, 0]):
        batch = rpo.rpo_batch_create(model, ng, G, int(max(np.diff(cu))), 8, 64, 256)
        last = torch.empty(ng, V, device="cuda")
        rpo.rpo_prefill_prefix(batch, torch.from_numpy(toks).cuda(), cu, last)
        rpo.rpo_kv_fork(batch)
        step_tok = torch.arange(8, dtype=torch.int32, device="cuda") * 7 + 3
        logits = torch.full((8, V), float("nan"), device="cuda")
        act = None if mask is None else torch.tensor(mask, dtype=torch.uint8, device="cuda")
        rpo.rpo_decode_step(batch, step_tok, 8, act, logits)
        rpo.rpo_decode_step(batch, step_tok + 1, 8, act, logits)
        torch.cuda.synchronize()
        outs.append(logits.cpu().numpy())
    live = np.array([1, 1, 0, 1, 1, 1, 1, 0], bool)
    np.testing.assert_array_equal(outs[0][live], outs[1][live])
    assert np.all(np.isfinite(outs[0]))


def test_state_and_argument_errors(rpo):
    from paper_2601_19404_amd import rollout
    mcfg = synth.TINY
    model = rpo.rpo_model_create(mcfg, util.to_device(synth.make_weights(mcfg)))
    with pytest.raises(rpo.RpoError):
        rpo.rpo_batch_create(model, 2, 4, 80, 16, 24, 128)            # page size not a power of two
    with pytest.raises(rpo.RpoError):
        rpo.rpo_batch_create(model, 2, 4, 80, 16, 16, 40)             # max_rows < max_prefix
    batch = rpo.rpo_batch_create(model, 2, 4, 80, 2, 16, 128)
    V = mcfg.vocab
    logits = torch.empty(8, V, device="cuda")
    tok = torch.zeros(8, dtype=torch.int32, device="cuda")
    with pytest.raises(rpo.RpoError) as e:
        rpo.rpo_decode_step(batch, tok, 8, None, logits)              # before prefill / fork
    assert e.value.code == rpo.RPO_ESTATE
    with pytest.raises(rpo.RpoError) as e:
        rpo.rpo_kv_fork(batch)
    assert e.value.code == rpo.RPO_ESTATE
    p, a, m = tiny_workload()
    toks, cu = rollout.cut_and_pack(p, a, m)
    bad = cu.copy()
    bad[1] = 200                                                      # longer than max_prefix
    with pytest.raises(rpo.RpoError) as e:
        rpo.rpo_prefill_prefix(batch, torch.from_numpy(toks).cuda(), bad, torch.empty(2, V, device="cuda"))
    assert e.value.code == rpo.RPO_EINVAL
    rpo.rpo_prefill_prefix(batch, torch.from_numpy(toks).cuda(), cu, torch.empty(2, V, device="cuda"))
    rpo.rpo_kv_fork(batch)
    rpo.rpo_decode_step(batch, tok, 8, None, logits)
    rpo.rpo_decode_step(batch, tok, 8, None, logits)
    with pytest.raises(rpo.RpoError) as e:
        rpo.rpo_decode_step(batch, tok, 8, None, logits)              # beyond max_suffix = 2
    assert e.value.code == rpo.RPO_ESTATE
    torch.cuda.synchronize()


def test_variable_length_rollouts_eos_and_shaped_rewards(rpo):
    """A rollout that samples the end-of-sequence id stops there: same tokens as the unconstrained
    run up to the stop, padding after it, per-rollout lengths, the other rollouts untouched
    (bit-identical logits); the lengths then drive Eq. 11 and Eq. 7."""
    from oracle import reward_shaping as ors
    from paper_2601_19404_amd import rollout
    rpo.rpo_set_kernel_path(0)
    mcfg = synth.TINY
    w = synth.make_weights(mcfg, seed=77)
    model = rpo.rpo_model_create(mcfg, util.to_device(w))
    p, a, m = tiny_workload(ng=3, seed=5)
    order = rollout.order_by_suffix_length(m)
    p, a, m = [p[i] for i in order], [a[i] for i in order], np.asarray(m)[order]
    G, ng = 4, 3
    seq_ids = util.seq_ids_dev(ng * G, base=50)

    def run(eos):
        batch = rpo.rpo_batch_create(model, ng, G, 80, 16, 16, 128)
        res = rollout.suffix_rollout(batch, p, a, m, 1.0, 9, seq_ids, keep_logits=True, eos_id=eos)
        torch.cuda.synchronize()
        return res

    free = run(None)
    ft = free.tokens.cpu().numpy()
    eos = int(ft[5, 3])                                   # rollout 5 (group 1) stops after its 4th token
    res = run(eos)
    tk, ln = res.tokens.cpu().numpy(), res.lengths.cpu().numpy()
    for r in range(ng * G):
        mg = int(m[r // G])
        hit = np.flatnonzero(ft[r, :mg] == eos)
        n = hit[0] + 1 if len(hit) else mg
        assert ln[r] == n
        np.testing.assert_array_equal(tk[r, :n], ft[r, :n])
        assert np.all(tk[r, n:mg] == eos)
    assert ln[5] == 4
    # rows that never stop see bit-identical logits at every step
    never = [r for r in range(ng * G) if ln[r] == m[r // G]]
    assert never
    for j in range(1, int(m.max())):
        rows = [r for r in never if r < res.logits[j].shape[0] and j < m[r // G]]
        if rows:
            np.testing.assert_array_equal(res.logits[j][rows].cpu().numpy(), free.logits[j][rows].cpu().numpy())
    # oracle parity of the stopped rollout: its logits rows up to the stop
    w_np = synth.weights_to_numpy(w)
    shape = util.oracle_shape(mcfg)
    g = 5 // G
    prefix = np.concatenate([p[g], a[g][:64 - int(m[g])]])
    ref = T.teacher_forced_logits(shape, w_np, prefix, tk[5, :4])
    for j in range(4):
        got = res.logits[j][g if j == 0 else 5].cpu().numpy()
        assert np.abs(got - ref[j]).max() < 1e-4
    # lengths -> shaped rewards -> advantages
    rewards = np.ones((ng, G), np.float32)
    shaped = torch.empty(ng, G, dtype=torch.float32, device="cuda")
    rpo.rpo_shape_rewards(torch.from_numpy(rewards).cuda(), res.lengths, ng, G, 0.05, 0.5, 1.0, shaped)
    adv = torch.empty(ng, G, dtype=torch.float32, device="cuda")
    rpo.grpo_advantages(shaped, ng, G, 0, 0.0, adv)
    torch.cuda.synchronize()
    np.testing.assert_allclose(shaped.cpu().numpy(), ors.shape_rewards(rewards, ln.reshape(ng, G), 0.05, 0.5, 1.0),
                               atol=1e-6)
    np.testing.assert_array_equal(adv.cpu().numpy(), oadv.grpo_advantages(shaped.cpu().numpy()))
    assert adv.cpu().numpy()[1, 1] > 0          # the rollout that stopped early is preferred in its group
