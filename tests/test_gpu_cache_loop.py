"""The loop RPO closes (Algorithm 1): rollout -> rewards -> epsilon-greedy cache update (Sec. 3.3,
Eq. 10) -> the next rollout conditions on what the first one produced.  The pool lives on the
device (rpo_cut_pack / rpo_cache_update); the oracle keeps its own host pool, is fed the tokens
the GPU sampled, and must end up with the same pool (integers: bit-exact), the same prefixes for
step 2, and -- teacher-forced on step 2's tokens -- the same logits within the float tolerance."""
import numpy as np
import pytest
import torch

from oracle import cache_update as ocu
from oracle import rollout as orollout
from oracle import transformer as T
from paper_2601_19404_amd import synth
from tests import util

pytestmark = pytest.mark.gpu

BF16_SMALL = synth.ModelCfg("bf16-small", 2, 768, 6, 1, 128, 1024, 2048, "bf16")


@pytest.mark.parametrize("mcfg,page,tol", [(synth.TINY, 16, 1e-4), (BF16_SMALL, 64, 2e-2)])
def test_two_rollout_steps_through_the_device_cache(mcfg, page, tol):
    from paper_2601_19404_amd import binding as rpo
    from paper_2601_19404_amd import cache, rollout
    rpo.lib()
    rpo.rpo_set_kernel_path(0)
    n, G, P, Ta, eps = 5, 4, 16, 96, 0.1
    rng = np.random.default_rng(17)
    prompts = rng.integers(0, mcfg.vocab, size=(n, P)).astype(np.int32)
    answers = rng.integers(0, mcfg.vocab, size=(n, Ta)).astype(np.int32)
    w = synth.perturb_gains(synth.make_weights(mcfg, seed=5))
    w_np = synth.weights_to_numpy(w)
    shape = util.oracle_shape(mcfg)
    model = rpo.rpo_model_create(mcfg, util.to_device(w))
    batch = rpo.rpo_batch_create(model, n, G, P + Ta, 24, page, 1024)
    pool = cache.DeviceCachePool(prompts, answers)
    host_pool = answers.copy()                                  # the oracle's pool
    seq_ids = util.seq_ids_dev(n * G, base=7)
    sid = np.arange(7, 7 + n * G).astype(np.uint64)
    for step in range(2):
        m_q = rng.integers(0 if step else 3, 25, size=n).astype(np.int32)   # step 2 may draw m = 0
        order = rollout.order_by_suffix_length(m_q)
        m = m_q[order]
        toks_dev, cu = pool.cut_pack(m, order)
        # the cut: q_k || a_k[0:-m_k] of the oracle's pool, group by group
        ref_prefix = [orollout.cut(prompts[q], host_pool[q], int(mk)) for q, mk in zip(order, m)]
        np.testing.assert_array_equal(toks_dev.cpu().numpy(), np.concatenate(ref_prefix))
        np.testing.assert_array_equal(np.diff(cu), [len(x) for x in ref_prefix])
        res = rollout.suffix_rollout(batch, None, None, m, 0.9, 100 + step, seq_ids, keep_logits=True,
                                     prefix=(toks_dev, cu))
        torch.cuda.synchronize()
        toks = res.tokens.cpu().numpy()
        # logits of this step against the oracle conditioned on ITS pool (step 2: the updated one)
        worst = 0.0
        for k in range(n):
            for i in (0, G - 1):
                r, mk = k * G + i, int(m[k])
                if mk == 0:
                    continue
                ref = T.teacher_forced_logits(shape, w_np, ref_prefix[k], toks[r, :mk])
                got = np.stack([res.logits[j][k if j == 0 else r].cpu().numpy() for j in range(mk)])
                worst = max(worst, float(np.abs(got - ref).max()))
        assert worst < tol, f"step {step}: logits differ from the oracle by {worst}"
        # rewards and random numbers of the update rule are inputs; u is an fp32 value on both sides
        rewards = (rng.random((n, G)) < 0.5).astype(np.float32)
        u = rng.random(n).astype(np.float32)
        u[0] = np.float32(eps)                                   # the boundary: u == eps is greedy
        gp = rng.integers(0, G, size=n).astype(np.int32)
        chosen = pool.update(m, order, res.tokens, torch.from_numpy(rewards).cuda(), u, gp, eps)
        torch.cuda.synchronize()
        # oracle update in batch order on the batch-ordered view of its pool, scattered back
        new_rows, chosen_ref = ocu.update_pool(host_pool[order], m, toks, rewards, u.astype(np.float64), gp,
                                               float(np.float32(eps)))
        host_pool[order] = new_rows
        np.testing.assert_array_equal(chosen.cpu().numpy(), chosen_ref)
        np.testing.assert_array_equal(pool.answers.cpu().numpy(), host_pool)
        np.testing.assert_array_equal(pool.answer_len.cpu().numpy(), np.full(n, Ta))
    assert not np.array_equal(host_pool, answers)               # the loop really changed the cache


def test_cache_update_variable_lengths_and_misfits():
    """Responses that stopped early (lengths from rpo_sample) shorten the cached answer; a cut longer
    than the answer or a response that does not fit the pool row leaves the entry alone and reports -1."""
    from paper_2601_19404_amd import binding as rpo
    rpo.lib()
    n, G, stride = 4, 3, 20
    rng = np.random.default_rng(3)
    pool0 = rng.integers(0, 1000, size=(n, stride)).astype(np.int32)
    alen = np.array([20, 12, 5, 18], np.int32)
    m = np.array([6, 4, 9, 4], np.int32)                        # question 2: cut 9 > length 5
    tokens = rng.integers(1000, 2000, size=(n * G, 8)).astype(np.int32)
    lengths = np.array([6, 2, 6, 4, 4, 1, 3, 3, 3, 4, 7, 4], np.int32)   # question 3, rollout 1: 14 + 7 > 20
    rewards = np.array([[0, 1, 1], [1, 0, 0], [0, 0, 1], [0, 0, 0]], np.float32)
    u = np.array([0.05, 0.5, 0.05, 0.9], np.float32)
    gp = np.array([2, 2, 0, 1], np.int32)
    dev = lambda a: torch.from_numpy(a).cuda()
    pool_d, alen_d, chosen_d = dev(pool0.copy()), dev(alen.copy()), torch.empty(n, dtype=torch.int32, device="cuda")
    rpo.rpo_cache_update(pool_d, alen_d, None, dev(m), dev(tokens), dev(lengths), dev(rewards), dev(u), dev(gp),
                         n, G, 0.1, chosen_d)
    torch.cuda.synchronize()
    picks = [ocu.select_response(rewards[k], float(u[k]), int(gp[k]), float(np.float32(0.1))) for k in range(n)]
    assert picks == [1, 2, 2, 1]
    exp_pool, exp_len, exp_chosen = pool0.copy(), alen.copy(), []
    for k in range(n):
        ln, keep = int(lengths[k * G + picks[k]]), int(alen[k] - m[k])
        if keep < 0 or keep + ln > stride:
            exp_chosen.append(-1)
            continue
        exp_pool[k, keep:keep + ln] = tokens[k * G + picks[k], :ln]
        exp_len[k] = keep + ln
        exp_chosen.append(picks[k])
    assert exp_chosen == [1, 2, -1, -1]
    np.testing.assert_array_equal(chosen_d.cpu().numpy(), exp_chosen)
    np.testing.assert_array_equal(pool_d.cpu().numpy(), exp_pool)
    np.testing.assert_array_equal(alen_d.cpu().numpy(), exp_len)
