"""Pins for oracle/rollout.py: structure of the RPO rollout (paper Eq. 3) and the
token accounting behind the paper's Table 2."""
import numpy as np

from oracle import rollout, sampler
from oracle import transformer as T
from paper_2601_19404_amd import synth
from tests.test_oracle_transformer import tiny_shape


def _tiny():
    w = synth.weights_to_numpy(synth.make_weights(synth.TINY, seed=1234))
    return tiny_shape(), w


def test_cut_keeps_prompt_and_drops_last_m():
    p = np.arange(5)
    a = 100 + np.arange(10)
    np.testing.assert_array_equal(rollout.cut(p, a, 3), np.concatenate([p, a[:7]]))
    np.testing.assert_array_equal(rollout.cut(p, a, 0), np.concatenate([p, a]))
    np.testing.assert_array_equal(rollout.cut(p, a, 10), p)


def test_rollout_is_ancestral_sampling_from_the_conditional():
    shape, w = _tiny()
    wl = synth.make_workload(synth.C0)
    m = int(wl.m[0])
    out = rollout.suffix_rollout(shape, w, wl.prompts[0], wl.cached[0], m, 4, 1.0, 3,
                                 wl.seq_ids[:4])
    assert out["tokens"].shape == (4, m)
    prefix = out["prefix"]
    assert len(prefix) == 16 + 64 - m
    # all rollouts of a group see the same first-row logits (shared prefix) ...
    for i in range(1, 4):
        np.testing.assert_array_equal(out["logits"][0, 0], out["logits"][i, 0])
    # ... but draw independently
    assert len({tuple(t) for t in out["tokens"]}) > 1
    # every later logits row is the conditional given prefix || own tokens so far
    for i in range(4):
        full = T.logits_full(shape, w, np.concatenate([prefix, out["tokens"][i]]))
        s = len(prefix)
        np.testing.assert_allclose(out["logits"][i].astype(np.float64), full[s - 1:s - 1 + m],
                                   atol=1e-6)
        # teacher-forced log-probs reproduce what the sampler saw (ratio == 1 for one policy)
        lp = T.suffix_logprobs(shape, w, prefix, out["tokens"][i], 1.0)
        np.testing.assert_allclose(lp, out["logprobs"][i], atol=1e-5)
        # and each token is what the sampler returns for that row, seq id and step
        for j in range(m):
            assert sampler.sample_row(out["logits"][i, j], 1.0, 3, int(wl.seq_ids[i]), j)[0] \
                == out["tokens"][i, j]


def test_token_reduction_accounting():
    """Table 2 of the paper: with L = 300 the rollout generates 145.88 (1.5B) /
    147.06 (7B) tokens per sample against 2689.51 / 2457.91 for full paths --
    m ~ U{0..L} has mean L/2 = 150, i.e. ~5.4-6 % of the tokens.  The benchmark's
    cut (last 5-10 % of a 2048-token answer) must land in the same regime."""
    assert abs(np.mean(np.arange(0, 301)) - 150.0) < 1e-12
    assert abs(145.88 / 150.0 - 1) < 0.03 and abs(147.06 / 150.0 - 1) < 0.03
    wl = synth.make_workload(synth.C1)
    assert wl.m.min() >= 103 and wl.m.max() <= 204
    frac = wl.m.mean() / synth.C1.traj_len
    assert 0.05 <= frac <= 0.10
    paper_frac = 145.88 / 2689.51
    assert 0.04 < paper_frac < 0.07


def test_rollout_stops_at_end_of_sequence():
    shape, w = _tiny()
    wl = synth.make_workload(synth.C0)
    m = int(wl.m[0])
    free = rollout.suffix_rollout(shape, w, wl.prompts[0], wl.cached[0], m, 4, 1.0, 3, wl.seq_ids[:4])
    eos = int(free["tokens"][1, 2])                     # rollout 1 will hit it at step 2
    out = rollout.suffix_rollout(shape, w, wl.prompts[0], wl.cached[0], m, 4, 1.0, 3, wl.seq_ids[:4], eos_id=eos)
    assert out["lengths"][1] == 3
    for i in range(4):
        n = int(out["lengths"][i])
        np.testing.assert_array_equal(out["tokens"][i, :n], free["tokens"][i, :n])   # same draws until the stop
        assert np.all(out["tokens"][i, n:] == eos)
        hit = np.flatnonzero(free["tokens"][i] == eos)
        assert n == (hit[0] + 1 if len(hit) else m)
