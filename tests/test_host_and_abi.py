"""CPU-side checks: the C-ABI library loads and exports every symbol the headers declare,
host-only entry points validate their arguments, and the host logic of the rollout (cut,
pack, ordering, suffix indexing) is right.  No compute call is made (no GPU here)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = set()
    for h in ("rpo.h", "rpo_kernels.h"):
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b((?:rpo|grpo)_[a-z0-9_]+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol():
    from paper_2601_19404_amd import binding
    lib = binding.lib()
    declared = _declared_symbols()
    assert {"rpo_prefill_prefix", "rpo_kv_fork", "rpo_decode_step", "rpo_sample", "rpo_suffix_logprobs",
            "grpo_advantages"} <= declared
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in include/ but not exported"
    assert declared == set(binding.EXPORTS)


def test_host_side_validation_without_a_gpu():
    from paper_2601_19404_amd import binding as b
    lib = b.lib()
    assert lib.rpo_last_error() is not None
    out = C.c_void_p()
    assert lib.rpo_model_create(None, None, C.byref(out)) == b.RPO_EINVAL
    assert b"NULL" in lib.rpo_last_error()
    desc = b.ModelDesc(2, 128, 4, 3, 32, 256, 512, 1e4, 1e-6, b.RPO_F32)       # 4 % 3 != 0
    fake = (C.c_void_p * 2)(1, 1)
    w = b.Weights(1, 1, 1, fake, fake, fake, fake, fake, fake)
    assert lib.rpo_model_create(C.byref(desc), C.byref(w), C.byref(out)) == b.RPO_EINVAL
    desc.n_kv_heads = 2
    assert lib.rpo_model_create(C.byref(desc), C.byref(w), C.byref(out)) == b.RPO_OK
    # sizes: monotone in every argument, zero on nonsense
    kv = lib.rpo_kv_pool_bytes(out, 2, 4, 80, 16, 16)
    assert kv == 2 * (2 * 5 + 8 * 2) * 2 * 2 * 16 * 32 * 4     # layers * pages * (K,V) * heads * tokens * dh * 4 B
    assert lib.rpo_kv_pool_bytes(out, 2, 4, 80, 16, 24) == 0   # page size not a power of two
    assert lib.rpo_workspace_bytes(out, 2, 4, 80, 16, 16, 40) == 0            # max_rows < max_prefix
    ws = lib.rpo_workspace_bytes(out, 2, 4, 80, 16, 16, 128)
    assert ws > 0 and lib.rpo_workspace_bytes(out, 2, 4, 80, 16, 16, 256) > ws
    assert lib.rpo_set_kernel_path(5) == b.RPO_EINVAL and lib.rpo_set_kernel_path(0) == b.RPO_OK
    assert lib.grpo_advantages(None, 1, 1, 0, C.c_float(0.0), None, None) == b.RPO_EINVAL
    lib.rpo_model_destroy(out)


def test_cut_pack_order_and_suffix_index():
    from paper_2601_19404_amd import rollout, synth
    wl = synth.make_workload(synth.C0, n_groups=5)
    order = rollout.order_by_suffix_length(wl.m)
    m = wl.m[order]
    assert np.all(np.diff(m) <= 0) and sorted(order) == list(range(5))
    toks, cu = rollout.cut_and_pack(wl.prompts[order], wl.cached[order], m)
    assert cu[0] == 0 and cu[-1] == len(toks) and toks.dtype == np.int32
    for k in range(5):
        seg = toks[cu[k]:cu[k + 1]]
        assert len(seg) == 16 + 64 - m[k]
        np.testing.assert_array_equal(seg[:16], wl.prompts[order[k]])
        np.testing.assert_array_equal(seg[16:], wl.cached[order[k]][:64 - m[k]])
    with pytest.raises(ValueError):
        rollout.cut_and_pack(wl.prompts[:1], wl.cached[:1], [65])
    idx, cu_s = rollout.suffix_index(m, 3, int(m.max()))
    assert len(cu_s) == 16 and cu_s[-1] == int(m.sum()) * 3 == len(idx)
    mat = np.arange(15 * int(m.max())).reshape(15, -1)
    flat = mat.reshape(-1)[idx]
    for r in range(15):
        np.testing.assert_array_equal(flat[cu_s[r]:cu_s[r + 1]], mat[r, :m[r // 3]])


def test_workload_recipes_match_the_benchmark_description():
    from paper_2601_19404_amd import synth
    for name, lo, hi, ng, g in (("C1", 103, 204, 64, 8), ("C3", 205, 409, 32, 8), ("C0", 8, 16, 2, 4)):
        cfg = synth.CONFIGS[name]
        wl = synth.make_workload(cfg)
        assert wl.m.min() >= lo and wl.m.max() <= hi and wl.prompts.shape == (ng, cfg.prompt_len)
        assert wl.rewards.shape == (ng, g) and set(np.unique(wl.rewards)) <= {0.0, 1.0}
        assert wl.cached.max() < cfg.model.vocab and wl.cached.min() >= 0
    assert synth.QWEN_1P5B.qkv_rows == 2048 and synth.QWEN_7B.qkv_rows == 4608
