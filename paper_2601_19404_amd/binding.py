"""ctypes binding of librpo.so: the same entry points as include/rpo.h and
include/rpo_kernels.h, argument marshalling only.  Device buffers are PyTorch-ROCm
tensors (PyTorch is used for device memory and streams, nothing else); every step
of the path runs in the library's HIP kernels.  There is no fallback: if the
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librpo.so")

RPO_OK, RPO_EINVAL, RPO_ESTATE, RPO_ENOMEM, RPO_EHIP = 0, -1, -2, -3, -4
RPO_F32, RPO_BF16 = 0, 1


class RpoError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"librpo error {code}: {msg}")
        self.code = code


class ModelDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32),
                ("vocab", C.c_int32), ("rope_base", C.c_float), ("rms_eps", C.c_float),
                ("dtype", C.c_int32)]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("wqkv", C.POINTER(C.c_void_p)),
                ("wo", C.POINTER(C.c_void_p)), ("ffn_norm", C.POINTER(C.c_void_p)),
                ("w_gate_up", C.POINTER(C.c_void_p)), ("w_down", C.POINTER(C.c_void_p))]


_lib = None


def lib() -> C.CDLL:
    """Load librpo.so (built in-tree by paper_2601_19404_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2601_19404_amd.build` "
                           "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, u64, u32, f32, sz = (C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_uint32,
                                       C.c_float, C.c_size_t)
    L.rpo_last_error.restype = C.c_char_p
    L.rpo_last_error.argtypes = []
    L.rpo_model_create.argtypes = [C.POINTER(ModelDesc), C.POINTER(Weights), C.POINTER(vp)]
    L.rpo_model_destroy.argtypes = [vp]
    L.rpo_model_destroy.restype = None
    L.rpo_kv_pool_bytes.argtypes = [vp, i32, i32, i32, i32, i32]
    L.rpo_kv_pool_bytes.restype = sz
    L.rpo_workspace_bytes.argtypes = [vp, i32, i32, i32, i32, i32, i32]
    L.rpo_workspace_bytes.restype = sz
    L.rpo_batch_create.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp, sz, vp, sz, vp, C.POINTER(vp)]
    L.rpo_batch_destroy.argtypes = [vp]
    L.rpo_batch_destroy.restype = None
    L.rpo_prefill_prefix.argtypes = [vp, vp, C.POINTER(i32), vp, vp]
    L.rpo_kv_fork.argtypes = [vp, vp]
    L.rpo_decode_step.argtypes = [vp, vp, i32, vp, vp, vp, vp]
    L.rpo_decode_step_compact.argtypes = [vp, vp, i32, vp, vp, vp, vp, C.POINTER(i32), vp]
    L.rpo_sample.argtypes = [vp, i32, i32, i64, vp, i32, f32, u64, vp, u32, vp, vp, i32, vp, vp, vp, vp]
    L.rpo_suffix_logprobs.argtypes = [vp, vp, C.POINTER(i32), f32, vp, vp]
    L.grpo_advantages.argtypes = [vp, i32, i32, i32, f32, vp, vp]
    L.rpo_objective_forward.argtypes = [vp, vp, vp, vp, vp, i32, i32, f32, f32, vp, vp, vp, vp]
    L.rpo_shape_rewards.argtypes = [vp, vp, i32, i32, f32, f32, f32, vp, vp]
    L.rpo_cut_pack.argtypes = [vp, i64, vp, vp, i64, vp, vp, i32, vp, vp]
    L.rpo_cache_update.argtypes = [vp, i64, vp, vp, vp, vp, i64, vp, vp, vp, vp, i32, i32, f32, vp, vp]
    L.rpo_attn_decode.argtypes = [vp, i32, vp, i32, i32, vp, vp, vp]
    L.rpo_gemm_nt.argtypes = [vp, i64, vp, i64, vp, i64, i32, i32, i32, i32, i32, vp, sz, vp]
    L.rpo_gemm_nt_noalloc.argtypes = [vp, i64, vp, i64, vp, i64, i32, i32, i32, i32, i32, vp]
    L.rpo_probe_peaks.argtypes = [vp, vp, sz, vp, C.POINTER(C.c_double), C.POINTER(C.c_double), vp]
    L.rpo_set_kernel_path.argtypes = [C.c_int]
    L.rpo_profile_start.argtypes = [C.c_int, C.c_int]
    L.rpo_profile_stop.argtypes = [C.c_int, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(C.c_double),
                                   C.POINTER(C.c_double)]
    for name in ("rpo_model_create", "rpo_batch_create", "rpo_prefill_prefix", "rpo_kv_fork",
                 "rpo_decode_step", "rpo_decode_step_compact", "rpo_sample", "rpo_suffix_logprobs", "grpo_advantages",
                 "rpo_shape_rewards", "rpo_objective_forward", "rpo_cut_pack", "rpo_cache_update", "rpo_gemm_nt",
                 "rpo_attn_decode", "rpo_gemm_nt_noalloc", "rpo_set_kernel_path", "rpo_profile_start", "rpo_profile_stop", "rpo_probe_peaks"):
        getattr(L, name).restype = C.c_int
    _lib = L
    return L


EXPORTS = ("rpo_model_create", "rpo_model_destroy", "rpo_kv_pool_bytes", "rpo_workspace_bytes",
           "rpo_batch_create", "rpo_batch_destroy", "rpo_prefill_prefix", "rpo_kv_fork",
           "rpo_decode_step", "rpo_decode_step_compact", "rpo_sample", "rpo_suffix_logprobs", "grpo_advantages",
           "rpo_shape_rewards", "rpo_objective_forward", "rpo_cut_pack", "rpo_cache_update", "rpo_last_error", "rpo_gemm_nt", "rpo_attn_decode", "rpo_gemm_nt_noalloc", "rpo_set_kernel_path", "rpo_profile_start",
           "rpo_profile_stop", "rpo_probe_peaks")


def _check(code: int) -> None:
    if code != RPO_OK:
        raise RpoError(code, lib().rpo_last_error().decode())


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream


def _dev(t: torch.Tensor, dtype: torch.dtype, name: str) -> torch.Tensor:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{name}: need a contiguous {dtype} device tensor")
    return t


def _i32_array(values):
    arr = (C.c_int32 * len(values))(*[int(v) for v in values])
    return arr


# ---------------------------------------------------------------------------
class Model:
    """rpo_model handle + references that keep the weight tensors alive."""

    def __init__(self, handle, cfg, weights):
        self.handle, self.cfg, self.weights = handle, cfg, weights

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.rpo_model_destroy(self.handle)
            self.handle = None


def rpo_model_create(cfg, weights: dict) -> Model:
    """cfg: anything with the rpo_model_desc field names (synth.ModelCfg works);
    weights: dict of device tensors laid out as rpo_weights describes."""
    dt = RPO_F32 if cfg.dtype in ("f32", RPO_F32) else RPO_BF16
    tdt = torch.float32 if dt == RPO_F32 else torch.bfloat16
    desc = ModelDesc(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                     cfg.d_ffn, cfg.vocab, cfg.rope_base, cfg.rms_eps, dt)
    n = len(weights["layers"])
    if n != cfg.n_layers:
        raise ValueError("weights['layers'] does not match cfg.n_layers")

    def table(key):
        return (C.c_void_p * n)(*[_dev(lw[key], tdt, key).data_ptr() for lw in weights["layers"]])

    w = Weights(_dev(weights["embed"], tdt, "embed").data_ptr(),
                _dev(weights["lm_head"], tdt, "lm_head").data_ptr(),
                _dev(weights["final_norm"], tdt, "final_norm").data_ptr(),
                table("attn_norm"), table("wqkv"), table("wo"), table("ffn_norm"),
                table("w_gate_up"), table("w_down"))
    out = C.c_void_p()
    _check(lib().rpo_model_create(C.byref(desc), C.byref(w), C.byref(out)))
    return Model(out, cfg, weights)


def rpo_model_destroy(model: Model) -> None:
    model.__del__()


def rpo_kv_pool_bytes(model: Model, n_groups, G, max_prefix, max_suffix, page_tokens) -> int:
    return lib().rpo_kv_pool_bytes(model.handle, n_groups, G, max_prefix, max_suffix, page_tokens)


def rpo_workspace_bytes(model: Model, n_groups, G, max_prefix, max_suffix, page_tokens, max_rows) -> int:
    return lib().rpo_workspace_bytes(model.handle, n_groups, G, max_prefix, max_suffix, page_tokens,
                                     max_rows)


class Batch:
    def __init__(self, handle, model, kv_pool, workspace, dims):
        self.handle, self.model, self.kv_pool, self.workspace = handle, model, kv_pool, workspace
        self.n_groups, self.G, self.max_prefix, self.max_suffix, self.page_tokens, self.max_rows = dims

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.rpo_batch_destroy(self.handle)
            self.handle = None


def rpo_batch_create(model: Model, n_groups, G, max_prefix, max_suffix, page_tokens, max_rows,
                     kv_pool: torch.Tensor | None = None, workspace: torch.Tensor | None = None,
                     stream=None) -> Batch:
    """kv_pool / workspace: uint8 device tensors of at least rpo_kv_pool_bytes /
    rpo_workspace_bytes; allocated here (through PyTorch) when not given."""
    kvb = rpo_kv_pool_bytes(model, n_groups, G, max_prefix, max_suffix, page_tokens)
    wsb = rpo_workspace_bytes(model, n_groups, G, max_prefix, max_suffix, page_tokens, max_rows)
    if kvb == 0 or wsb == 0:
        raise RpoError(RPO_EINVAL, "invalid batch dimensions")
    if kv_pool is None:
        kv_pool = torch.empty(kvb, dtype=torch.uint8, device="cuda")
    if workspace is None:
        workspace = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    out = C.c_void_p()
    _check(lib().rpo_batch_create(model.handle, n_groups, G, max_prefix, max_suffix, page_tokens,
                                  max_rows, kv_pool.data_ptr(), kv_pool.numel(), workspace.data_ptr(),
                                  workspace.numel(), _stream(stream), C.byref(out)))
    return Batch(out, model, kv_pool, workspace,
                 (n_groups, G, max_prefix, max_suffix, page_tokens, max_rows))


def rpo_batch_destroy(batch: Batch) -> None:
    batch.__del__()


def rpo_prefill_prefix(batch: Batch, tokens_dev: torch.Tensor, cu_len_host, last_logits_dev: torch.Tensor,
                       stream=None) -> None:
    _dev(tokens_dev, torch.int32, "tokens_dev")
    _dev(last_logits_dev, torch.float32, "last_logits_dev")
    if len(cu_len_host) != batch.n_groups + 1 or tokens_dev.numel() < int(cu_len_host[-1]):
        raise ValueError("cu_len_host / tokens_dev do not match the batch")
    if last_logits_dev.numel() < batch.n_groups * batch.model.cfg.vocab:
        raise ValueError("last_logits_dev too small")
    _check(lib().rpo_prefill_prefix(batch.handle, tokens_dev.data_ptr(), _i32_array(cu_len_host),
                                    last_logits_dev.data_ptr(), _stream(stream)))


def rpo_kv_fork(batch: Batch, stream=None) -> None:
    _check(lib().rpo_kv_fork(batch.handle, _stream(stream)))


def rpo_decode_step(batch: Batch, tokens_dev: torch.Tensor, n_rows: int, active_dev, logits_dev: torch.Tensor,
                    stream=None, row_max_out_dev=None) -> None:
    if tokens_dev.numel() < n_rows or logits_dev.numel() < n_rows * batch.model.cfg.vocab:
        raise ValueError("tokens_dev / logits_dev smaller than n_rows")
    if row_max_out_dev is not None and (row_max_out_dev.dtype != torch.float32 or row_max_out_dev.numel() < n_rows):
        raise ValueError("row_max_out_dev must be float32 with at least n_rows elements")
    _check(lib().rpo_decode_step(batch.handle, tokens_dev.data_ptr(), n_rows, _ptr(active_dev),
                                 logits_dev.data_ptr(), _ptr(row_max_out_dev), _stream(stream)))


def rpo_decode_step_compact(batch: Batch, tokens_dev: torch.Tensor, n_rows: int, active_dev: torch.Tensor,
                            logits_dev: torch.Tensor, row_of_out_dev: torch.Tensor, stream=None,
                            row_max_out_dev=None) -> int:
    """rpo_decode_step on the live rollouts only; returns the number of logits rows computed."""
    if tokens_dev.numel() < n_rows or logits_dev.numel() < n_rows * batch.model.cfg.vocab:
        raise ValueError("tokens_dev / logits_dev smaller than n_rows")
    if active_dev is None or active_dev.dtype != torch.uint8 or active_dev.numel() < n_rows:
        raise ValueError("active_dev must be uint8 with at least n_rows elements")
    if row_of_out_dev.dtype != torch.int32 or row_of_out_dev.numel() < n_rows:
        raise ValueError("row_of_out_dev must be int32 with at least n_rows elements")
    if row_max_out_dev is not None and (row_max_out_dev.dtype != torch.float32 or row_max_out_dev.numel() < n_rows):
        raise ValueError("row_max_out_dev must be float32 with at least n_rows elements")
    n = C.c_int32(0)
    _check(lib().rpo_decode_step_compact(batch.handle, tokens_dev.data_ptr(), n_rows, active_dev.data_ptr(),
                                         logits_dev.data_ptr(), _ptr(row_max_out_dev), row_of_out_dev.data_ptr(),
                                         C.byref(n), _stream(stream)))
    return n.value


def rpo_sample(logits_dev: torch.Tensor, n_logit_rows: int, vocab: int, row_stride: int, row_map_dev,
               n_out_rows: int, temperature: float, seed: int, seq_id_dev: torch.Tensor, step: int,
               tokens_out_dev: torch.Tensor, logprob_out_dev=None, stream=None, eos_id: int = -1,
               active_inout_dev=None, lengths_inout_dev=None, row_max_dev=None) -> None:
    if logits_dev.dtype != torch.float32 or tokens_out_dev.dtype != torch.int32:
        raise ValueError("logits must be float32, tokens int32")
    if row_max_dev is not None and (row_max_dev.dtype != torch.float32 or row_max_dev.numel() < n_logit_rows):
        raise ValueError("row_max_dev must be float32 with at least n_logit_rows elements")
    if logits_dev.numel() < (n_logit_rows - 1) * row_stride + vocab:
        raise ValueError("logits_dev smaller than n_logit_rows x row_stride")
    if seq_id_dev.numel() < n_out_rows or tokens_out_dev.numel() < n_out_rows:
        raise ValueError("seq_id_dev / tokens_out_dev smaller than n_out_rows")
    _check(lib().rpo_sample(logits_dev.data_ptr(), n_logit_rows, vocab, row_stride, _ptr(row_map_dev),
                            n_out_rows, temperature, seed, seq_id_dev.data_ptr(), step,
                            tokens_out_dev.data_ptr(), _ptr(logprob_out_dev), eos_id, _ptr(active_inout_dev),
                            _ptr(lengths_inout_dev), _ptr(row_max_dev), _stream(stream)))


def rpo_suffix_logprobs(batch: Batch, suffix_tokens_dev: torch.Tensor, cu_suffix_host, temperature: float,
                        logprobs_out_dev: torch.Tensor, stream=None) -> None:
    _dev(suffix_tokens_dev, torch.int32, "suffix_tokens_dev")
    _dev(logprobs_out_dev, torch.float32, "logprobs_out_dev")
    n = int(cu_suffix_host[-1])
    if len(cu_suffix_host) != batch.n_groups * batch.G + 1 or suffix_tokens_dev.numel() < n \
            or logprobs_out_dev.numel() < n:
        raise ValueError("cu_suffix_host / buffers do not match the batch")
    _check(lib().rpo_suffix_logprobs(batch.handle, suffix_tokens_dev.data_ptr(), _i32_array(cu_suffix_host),
                                     temperature, logprobs_out_dev.data_ptr(), _stream(stream)))


def grpo_advantages(rewards_dev: torch.Tensor, n_groups: int, G: int, ddof: int, eps: float,
                    adv_out_dev: torch.Tensor, stream=None) -> None:
    _dev(rewards_dev, torch.float32, "rewards_dev")
    _dev(adv_out_dev, torch.float32, "adv_out_dev")
    if rewards_dev.numel() < n_groups * G or adv_out_dev.numel() < n_groups * G:
        raise ValueError("rewards / advantages smaller than n_groups x G")
    _check(lib().grpo_advantages(rewards_dev.data_ptr(), n_groups, G, ddof, eps, adv_out_dev.data_ptr(),
                                 _stream(stream)))


def rpo_objective_forward(lp_new_dev, lp_old_dev, lp_ref_dev, cu_suffix_dev, adv_dev, n_groups: int, G: int,
                          eps_clip: float, beta: float, token_out_dev, group_out_dev, stream=None) -> None:
    for t, nm in ((lp_new_dev, "lp_new_dev"), (lp_old_dev, "lp_old_dev"), (adv_dev, "adv_dev"),
                  (group_out_dev, "group_out_dev")):
        _dev(t, torch.float32, nm)
    _dev(cu_suffix_dev, torch.int32, "cu_suffix_dev")
    if cu_suffix_dev.numel() < n_groups * G + 1 or adv_dev.numel() < n_groups * G or group_out_dev.numel() < n_groups:
        raise ValueError("buffers do not match n_groups x G")
    scratch = torch.empty(max(n_groups * G, 1), dtype=torch.float64, device=lp_new_dev.device)
    _check(lib().rpo_objective_forward(lp_new_dev.data_ptr(), lp_old_dev.data_ptr(), _ptr(lp_ref_dev),
                                       cu_suffix_dev.data_ptr(), adv_dev.data_ptr(), n_groups, G, eps_clip, beta,
                                       _ptr(token_out_dev), scratch.data_ptr(), group_out_dev.data_ptr(),
                                       _stream(stream)))


def rpo_shape_rewards(rewards_dev: torch.Tensor, lengths_dev: torch.Tensor, n_groups: int, G: int,
                      alpha: float, lo: float, hi: float, shaped_out_dev: torch.Tensor, stream=None) -> None:
    _dev(rewards_dev, torch.float32, "rewards_dev")
    _dev(lengths_dev, torch.int32, "lengths_dev")
    _dev(shaped_out_dev, torch.float32, "shaped_out_dev")
    if min(rewards_dev.numel(), lengths_dev.numel(), shaped_out_dev.numel()) < n_groups * G:
        raise ValueError("buffers smaller than n_groups x G")
    _check(lib().rpo_shape_rewards(rewards_dev.data_ptr(), lengths_dev.data_ptr(), n_groups, G, alpha, lo, hi,
                                   shaped_out_dev.data_ptr(), _stream(stream)))


def rpo_cut_pack(prompts_dev: torch.Tensor, prompt_len_dev: torch.Tensor, pool_dev: torch.Tensor,
                 question_dev, cu_len_dev: torch.Tensor, n_groups: int, tokens_out_dev: torch.Tensor,
                 stream=None) -> None:
    for t, nm in ((prompts_dev, "prompts_dev"), (prompt_len_dev, "prompt_len_dev"), (pool_dev, "pool_dev"),
                  (cu_len_dev, "cu_len_dev"), (tokens_out_dev, "tokens_out_dev")):
        _dev(t, torch.int32, nm)
    if prompts_dev.dim() != 2 or pool_dev.dim() != 2 or cu_len_dev.numel() < n_groups + 1:
        raise ValueError("prompts / pool must be 2-D, cu_len_dev [n_groups + 1]")
    if question_dev is not None and (question_dev.dtype != torch.int32 or question_dev.numel() < n_groups):
        raise ValueError("question_dev must be int32 [n_groups]")
    _check(lib().rpo_cut_pack(prompts_dev.data_ptr(), prompts_dev.stride(0), prompt_len_dev.data_ptr(),
                              pool_dev.data_ptr(), pool_dev.stride(0), _ptr(question_dev), cu_len_dev.data_ptr(),
                              n_groups, tokens_out_dev.data_ptr(), _stream(stream)))


def rpo_cache_update(pool_dev: torch.Tensor, answer_len_dev: torch.Tensor, question_dev, m_dev: torch.Tensor,
                     tokens_dev: torch.Tensor, lengths_dev, rewards_dev: torch.Tensor, u_dev: torch.Tensor,
                     g_prime_dev: torch.Tensor, n_groups: int, G: int, eps: float, chosen_out_dev=None,
                     stream=None) -> None:
    for t, nm in ((pool_dev, "pool_dev"), (answer_len_dev, "answer_len_dev"), (m_dev, "m_dev"),
                  (g_prime_dev, "g_prime_dev")):
        _dev(t, torch.int32, nm)
    _dev(rewards_dev, torch.float32, "rewards_dev")
    _dev(u_dev, torch.float32, "u_dev")
    if tokens_dev.dtype != torch.int32 or tokens_dev.dim() != 2 or tokens_dev.stride(1) != 1 or not tokens_dev.is_cuda:
        raise ValueError("tokens_dev: need a 2-D int32 device tensor with unit column stride")
    if tokens_dev.shape[0] < n_groups * G or rewards_dev.numel() < n_groups * G or pool_dev.dim() != 2 \
            or min(m_dev.numel(), u_dev.numel(), g_prime_dev.numel()) < n_groups:
        raise ValueError("buffers do not match n_groups x G")
    _check(lib().rpo_cache_update(pool_dev.data_ptr(), pool_dev.stride(0), answer_len_dev.data_ptr(),
                                  _ptr(question_dev), m_dev.data_ptr(), tokens_dev.data_ptr(), tokens_dev.stride(0),
                                  _ptr(lengths_dev), rewards_dev.data_ptr(), u_dev.data_ptr(), g_prime_dev.data_ptr(),
                                  n_groups, G, eps, _ptr(chosen_out_dev), _stream(stream)))


def rpo_gemm_nt(a_dev: torch.Tensor, w_dev: torch.Tensor, c_dev: torch.Tensor, epilogue: int,
                ws_dev: torch.Tensor | None = None, stream=None) -> None:
    """C (op)= A W^T for 2-D tensors (row strides taken from the tensors); epilogue 3 is the
    fused SwiGLU (C is [M, N/2]).  ws_dev: optional uint8 scratch for K-split partial sums."""
    M, K = a_dev.shape
    N, K2 = w_dev.shape
    n_out = N // 2 if epilogue == 3 else N
    if K != K2 or tuple(c_dev.shape) != (M, n_out) or a_dev.stride(1) != 1 or w_dev.stride(1) != 1 \
            or c_dev.stride(1) != 1:
        raise ValueError("shape / stride mismatch")
    dt = RPO_F32 if a_dev.dtype == torch.float32 else RPO_BF16
    _check(lib().rpo_gemm_nt(a_dev.data_ptr(), a_dev.stride(0), w_dev.data_ptr(), w_dev.stride(0),
                             c_dev.data_ptr(), c_dev.stride(0), M, N, K, dt, epilogue, _ptr(ws_dev),
                             0 if ws_dev is None else ws_dev.numel(), _stream(stream)))


def rpo_attn_decode(batch: Batch, layer: int, q_dev: torch.Tensor, n_rows: int, n_suffix: int, active_dev,
                    out_dev: torch.Tensor, stream=None) -> None:
    """One layer's shared-prefix decode attention on caller-given (rotated) queries."""
    cfg = batch.model.cfg
    width = cfg.n_q_heads * cfg.head_dim
    tdt = torch.float32 if cfg.dtype in ("f32", RPO_F32) else torch.bfloat16
    _dev(q_dev, tdt, "q_dev")
    _dev(out_dev, tdt, "out_dev")
    if q_dev.numel() < n_rows * width or out_dev.numel() < n_rows * width:
        raise ValueError("q_dev / out_dev smaller than n_rows x n_q_heads x head_dim")
    _check(lib().rpo_attn_decode(batch.handle, layer, q_dev.data_ptr(), n_rows, n_suffix, _ptr(active_dev),
                                 out_dev.data_ptr(), _stream(stream)))


def rpo_gemm_nt_noalloc(a_dev: torch.Tensor, w_dev: torch.Tensor, c_dev: torch.Tensor, epilogue: int,
                        stream=None) -> None:
    """rpo_gemm_nt with the library's own fixed scratch for K-split partial sums (no workspace
    argument, nothing allocated)."""
    M, K = a_dev.shape
    N, K2 = w_dev.shape
    n_out = N // 2 if epilogue == 3 else N
    if K != K2 or tuple(c_dev.shape) != (M, n_out) or a_dev.stride(1) != 1 or w_dev.stride(1) != 1 \
            or c_dev.stride(1) != 1:
        raise ValueError("shape / stride mismatch")
    dt = RPO_F32 if a_dev.dtype == torch.float32 else RPO_BF16
    _check(lib().rpo_gemm_nt_noalloc(a_dev.data_ptr(), a_dev.stride(0), w_dev.data_ptr(), w_dev.stride(0),
                                     c_dev.data_ptr(), c_dev.stride(0), M, N, K, dt, epilogue, _stream(stream)))


def rpo_set_kernel_path(path: int) -> None:
    _check(lib().rpo_set_kernel_path(path))


def rpo_last_error() -> str:
    return lib().rpo_last_error().decode()


def rpo_probe_peaks(n_bytes: int = 1 << 30, stream=None):
    """(copy GB/s counting read + write, bf16 MFMA issue-loop TFLOP/s) of the current GPU."""
    src = torch.ones(n_bytes // 4, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    scratch = torch.empty(512 * 256, dtype=torch.float32, device="cuda")
    gbps, tflops = C.c_double(0.0), C.c_double(0.0)
    _check(lib().rpo_probe_peaks(_ptr(src), _ptr(dst), C.c_size_t(n_bytes), _ptr(scratch), C.byref(gbps),
                                 C.byref(tflops), _stream(stream)))
    return gbps.value, tflops.value


KERNEL_IDS = {"gemm256": 1, "gemm128": 3, "gemm64": 4, "gemm32": 5, "gemm64x64": 6,
              "gemm_generic": 7, "gemm256x192": 11, "attn_decode": 8, "attn_chunk": 9, "sample": 10,
              "gemm256_swiglu": 12, "gemm256x160": 13}


def rpo_profile_start(kernel_id: int, every: int = 1) -> None:
    """Bracket every `every`-th launch of the kernel with HIP events until rpo_profile_stop."""
    _check(lib().rpo_profile_start(kernel_id, every))


def rpo_profile_stop(kernel_id: int):
    """-> (launches, total_ms, total_flops, total_bytes) of the bracketed launches of that kernel."""
    n, ms, fl, by = C.c_int64(), C.c_double(), C.c_double(), C.c_double()
    _check(lib().rpo_profile_stop(kernel_id, C.byref(n), C.byref(ms), C.byref(fl), C.byref(by)))
    return n.value, ms.value, fl.value, by.value
