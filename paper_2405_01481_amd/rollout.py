"""Thin ctypes binding of librollout.so (include/rollout.h): argument marshalling only.

Every step of generation and scoring runs inside the library's HIP kernels.  PyTorch
appears here only as the owner of device memory and streams.  There is no CPU
fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librollout.so")

RL_OK, RL_EINVAL, RL_ENOMEM_PAGES, RL_ESTATE, RL_EHIP, RL_ENOSPACE = 0, -1, -2, -3, -4, -5
RL_FP32, RL_BF16 = 0, 1
RL_K_GEMM_DECODE, RL_K_ATTN_DECODE, RL_K_GEMM_PREFILL, RL_K_ATTN_PREFILL, RL_K_LMHEAD_SCORE = range(5)


class RolloutError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"librollout error {code}: {msg}")
        self.code = code


class rl_model_cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + \
               [("rope_base", C.c_float), ("rms_eps", C.c_float), ("dtype", C.c_int32), ("max_batch", C.c_int32),
                ("max_seq", C.c_int32), ("page_tokens", C.c_int32), ("max_chunk_tokens", C.c_int32),
                ("n_pages", C.c_int64)]


class rl_weights(C.Structure):
    _fields_ = [("tok_embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")] + \
               [("location", C.c_int32), ("staging", C.c_void_p), ("staging_bytes", C.c_size_t),
                ("fp16_copy", C.c_void_p), ("fp16_copy_bytes", C.c_size_t)]


class rl_sample_cfg(C.Structure):
    _fields_ = [("seed", C.c_uint64), ("temperature", C.c_float), ("eos_id", C.c_int32), ("seq_id_base", C.c_int64)]


_lib = None


def lib():
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RolloutError(RL_EINVAL, f"{LIB_PATH} not built (run python -m paper_2405_01481_amd.build)")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
        L.rollout_last_error.restype = C.c_char_p
        L.rollout_workspace_bytes.restype = C.c_size_t
        L.rollout_workspace_bytes.argtypes = [C.POINTER(rl_model_cfg)]
        L.rollout_kv_pool_bytes.restype = C.c_size_t
        L.rollout_kv_pool_bytes.argtypes = [C.POINTER(rl_model_cfg)]
        L.rollout_weight_shadow_bytes.restype = C.c_size_t
        L.rollout_weight_shadow_bytes.argtypes = [C.POINTER(rl_model_cfg)]
        L.rollout_refresh_policy.argtypes = [vp, vp]
        L.rollout_weight_resident_bytes.restype = C.c_size_t
        L.rollout_weight_resident_bytes.argtypes = [C.POINTER(rl_model_cfg)]
        L.rollout_weight_staging_bytes.restype = C.c_size_t
        L.rollout_weight_staging_bytes.argtypes = [C.POINTER(rl_model_cfg)]
        L.rollout_init.argtypes = [C.POINTER(rl_model_cfg), C.POINTER(rl_weights), vp, C.c_size_t, vp, C.c_size_t,
                                   C.POINTER(vp)]
        L.rollout_prefill.argtypes = [vp, vp, vp, i32, i32, vp]
        L.rollout_decode_step.argtypes = [vp, C.POINTER(rl_sample_cfg), vp, vp, vp, vp]
        L.rollout_generate.argtypes = [vp, C.POINTER(rl_sample_cfg), vp, vp, i32, i32, i32, vp, vp, vp, vp]
        L.rollout_generate_queue.argtypes = [vp, C.POINTER(rl_sample_cfg), vp, vp, vp, i32, i32, i32, vp, vp, vp, vp]
        L.score_logprobs_kl.argtypes = [vp, C.POINTER(rl_weights), C.POINTER(rl_weights), vp, vp, vp, i32, i32, f32,
                                        vp, vp, vp, vp, vp]
        L.rollout_check.argtypes = [vp, vp]
        L.score_kl_exact.argtypes = [vp, C.POINTER(rl_weights), C.POINTER(rl_weights), vp, vp, vp, i32, i32, vp, vp]
        L.score_values.argtypes = [vp, C.POINTER(rl_weights), vp, vp, vp, i32, i32, vp, vp]
        L.ppo_rewards.argtypes = [vp, vp, vp, vp, vp, i32, i32, f32, vp, vp]
        L.ppo_rewards_noalloc.argtypes = [vp, vp, vp, vp, i32, i32, f32, vp, vp]
        L.rollout_set_policy.argtypes = [vp, C.POINTER(rl_weights)]
        L.rollout_reset.argtypes = [vp]
        L.rollout_destroy.argtypes = [vp]
        L.rollout_destroy.restype = None
        L.rollout_set_impl.argtypes = [vp, i32]
        L.rollout_set_decode_tile_rows.argtypes = [i32]
        L.rollout_set_large_gemm_copy.argtypes = [i32]
        L.rollout_set_precise_layers.argtypes = [vp, i32]
        L.rollout_set_fused_sampling.argtypes = [vp, i32]
        L.rollout_set_fused_qkv_consumer.argtypes = [vp, i32]
        L.rollout_forget_fp16_copies.argtypes = [vp]
        L.rollout_profile_enable.argtypes = [vp, i32, i32]
        L.rollout_profile_read.argtypes = [vp, i32, C.POINTER(C.c_double), C.POINTER(i64)]
        L.rollout_profile_event_overhead.argtypes = [vp, i32, C.POINTER(C.c_double), vp]
        L.rollout_probe_mfma_rate.argtypes = [vp, i32, C.POINTER(C.c_double), vp]
        _lib = L
    return _lib


def _chk(rc):
    if rc != 0:
        raise RolloutError(rc, lib().rollout_last_error().decode())


def rollout_last_error() -> str:
    return lib().rollout_last_error().decode()


def make_cfg(shape, max_batch, max_seq, n_pages=None, max_chunk_tokens=None) -> rl_model_cfg:
    pt = shape.page_tokens
    if n_pages is None:
        n_pages = max_batch * ((max_seq + pt - 1) // pt)
    if max_chunk_tokens is None:
        max_chunk_tokens = max(max_seq, min(max_batch * max_seq, 16384))
    return rl_model_cfg(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                        shape.vocab, shape.rope_base, shape.rms_eps, RL_FP32 if shape.dtype == "fp32" else RL_BF16,
                        max_batch, max_seq, pt, max_chunk_tokens, n_pages)


def rollout_workspace_bytes(cfg: rl_model_cfg) -> int:
    return int(lib().rollout_workspace_bytes(C.byref(cfg)))


def rollout_kv_pool_bytes(cfg: rl_model_cfg) -> int:
    return int(lib().rollout_kv_pool_bytes(C.byref(cfg)))


def rollout_weight_shadow_bytes(cfg: rl_model_cfg) -> int:
    return int(lib().rollout_weight_shadow_bytes(C.byref(cfg)))


def rollout_weight_resident_bytes(cfg: rl_model_cfg) -> int:
    return int(lib().rollout_weight_resident_bytes(C.byref(cfg)))


def rollout_weight_staging_bytes(cfg: rl_model_cfg) -> int:
    return int(lib().rollout_weight_staging_bytes(C.byref(cfg)))


class Weights:
    """Marshals a dict of torch tensors (layout of the input generator) into rl_weights; keeps them alive.
    With `staging` (a device uint8 tensor of rollout_weight_staging_bytes) the tensors are taken to be host
    memory and the set is marked location 1 (streamed during scoring)."""

    _LAYER = ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")

    def __init__(self, w, staging=None, shadow=None):
        self.tensors = w
        self.staging = staging
        self.shadow = shadow
        n = len(w["layers"])
        self._arrays = {}
        s = rl_weights()
        for k in ("tok_embed", "final_norm", "lm_head"):
            assert w[k].is_contiguous()
            setattr(s, k, w[k].data_ptr())
        for k in self._LAYER:
            arr = (C.c_void_p * n)()
            for l in range(n):
                t = w["layers"][l][k]
                assert t.is_contiguous()
                arr[l] = t.data_ptr()
            self._arrays[k] = arr
            setattr(s, k, C.cast(arr, C.POINTER(C.c_void_p)))
        s.location = 0
        if staging is not None:
            assert staging.is_cuda and all(not w[k].is_cuda for k in ("tok_embed", "final_norm", "lm_head"))
            s.location = 1
            s.staging = staging.data_ptr()
            s.staging_bytes = staging.numel() * staging.element_size()
        if shadow is not None:
            # a policy with a buffer for the library's fp16 copy (rollout_weight_shadow_bytes)
            assert shadow.is_cuda
            s.fp16_copy = shadow.data_ptr()
            s.fp16_copy_bytes = shadow.numel() * shadow.element_size()
        self.struct = s


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _host_i32(a):
    a = np.ascontiguousarray(np.asarray(a, dtype=np.int32))
    return a, a.ctypes.data_as(C.c_void_p)


class Rollout:
    """A context plus the device buffers it borrows.  Methods carry the C ABI's names."""

    def __init__(self, cfg: rl_model_cfg, policy: Weights, device="cuda:0"):
        self.cfg = cfg
        self.policy = policy
        self.device = torch.device(device)
        wsb, kvb = rollout_workspace_bytes(cfg), rollout_kv_pool_bytes(cfg)
        if wsb == 0:
            raise RolloutError(RL_EINVAL, rollout_last_error())
        self.workspace = torch.empty(wsb, dtype=torch.uint8, device=self.device)
        self.kv_pool = torch.zeros(kvb, dtype=torch.uint8, device=self.device)
        h = C.c_void_p()
        torch.cuda.synchronize()
        _chk(lib().rollout_init(C.byref(cfg), C.byref(policy.struct), _ptr(self.workspace), wsb, _ptr(self.kv_pool),
                                kvb, C.byref(h)))
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            torch.cuda.synchronize()
            lib().rollout_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the C ABI, one method per entry point
    def rollout_prefill(self, prompt_ids: torch.Tensor, prompt_len):
        pl, plp = _host_i32(prompt_len)
        B, Pmax = prompt_ids.shape
        _chk(lib().rollout_prefill(self.h, _ptr(prompt_ids), plp, B, Pmax, _stream()))

    def rollout_decode_step(self, sample: rl_sample_cfg, tok_in=None, tok_out=None, logp_out=None):
        _chk(lib().rollout_decode_step(self.h, C.byref(sample), _ptr(tok_in), _ptr(tok_out), _ptr(logp_out), _stream()))

    def rollout_generate(self, sample: rl_sample_cfg, prompt_ids: torch.Tensor, prompt_len, G, out_ids, out_len=None,
                         out_logp=None):
        pl, plp = _host_i32(prompt_len)
        B, Pmax = prompt_ids.shape
        _chk(lib().rollout_generate(self.h, C.byref(sample), _ptr(prompt_ids), plp, B, Pmax, G, _ptr(out_ids),
                                    _ptr(out_len), _ptr(out_logp), _stream()))

    def rollout_generate_queue(self, sample: rl_sample_cfg, prompt_ids: torch.Tensor, prompt_len, gen_limit, Gmax,
                               out_ids, out_len, out_logp=None):
        pl, plp = _host_i32(prompt_len)
        gl, glp = _host_i32(gen_limit)
        Q, Pmax = prompt_ids.shape
        _chk(lib().rollout_generate_queue(self.h, C.byref(sample), _ptr(prompt_ids), plp, glp, Q, Pmax, Gmax,
                                          _ptr(out_ids), _ptr(out_len), _ptr(out_logp), _stream()))

    def score_logprobs_kl(self, policy: Weights, reference, ids: torch.Tensor, seq_len, prompt_len, kl_coef,
                          logp_policy=None, logp_ref=None, kl=None, kl_penalty=None):
        sl, slp = _host_i32(seq_len)
        pl, plp = _host_i32(prompt_len)
        B, Lmax = ids.shape
        ref = C.byref(reference.struct) if reference is not None else None
        pol = C.byref(policy.struct) if policy is not None else None
        _chk(lib().score_logprobs_kl(self.h, pol, ref, _ptr(ids), slp, plp, B, Lmax, kl_coef,
                                     _ptr(logp_policy), _ptr(logp_ref), _ptr(kl), _ptr(kl_penalty), _stream()))

    def score_kl_exact(self, policy: Weights, reference: Weights, ids: torch.Tensor, seq_len, prompt_len, kl_full):
        sl, slp = _host_i32(seq_len)
        pl, plp = _host_i32(prompt_len)
        B, Lmax = ids.shape
        _chk(lib().score_kl_exact(self.h, C.byref(policy.struct), C.byref(reference.struct), _ptr(ids), slp, plp, B,
                                  Lmax, _ptr(kl_full), _stream()))

    def score_values(self, model: Weights, value_head: torch.Tensor, ids: torch.Tensor, seq_len, values):
        sl, slp = _host_i32(seq_len)
        B, Lmax = ids.shape
        _chk(lib().score_values(self.h, C.byref(model.struct), _ptr(value_head), _ptr(ids), slp, B, Lmax,
                                _ptr(values), _stream()))

    def ppo_rewards(self, kl: torch.Tensor, seq_reward: torch.Tensor, seq_len, prompt_len, kl_coef, rewards):
        sl, slp = _host_i32(seq_len)
        pl, plp = _host_i32(prompt_len)
        B, Lmax = kl.shape
        _chk(lib().ppo_rewards(self.h, _ptr(kl), _ptr(seq_reward), slp, plp, B, Lmax, kl_coef, _ptr(rewards),
                               _stream()))

    def rollout_check(self):
        _chk(lib().rollout_check(self.h, _stream()))

    def rollout_set_policy(self, policy: Weights):
        _chk(lib().rollout_set_policy(self.h, C.byref(policy.struct)))
        self.policy = policy            # keep the tensors alive

    def rollout_refresh_policy(self):
        _chk(lib().rollout_refresh_policy(self.h, _stream()))

    def rollout_reset(self):
        _chk(lib().rollout_reset(self.h))

    def rollout_set_impl(self, impl: int):
        _chk(lib().rollout_set_impl(self.h, impl))

    def rollout_set_precise_layers(self, n: int):
        _chk(lib().rollout_set_precise_layers(self.h, n))

    def rollout_forget_fp16_copies(self):
        _chk(lib().rollout_forget_fp16_copies(self.h))

    def rollout_set_fused_sampling(self, on: bool):
        _chk(lib().rollout_set_fused_sampling(self.h, 1 if on else 0))

    def rollout_set_fused_qkv_consumer(self, on: bool):
        _chk(lib().rollout_set_fused_qkv_consumer(self.h, 1 if on else 0))

    def rollout_profile_enable(self, kernel_class: int, every: int):
        _chk(lib().rollout_profile_enable(self.h, kernel_class, int(every)))

    def rollout_profile_read(self, kernel_class: int):
        ms, n = C.c_double(), C.c_int64()
        _chk(lib().rollout_profile_read(self.h, kernel_class, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def rollout_probe_mfma_rate(self, random_operands: bool = True) -> float:
        tf = C.c_double()
        _chk(lib().rollout_probe_mfma_rate(self.h, 1 if random_operands else 0, C.byref(tf), _stream()))
        return tf.value

    def rollout_profile_event_overhead(self, pairs: int = 256) -> float:
        ms = C.c_double()
        _chk(lib().rollout_profile_event_overhead(self.h, int(pairs), C.byref(ms), _stream()))
        return ms.value


def ppo_rewards_noalloc(kl: torch.Tensor, seq_reward: torch.Tensor, seq_len, prompt_len, kl_coef, rewards):
    """ppo_rewards without a context: allocates nothing, copies nothing (include/rollout.h)."""
    sl, slp = _host_i32(seq_len)
    pl, plp = _host_i32(prompt_len)
    B, Lmax = kl.shape
    _chk(lib().ppo_rewards_noalloc(_ptr(kl), _ptr(seq_reward), slp, plp, B, Lmax, kl_coef, _ptr(rewards), _stream()))


def rollout_set_decode_tile_rows(rows: int):
    _chk(lib().rollout_set_decode_tile_rows(int(rows)))


def rollout_set_large_gemm_copy(on: bool):
    _chk(lib().rollout_set_large_gemm_copy(1 if on else 0))


def sample_cfg(seed=0, temperature=0.0, eos_id=-1, seq_id_base=0) -> rl_sample_cfg:
    return rl_sample_cfg(seed, temperature, eos_id, seq_id_base)
