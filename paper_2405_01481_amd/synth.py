"""Seeded synthetic inputs: model shapes, weight bytes, prompts, ragged lengths.

This module serves both the CPU oracle's tests and the HIP path.  It contains
no arithmetic of the method itself (no norm, attention, softmax, sampling):
only shapes, seeded random draws and dtype/container conversions.  Whoever
consumes a weight set consumes the *same bytes*; nobody regenerates weights
from the seed on their own.

The five presets follow the benchmark's workload list: Llama-style decoder
shapes (pre-norm, RMSNorm, RoPE, SwiGLU, grouped-query attention, untied
embedding / LM head) at the tiny / 1B / 8B / 8B-long / 70B sizes, standing in
for the Llama-3 actors and HelpSteer2 prompts of the paper's PPO runs
(Section 3.3), which are not available here.

Weight layout (row-major, ``[out_features, in_features]`` like a linear layer
applied as ``y = x @ W.T``):

    tok_embed  [V, d]          final_norm [d]          lm_head [V, d]
    per layer: attn_norm [d]   wqkv [(Hq+2*Hkv)*hd, d] (q heads, then k, then v)
               wo [d, Hq*hd]   ffn_norm [d]
               w_gate_up [2*F, d] (gate rows, then up rows)   w_down [d, F]
"""
from __future__ import annotations

from dataclasses import dataclass, asdict

import numpy as np
import torch


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_base: float
    dtype: str            # "fp32" | "bf16"
    w_std: float
    rms_eps: float = 1e-5
    page_tokens: int = 16

    @property
    def qkv_rows(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16

    def body_params(self) -> int:
        d, hd = self.d_model, self.head_dim
        per_layer = (self.qkv_rows * d + d * self.n_q_heads * hd + 3 * d * self.d_ffn)
        return per_layer * self.n_layers

    def head_params(self) -> int:
        return self.vocab * self.d_model

    def kv_bytes_per_token(self) -> int:
        esz = 4 if self.dtype == "fp32" else 2
        return self.n_layers * 2 * self.n_kv_heads * self.head_dim * esz

    def as_dict(self):
        return asdict(self)


@dataclass(frozen=True)
class Workload:
    """One benchmark configuration: a shape plus batch / length / sampling recipe."""
    shape: ModelShape
    batch: int
    prompt_max: int       # prompt buffer width
    prompt_min: int       # == prompt_max unless ragged
    gen: int
    temperature: float    # 0 = greedy
    policy_seed: int = 1
    ref_seed: int = 2
    prompt_seed: int = 3
    sample_seed: int = 4


TINY = ModelShape("tiny", 2, 256, 4, 4, 64, 1024, 4096, 10000.0, "fp32", 0.02)
L1B = ModelShape("1b", 16, 2048, 32, 8, 64, 8192, 32000, 10000.0, "bf16", 0.02)
L8B = ModelShape("8b", 32, 4096, 32, 8, 128, 14336, 128256, 500000.0, "bf16", 0.02)
L70B = ModelShape("70b", 80, 8192, 64, 8, 128, 28672, 128256, 500000.0, "bf16", 0.01)

WORKLOADS = {
    "tiny": Workload(TINY, 4, 32, 32, 32, 0.0),
    "1b": Workload(L1B, 64, 256, 256, 256, 1.0),
    "8b": Workload(L8B, 128, 512, 512, 512, 1.0),
    "8b_long": Workload(L8B, 32, 2048, 1024, 2048, 1.0),
    "70b": Workload(L70B, 64, 1024, 1024, 1024, 1.0),
}


def scaled_shape(base: ModelShape, name: str, **kw) -> ModelShape:
    """A copy of ``base`` with some fields replaced (reduced-depth test cases)."""
    d = asdict(base)
    d.update(kw)
    d["name"] = name
    return ModelShape(**d)


# --------------------------------------------------------------------------
# weights
# --------------------------------------------------------------------------
_TENSOR_IDS = {"tok_embed": 1, "final_norm": 2, "lm_head": 3}
_LAYER_IDS = {"attn_norm": 0, "wqkv": 1, "wo": 2, "ffn_norm": 3, "w_gate_up": 4, "w_down": 5}


def _draw(shape, std, mean, seed, dtype, device):
    """N(mean, std) in fp32 from a per-tensor seeded stream, rounded once (RNE) to dtype."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    rows = shape[0]
    out = torch.empty(shape, dtype=dtype, device=device)
    # chunked over rows so a 128256 x 8192 tensor never needs a second full fp32 copy
    step = max(1, (1 << 27) // max(1, int(np.prod(shape[1:]))))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        t = torch.randn((r1 - r0,) + tuple(shape[1:]), generator=g, dtype=torch.float32, device=device)
        out[r0:r1] = (t * std + mean).to(dtype)
    return out


def layer_shapes(s: ModelShape):
    d, hd = s.d_model, s.head_dim
    return {
        "attn_norm": (d,),
        "wqkv": (s.qkv_rows, d),
        "wo": (d, s.n_q_heads * hd),
        "ffn_norm": (d,),
        "w_gate_up": (2 * s.d_ffn, d),
        "w_down": (d, s.d_ffn),
    }


def make_layer(s: ModelShape, seed: int, layer: int, device="cpu"):
    """One layer's tensors; every tensor has its own stream so layers can be made one at a time."""
    out = {}
    for name, shp in layer_shapes(s).items():
        tseed = (seed * 1_000_003 + (layer + 1) * 101 + _LAYER_IDS[name]) & 0x7FFFFFFFFFFFFFFF
        if name.endswith("_norm"):
            out[name] = _draw(shp, 0.02, 1.0, tseed, s.torch_dtype, device)   # gain = 1 + N(0, 0.02)
        else:
            out[name] = _draw(shp, s.w_std, 0.0, tseed, s.torch_dtype, device)
    return out


def make_globals(s: ModelShape, seed: int, device="cpu"):
    out = {}
    for name, shp in (("tok_embed", (s.vocab, s.d_model)), ("final_norm", (s.d_model,)),
                      ("lm_head", (s.vocab, s.d_model))):
        tseed = (seed * 1_000_003 + _TENSOR_IDS[name]) & 0x7FFFFFFFFFFFFFFF
        if name == "final_norm":
            out[name] = _draw(shp, 0.02, 1.0, tseed, s.torch_dtype, device)
        else:
            out[name] = _draw(shp, s.w_std, 0.0, tseed, s.torch_dtype, device)
    return out


def make_weights(s: ModelShape, seed: int, device="cpu"):
    """Full weight set as torch tensors of the shape's dtype on ``device``."""
    w = make_globals(s, seed, device)
    w["layers"] = [make_layer(s, seed, l, device) for l in range(s.n_layers)]
    return w


def to_numpy_f32(t: torch.Tensor) -> np.ndarray:
    """Exact upcast of a bf16 / fp32 tensor to a host float32 array (bf16 -> fp32 is lossless)."""
    return t.detach().to("cpu").to(torch.float32).numpy()


def weights_for_oracle(w):
    """Same bytes, host float32 numpy containers (lossless); no arithmetic."""
    out = {k: to_numpy_f32(v) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: to_numpy_f32(v) for k, v in lw.items()} for lw in w["layers"]]
    return out


# --------------------------------------------------------------------------
# prompts
# --------------------------------------------------------------------------
def make_prompts(vocab: int, batch: int, prompt_max: int, prompt_min: int, seed: int):
    """Uniform i.i.d. token ids in [0, vocab); lengths uniform in [prompt_min, prompt_max].

    Returns (ids int32 [batch, prompt_max], lens int32 [batch]); entries beyond a
    row's length are filled with 0 and must be ignored by every consumer.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    ids = rng.integers(0, vocab, size=(batch, prompt_max), dtype=np.int64).astype(np.int32)
    if prompt_min == prompt_max:
        lens = np.full((batch,), prompt_max, dtype=np.int32)
    else:
        lens = rng.integers(prompt_min, prompt_max + 1, size=(batch,), dtype=np.int64).astype(np.int32)
    for b in range(batch):
        ids[b, lens[b]:] = 0
    return ids, lens


def make_sequences(vocab: int, batch: int, len_max: int, len_min: int, prompt_frac: float, seed: int):
    """Random full sequences for scoring tests: (ids [B,Lmax], seq_len [B], prompt_len [B])."""
    ids, lens = make_prompts(vocab, batch, len_max, len_min, seed)
    plen = np.maximum(1, (lens * prompt_frac).astype(np.int32))
    return ids, lens, plen
