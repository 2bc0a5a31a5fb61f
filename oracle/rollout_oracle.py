"""CPU oracle for PPO rollout: generation, teacher-forced log-probs, KL term.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file;
only tests, the smoke check and the benchmark's cpu_baseline leg do.  It shares
no code, tables or helpers with the HIP library.

The paper (NeMo-Aligner, Section 3.1-3.3) names the computations -- response
generation as repeated forward passes with one new token each (Section 3.2),
log-probabilities under the actor and under the frozen reference policy, and
the KL penalty between them (Section 2.2 step 3, Section 3.1 item 2, KL
coefficient in Section 3.3) -- but prints no formula for any of them.  The
definitions below are therefore the standard ones for a Llama-style decoder,
written out plainly in float64 numpy: no blocking, no fusion, no cache tricks
beyond the KV cache the paper itself mentions (Section 3.2).

Every reduction is float64.  Weights arrive as float32 arrays holding exactly
the bytes the GPU sees (bf16 upcasts losslessly) and are promoted to float64 at
use.  Linear maps are ``y = x @ W.T`` with ``W [out, in]``.

Parity pins: see tests/test_oracle_pins.py (closed forms, invariants, brute
force, independent torch-CPU cross-checks).  The paper prints no worked
numeric value, so beyond those pins parity is unpinned by the paper.
"""
from __future__ import annotations

import math

import numpy as np

F64 = np.float64
_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15


# ---------------------------------------------------------------------------
# counter-based uniforms (the benchmark's "counter-based hash of (seed,
# sequence, step)"; the paper does not describe a sampler).  mix64 is the
# published splitmix64 output function; chaining it over the three counters
# is this repository's choice and the HIP side implements the same integers.
# ---------------------------------------------------------------------------
def mix64(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def hash_uniform(seed: int, seq: int, step: int) -> float:
    """u in [0,1) with 24 random bits, exactly representable in float32."""
    h = mix64((seed + _GOLDEN * (seq + 1)) & _M64)
    h = mix64((h + _GOLDEN * (step + 1)) & _M64)
    return (h >> 40) * (1.0 / (1 << 24))


# ---------------------------------------------------------------------------
# model pieces
# ---------------------------------------------------------------------------
def rmsnorm(x, g, eps):
    """x / sqrt(mean(x^2) + eps) * g over the last axis."""
    x = np.asarray(x, F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(g, F64)


def rope(x, pos, base):
    """Rotary embedding, half-split pairing (j, j + hd/2), theta_j = base^(-2j/hd).

    x [n, H, hd]; pos [n] absolute positions starting at 0.
    """
    x = np.asarray(x, F64)
    hd = x.shape[-1]
    half = hd // 2
    theta = np.power(F64(base), -2.0 * np.arange(half, dtype=F64) / hd)
    ang = np.asarray(pos, F64)[:, None] * theta[None, :]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(y):
    return y / (1.0 + np.exp(-y))


def attention(q, k, v, q_pos0):
    """Causal grouped-query attention of one sequence.

    q [nq, Hq, hd] are the queries at absolute positions q_pos0 .. q_pos0+nq-1;
    k, v [nk, Hkv, hd] are all keys/values at positions 0 .. nk-1 (nk = q_pos0+nq).
    Query head j reads KV head j // (Hq // Hkv).  Query i attends keys m <= q_pos0+i.
    """
    nq, Hq, hd = q.shape
    nk, Hkv, _ = k.shape
    rep = Hq // Hkv
    out = np.empty((nq, Hq, hd), F64)
    qi = q_pos0 + np.arange(nq)[:, None]
    km = np.arange(nk)[None, :]
    allowed = km <= qi
    for j in range(Hq):
        g = j // rep
        s = (q[:, j, :] @ k[:, g, :].T) / math.sqrt(hd)
        s = np.where(allowed, s, -np.inf)
        s = s - s.max(axis=-1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=-1, keepdims=True)
        out[:, j, :] = p @ v[:, g, :]
    return out


class Model:
    """Shape + weights.  ``weights`` is the dict layout documented in the input generator."""

    def __init__(self, shape, weights):
        self.s = shape
        self.w = weights

    def layer(self, l):
        return self.w["layers"][l]


def _lin(x, W):
    return x @ np.asarray(W, F64).T


def layer_forward(m: Model, l: int, x, pos0: int, cache):
    """One pre-norm decoder layer on n new tokens of one sequence.

    x [n, d] residual stream; cache = (K, V) arrays of the pos0 earlier tokens
    ([pos0, Hkv, hd] each) or None.  Returns (x_out, (K_all, V_all)).
    """
    s = m.s
    w = m.layer(l)
    n = x.shape[0]
    Hq, Hkv, hd = s.n_q_heads, s.n_kv_heads, s.head_dim
    h = rmsnorm(x, w["attn_norm"], s.rms_eps)
    qkv = _lin(h, w["wqkv"])
    q = qkv[:, : Hq * hd].reshape(n, Hq, hd)
    k = qkv[:, Hq * hd: (Hq + Hkv) * hd].reshape(n, Hkv, hd)
    v = qkv[:, (Hq + Hkv) * hd:].reshape(n, Hkv, hd)
    pos = pos0 + np.arange(n)
    q = rope(q, pos, s.rope_base)
    k = rope(k, pos, s.rope_base)
    if cache is not None and cache[0].shape[0] > 0:
        k_all = np.concatenate([cache[0], k], axis=0)
        v_all = np.concatenate([cache[1], v], axis=0)
    else:
        k_all, v_all = k, v
    a = attention(q, k_all, v_all, pos0).reshape(n, Hq * hd)
    x = x + _lin(a, w["wo"])
    h2 = rmsnorm(x, w["ffn_norm"], s.rms_eps)
    gu = _lin(h2, w["w_gate_up"])
    F = s.d_ffn
    act = silu(gu[:, :F]) * gu[:, F:]
    x = x + _lin(act, w["w_down"])
    return x, (k_all, v_all)


def forward_hidden(m: Model, tokens, caches=None, pos0=0):
    """Final residual stream [n, d] for n new tokens of one sequence (caches updated in place)."""
    tokens = np.asarray(tokens, np.int64)
    x = np.asarray(m.w["tok_embed"][tokens], F64)
    for l in range(m.s.n_layers):
        c = None if caches is None else caches[l]
        x, c2 = layer_forward(m, l, x, pos0, c)
        if caches is not None:
            caches[l] = c2
    return x


def logits_from_hidden(m: Model, x):
    """z = RMSNorm(x; g_final) @ W_lm.T, [n, V]."""
    return _lin(rmsnorm(x, m.w["final_norm"], m.s.rms_eps), m.w["lm_head"])


def forward_logits(m: Model, tokens):
    """Full-recompute logits [n, V] at every position of one sequence."""
    return logits_from_hidden(m, forward_hidden(m, tokens))


def log_softmax(z):
    z = np.asarray(z, F64)
    zmax = z.max(axis=-1, keepdims=True)
    return z - zmax - np.log(np.exp(z - zmax).sum(axis=-1, keepdims=True))


# ---------------------------------------------------------------------------
# generation (Section 3.2: one token per forward pass, KV cache kept)
# ---------------------------------------------------------------------------
def pick_token(z, temperature, u):
    """Greedy arg-max (lowest index on ties) at temperature 0, else inverse CDF:
    smallest v with sum_{j<=v} softmax(z/T)_j > u, falling back to V-1."""
    z = np.asarray(z, F64)
    if temperature == 0.0:
        return int(np.argmax(z))
    p = np.exp(log_softmax(z / temperature))
    c = np.cumsum(p)
    idx = int(np.searchsorted(c, u, side="right"))
    return min(idx, z.shape[0] - 1)


def generate(m: Model, prompts, gen_len, temperature=0.0, seed=0, seq_id_base=0, use_cache=True):
    """Autoregressive rollouts for a list of prompts (each a 1-D int array, ragged allowed).

    Returns (ids int32 [B, gen_len], logp float64 [B, gen_len]) where logp is the
    temperature-1 log-probability of each emitted token.  With use_cache=False
    every step recomputes the whole prefix (for the cache == recompute invariant).
    """
    B = len(prompts)
    ids = np.zeros((B, gen_len), np.int32)
    lps = np.zeros((B, gen_len), F64)
    for b, prompt in enumerate(prompts):
        toks = [int(t) for t in prompt]
        caches = [None] * m.s.n_layers
        x = None
        for n in range(gen_len):
            if use_cache:
                if n == 0:
                    x = forward_hidden(m, toks, caches, 0)[-1:]
                else:
                    x = forward_hidden(m, toks[-1:], caches, len(toks) - 1)
            else:
                x = forward_hidden(m, toks)[-1:]
            z = logits_from_hidden(m, x)[0]
            u = hash_uniform(seed, seq_id_base + b, n)
            t = pick_token(z, temperature, u)
            ids[b, n] = t
            lps[b, n] = log_softmax(z)[t]
            toks.append(t)
    return ids, lps


# ---------------------------------------------------------------------------
# scoring and KL (Section 3.1: actor and reference are the same network with
# different weights; Section 2.2 step 3: KL regulariser w.r.t. the SFT model)
# ---------------------------------------------------------------------------
def score(m: Model, tokens):
    """logp[t] = log softmax(z_{t-1})[tokens[t]] for t >= 1, logp[0] = 0.  float64 [L]."""
    tokens = np.asarray(tokens, np.int64)
    L = tokens.shape[0]
    out = np.zeros((L,), F64)
    if L < 2:
        return out
    lsm = log_softmax(forward_logits(m, tokens)[:-1])
    out[1:] = lsm[np.arange(L - 1), tokens[1:]]
    return out


def kl_sampled(logp_policy, logp_ref, prompt_len, seq_len):
    """Per-token KL estimate on the rollout's own tokens: logp_policy - logp_ref on
    response positions [prompt_len, seq_len), 0 elsewhere."""
    lp = np.asarray(logp_policy, F64)
    lr = np.asarray(logp_ref, F64)
    out = np.zeros_like(lp)
    out[prompt_len:seq_len] = lp[prompt_len:seq_len] - lr[prompt_len:seq_len]
    return out


def kl_full(m_policy: Model, m_ref: Model, tokens):
    """Exact KL(pi_policy(.|<t) || pi_ref(.|<t)) for t >= 1 (0 at t = 0).  float64 [L]."""
    tokens = np.asarray(tokens, np.int64)
    L = tokens.shape[0]
    out = np.zeros((L,), F64)
    if L < 2:
        return out
    lp = log_softmax(forward_logits(m_policy, tokens)[:-1])
    lr = log_softmax(forward_logits(m_ref, tokens)[:-1])
    out[1:] = (np.exp(lp) * (lp - lr)).sum(axis=-1)
    return out


def score_batch(m_policy: Model, m_ref: Model, ids, seq_len, prompt_len, kl_coef=0.003):
    """Batch form with the output convention of the library call: arrays [B, Lmax],
    zeros outside the scored range.  Returns (logp_policy, logp_ref, kl, kl_penalty)."""
    ids = np.asarray(ids)
    B, Lmax = ids.shape
    lp = np.zeros((B, Lmax), F64)
    lr = np.zeros((B, Lmax), F64)
    kl = np.zeros((B, Lmax), F64)
    for b in range(B):
        L = int(seq_len[b])
        lp[b, :L] = score(m_policy, ids[b, :L])
        lr[b, :L] = score(m_ref, ids[b, :L])
        kl[b, :L] = kl_sampled(lp[b, :L], lr[b, :L], int(prompt_len[b]), L)
    return lp, lr, kl, kl_coef * kl


# --------------------------------------------------------------------------
# critic / reward-model head and the PPO reward (Section 2.2 steps 2-3, Section 3.1)
# --------------------------------------------------------------------------
def values(m: Model, value_head, tokens):
    """Per-token scalar of a critic or reward model: the same decoder body with a [d] -> 1 head in
    place of the LM head (Section 3.1: the critic is initialised from the reward model and "the reward
    model and the critic" are served for inference).  v[t] = head . RMSNorm(x_t; g_final), the state
    after reading token t.  A sequence-level reward is v[L-1]."""
    x = forward_hidden(m, tokens)
    h = rmsnorm(x, m.w["final_norm"], m.s.rms_eps)
    return h @ np.asarray(value_head, F64)


def values_batch(m: Model, value_head, ids, seq_len):
    """[B, Lmax] with zeros past each row's length (the library call's convention)."""
    ids = np.asarray(ids)
    out = np.zeros(ids.shape, F64)
    for b in range(ids.shape[0]):
        L = int(seq_len[b])
        out[b, :L] = values(m, value_head, ids[b, :L])
    return out


def ppo_rewards(kl, seq_reward, seq_len, prompt_len, kl_coef):
    """Per-token PPO reward (Section 2.2 step 3: the reward-model score of the rollout, regularised by
    the KL penalty towards the reference policy): r[b,t] = -kl_coef * kl[b,t] on response positions
    [prompt_len, L), plus the sequence's scalar reward on its last token; 0 elsewhere."""
    kl = np.asarray(kl, F64)
    r = np.zeros_like(kl)
    for b in range(kl.shape[0]):
        L, P = int(seq_len[b]), int(prompt_len[b])
        r[b, P:L] = -kl_coef * kl[b, P:L]
        if L > P:
            r[b, L - 1] += float(seq_reward[b])
    return r
