"""Host-only checks of the C ABI: the library loads, exports every declared symbol, and
rejects bad arguments before touching the GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2405_01481_amd import rollout as R
from paper_2405_01481_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "rollout.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b((?:rollout|score|ppo)_[a-z_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert {"rollout_init", "rollout_decode_step", "rollout_generate", "score_logprobs_kl"} <= set(names)
    assert {"ppo_rewards", "score_values", "score_kl_exact", "rollout_generate_queue", "rollout_set_policy",
            "rollout_refresh_policy", "rollout_weight_shadow_bytes"} <= set(names)
    lib = R.lib()
    for n in names:
        assert hasattr(lib, n), n


def test_sizes_and_cfg_validation():
    good = R.make_cfg(synth.TINY, 4, 64)
    assert R.rollout_workspace_bytes(good) > 0
    exp_kv = 2 * 2 * good.n_pages * 4 * 16 * 64 * 4
    assert R.rollout_kv_pool_bytes(good) == exp_kv
    for field, bad in [("head_dim", 96), ("n_kv_heads", 3), ("page_tokens", 8), ("dtype", 7), ("d_model", 100),
                       ("max_chunk_tokens", 8), ("n_pages", 0), ("max_batch", 0)]:
        cfg = R.make_cfg(synth.TINY, 4, 64)
        setattr(cfg, field, bad)
        assert R.rollout_workspace_bytes(cfg) == 0, field
        assert R.rollout_last_error() != ""
    assert R.lib().rollout_workspace_bytes(None) == 0
    # staging for a host-resident weight set: two layers + one [vocab, d] table + fp32 residual of all tokens
    t = synth.TINY
    layer = (2 * t.d_model + (t.n_q_heads + 2 * t.n_kv_heads) * t.head_dim * t.d_model
             + t.d_model * t.n_q_heads * t.head_dim + 3 * t.d_ffn * t.d_model) * 4
    lo = 2 * layer + t.vocab * t.d_model * 4 + 4 * 64 * t.d_model * 4
    got = R.rollout_weight_staging_bytes(good)
    assert lo <= got <= lo + 16 * 256 + t.d_model * 4
    assert R.lib().rollout_weight_staging_bytes(None) == 0


def test_null_and_state_errors_without_gpu():
    lib = R.lib()
    h = C.c_void_p()
    cfg = R.make_cfg(synth.TINY, 4, 64)
    assert lib.rollout_init(C.byref(cfg), None, None, 0, None, 0, C.byref(h)) == R.RL_EINVAL
    assert lib.rollout_init(C.byref(cfg), None, None, 0, None, 0, None) == R.RL_EINVAL
    assert lib.rollout_prefill(None, None, None, 1, 1, None) == R.RL_EINVAL
    s = R.sample_cfg()
    assert lib.rollout_decode_step(None, C.byref(s), None, None, None, None) == R.RL_EINVAL
    assert lib.rollout_generate(None, C.byref(s), None, None, 1, 1, 1, None, None, None, None) == R.RL_EINVAL
    assert lib.score_logprobs_kl(None, None, None, None, None, None, 1, 1, 0.0, None, None, None, None, None) == R.RL_EINVAL
    assert lib.rollout_reset(None) == R.RL_EINVAL
    assert lib.rollout_check(None, None) == R.RL_EINVAL
    lib.rollout_destroy(None)
    assert b"NULL" in lib.rollout_last_error()


def test_binding_fails_loudly_when_library_missing(monkeypatch):
    monkeypatch.setattr(R, "_lib", None)
    monkeypatch.setattr(R, "LIB_PATH", "/nonexistent/librollout.so")
    with pytest.raises(R.RolloutError):
        R.lib()
