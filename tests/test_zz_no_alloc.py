"""The entry point that allocates nothing (ppo_rewards_noalloc) against the entry point it is a variant of
(ppo_rewards), through the C ABI: two calls in a row, the second with a smaller input, so that what the first
call left in the library's fixed array cannot leak into the second."""
import numpy as np
import pytest
import torch

from oracle import rollout_oracle as O
from paper_2405_01481_amd import rollout as R
from paper_2405_01481_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(B, Lmax, seed):
    rng = np.random.default_rng(seed)
    L = rng.integers(1, Lmax + 1, B).astype(np.int32)
    P = np.array([rng.integers(0, l + 1) for l in L], np.int32)
    L[0], P[0] = Lmax, 0
    if B > 1:
        L[1], P[1] = 1, 1
    kl = torch.tensor(rng.normal(0, 0.3, (B, Lmax)).astype(np.float32), device=DEV)
    rw = torch.tensor(rng.normal(0, 1.0, B).astype(np.float32), device=DEV)
    return kl, rw, L, P


def test_ppo_rewards_noalloc_matches_ppo_rewards():
    shape = synth.TINY
    wp = synth.make_weights(shape, 1, DEV)
    ro = R.Rollout(R.make_cfg(shape, 600, 64), R.Weights(wp), DEV)
    for B, Lmax, seed in ((600, 64, 1), (37, 41, 2)):          # several 192-value chunks, then fewer rows
        kl, rw, L, P = _case(B, Lmax, seed)
        want = torch.full((B, Lmax), 7.0, dtype=torch.float32, device=DEV)
        got = torch.full((B, Lmax), -7.0, dtype=torch.float32, device=DEV)
        ro.ppo_rewards(kl, rw, L, P, 0.003, want)
        before = torch.cuda.memory_allocated()
        R.ppo_rewards_noalloc(kl, rw, L, P, 0.003, got)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        assert torch.equal(got, want)                                      # same kernel, same inputs: same bits
        ref = O.ppo_rewards(kl.cpu().numpy(), rw.cpu().numpy(), L, P, 0.003)
        assert np.abs(got.cpu().numpy() - ref).max() <= 1e-6
    with pytest.raises(R.RolloutError):
        big = torch.zeros(4097, 2, dtype=torch.float32, device=DEV)
        R.ppo_rewards_noalloc(big, torch.zeros(4097, device=DEV), np.ones(4097, np.int32), np.zeros(4097, np.int32),
                              0.003, big.clone())
    ro.close()
