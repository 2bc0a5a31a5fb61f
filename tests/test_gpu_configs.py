"""GPU parity at the benchmark's real widths: the oracle runs at true width and depth on a
subset of rows / positions (it cannot finish the full batches in reasonable time)."""
import numpy as np
import pytest
import torch

from oracle import rollout_oracle as O
from paper_2405_01481_amd import rollout as R
from paper_2405_01481_amd import synth
from tests.helpers import check_scores, verify_rollout

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_1b_shape_scoring_and_rollout_subset():
    """Config 2 (1B Llama shape, bf16, temperature-1 hash sampling), reduced batch/lengths:
    8 rows, prompts of 48, 24 generated tokens; oracle on 2 rows at full width and depth."""
    wl = synth.WORKLOADS["1b"]
    s = wl.shape
    B, P, G = 8, 48, 24
    wp, wr = synth.make_weights(s, wl.policy_seed, DEV), synth.make_weights(s, wl.ref_seed, DEV)
    Wp, Wr = R.Weights(wp), R.Weights(wr)
    ro = R.Rollout(R.make_cfg(s, B, P + G), Wp, DEV)
    ids, lens = synth.make_prompts(s.vocab, B, P, P, wl.prompt_seed)
    out = torch.zeros(B, G, dtype=torch.int32, device=DEV)
    olp = torch.zeros(B, G, dtype=torch.float32, device=DEV)
    ro.rollout_generate(R.sample_cfg(wl.sample_seed, 1.0), torch.tensor(ids, device=DEV), lens, G, out, None, olp)
    ro.rollout_check()
    g = out.cpu().numpy()
    full = np.concatenate([ids, g], axis=1).astype(np.int32)
    L = np.full(B, P + G, np.int32)
    outs = [torch.zeros(B, P + G, dtype=torch.float32, device=DEV) for _ in range(4)]
    ro.score_logprobs_kl(Wp, Wr, torch.tensor(full, device=DEV), L, lens, 0.003, *outs)
    ro.rollout_check()
    got = [o.cpu().numpy() for o in outs]
    mp = O.Model(s, synth.weights_for_oracle(wp))
    mr = O.Model(s, synth.weights_for_oracle(wr))
    rows = [0, 5]
    st = verify_rollout(mp, [ids[b] for b in range(B)], g, olp.cpu().numpy(), 1.0, wl.sample_seed, 0, 1e-3, 2e-2,
                        rows=rows)
    ref = O.score_batch(mp, mr, full[rows], L[rows], lens[rows], 0.003)
    errs = check_scores(*[a[rows] for a in got], ref, 2e-2, 0.003)
    print("1b subset:", st, errs)
    ro.close()


def _run_and_check(shape, B, P_lo, P_hi, G, rows, seed=4, temp=1.0, chunk=None, score_positions=None,
                   ref_on_host=False):
    """Generate with the GPU path, then verify `rows` with the oracle at the shape's full width and
    depth: every generated token along the GPU trajectory, and teacher-forced scores of both models."""
    wp, wr = synth.make_weights(shape, 1, DEV), synth.make_weights(shape, 2, DEV)
    Lmax = P_hi + G
    cfg = R.make_cfg(shape, B, Lmax, max_chunk_tokens=chunk)
    if ref_on_host:
        # reference weights live in pinned host memory and are streamed layer by layer while scoring
        pin = lambda t: t.cpu().pin_memory()
        wr = {**{k: pin(wr[k]) for k in ("tok_embed", "final_norm", "lm_head")},
              "layers": [{k: pin(v) for k, v in lay.items()} for lay in wr["layers"]]}
        torch.cuda.empty_cache()
        staging = torch.empty(R.rollout_weight_staging_bytes(cfg), dtype=torch.uint8, device=DEV)
        Wp, Wr = R.Weights(wp), R.Weights(wr, staging=staging)
    else:
        Wp, Wr = R.Weights(wp), R.Weights(wr)
    ro = R.Rollout(cfg, Wp, DEV)
    ids, lens = synth.make_prompts(shape.vocab, B, P_hi, P_lo, 3)
    out = torch.zeros(B, G, dtype=torch.int32, device=DEV)
    olp = torch.zeros(B, G, dtype=torch.float32, device=DEV)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):                      # captured-graph decode, as bench.py runs it
        ro.rollout_generate(R.sample_cfg(seed, temp), torch.tensor(ids, device=DEV), lens, G, out, None, olp)
        side.synchronize()
    ro.rollout_check()
    g = out.cpu().numpy()
    full = np.zeros((B, Lmax), np.int32)
    for b in range(B):
        full[b, :lens[b]] = ids[b, :lens[b]]
        full[b, lens[b]:lens[b] + G] = g[b]
    L = (lens + G).astype(np.int32)
    outs = [torch.zeros(B, Lmax, dtype=torch.float32, device=DEV) for _ in range(4)]
    ro.score_logprobs_kl(Wp, Wr, torch.tensor(full, device=DEV), L, lens, 0.003, *outs)
    ro.rollout_check()
    got = [o.cpu().numpy() for o in outs]
    ro.close()
    del ro
    mp = O.Model(shape, synth.weights_for_oracle(wp))
    mr = O.Model(shape, synth.weights_for_oracle(wr))
    del wp, wr
    torch.cuda.empty_cache()
    st = verify_rollout(mp, [ids[b, :lens[b]] for b in range(B)], g, olp.cpu().numpy(), temp, seed, 0, 1e-3, 2e-2,
                        rows=rows)
    ref = O.score_batch(mp, mr, full[rows], L[rows], lens[rows], 0.003)
    errs = check_scores(*[a[rows] for a in got], ref, 2e-2, 0.003)
    # generation log-probs are the teacher-forced policy scores of the same tokens
    for b in rows:
        assert np.abs(got[0][b, lens[b]:L[b]] - olp.cpu().numpy()[b]).max() < 2e-2
    return st, errs


def test_70b_shape_three_layers_reference_on_host():
    """Config 5's width (d 8192, 64 query / 8 KV heads: GQA group of 8, FFN 28672, vocab 128256) and its
    residency: the policy is on the device, the reference weights sit in pinned host memory and are
    streamed layer by layer during scoring.  Three layers, so a staging slot is refilled while in use
    elsewhere; exercises the widest rows and the 8-wave attention workgroups."""
    s = synth.scaled_shape(synth.L70B, "70b_3l", n_layers=3)
    st, errs = _run_and_check(s, 3, 30, 44, 6, rows=[1], ref_on_host=True)
    print("70b-shape 3 layers, reference on host:", st, errs)


def test_8b_long_ragged_four_layers():
    """Config 4's regime (ragged prompts, contexts of 1-2 k tokens, split-KV decode, long causal
    prefill) at the 8B width with four layers, so the oracle finishes in about a minute."""
    s = synth.scaled_shape(synth.L8B, "8b_4l", n_layers=4)
    st, errs = _run_and_check(s, 3, 1030, 1700, 5, rows=[0])
    print("8b long ragged 4 layers:", st, errs)


@pytest.mark.slow
def test_8b_full_depth_subset():
    """Config 3's model at full width and depth (32 layers): batch 4, prompts of 40, 8 generated
    tokens; the oracle checks one row (both models)."""
    s = synth.L8B
    st, errs = _run_and_check(s, 4, 40, 40, 8, rows=[2])
    print("8b full depth:", st, errs)


@pytest.mark.slow
def test_8b_bench_configuration_full_length_row():
    """The configuration bench.py times (config 3: batch 128, prompts of 512, 512 sampled tokens, 32
    layers, chunks of 16384 tokens, decode replayed as a captured graph -- so the 256 x 256 GEMM tiles,
    the ring decode GEMM at 128 rows and the paged attention at contexts up to 1023 are the kernels
    that run), checked on one full row: the oracle is teacher-forced over the row's 1024 tokens under
    both models.  The bar is the contract's: every scored position of the row within 2e-2 of the
    oracle for the policy's and the reference's log-probs, the generation log-probs and the KL term;
    every sampled token inside the oracle's CDF bracket."""
    wl = synth.WORKLOADS["8b"]
    s, B, P, G = wl.shape, wl.batch, wl.prompt_max, wl.gen
    row = 77
    wp, wr = synth.make_weights(s, wl.policy_seed, DEV), synth.make_weights(s, wl.ref_seed, DEV)
    Wp, Wr = R.Weights(wp), R.Weights(wr)
    ro = R.Rollout(R.make_cfg(s, B, P + G, max_chunk_tokens=16384), Wp, DEV)
    ids, lens = synth.make_prompts(s.vocab, B, P, P, wl.prompt_seed)
    out = torch.zeros(B, G, dtype=torch.int32, device=DEV)
    olp = torch.zeros(B, G, dtype=torch.float32, device=DEV)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ro.rollout_generate(R.sample_cfg(wl.sample_seed, wl.temperature), torch.tensor(ids, device=DEV), lens, G,
                            out, None, olp)
        side.synchronize()
    ro.rollout_check()
    g = out.cpu().numpy()
    full = np.concatenate([ids, g], axis=1).astype(np.int32)
    L = np.full(B, P + G, np.int32)
    outs = [torch.zeros(B, P + G, dtype=torch.float32, device=DEV) for _ in range(4)]
    ro.score_logprobs_kl(Wp, Wr, torch.tensor(full, device=DEV), L, lens, 0.003, *outs)
    ro.rollout_check()
    lp_g, lr_g, kl_g, _ = [o.cpu().numpy()[row] for o in outs]
    gen_lp = olp.cpu().numpy()[row]
    ro.close()
    del ro
    print("gpu done", flush=True)

    seq = full[row].astype(np.int64)
    stats = {}
    for name, w, got in (("policy", wp, lp_g), ("reference", wr, lr_g)):
        m = O.Model(s, synth.weights_for_oracle(w))
        z = O.forward_logits(m, seq[:-1])                     # logits for positions 1 .. L-1
        lsm = np.stack([O.log_softmax(z[t]) for t in range(z.shape[0])])
        want = lsm[np.arange(P + G - 1), seq[1:]]
        err = got[1:] - want
        stats[name] = (float(np.sqrt(np.mean(err ** 2))), float(np.mean(np.abs(err) > 2e-2)), float(np.abs(err).max()))
        if name == "policy":
            lp_o = want
            # sampled tokens along the GPU trajectory: shared uniform inside the oracle's CDF bracket
            viol = []
            for n in range(G):
                c = np.cumsum(np.exp(lsm[P - 1 + n]))
                u = O.hash_uniform(wl.sample_seed, row, n)
                t = int(g[row, n])
                lo = c[t - 1] if t > 0 else 0.0
                viol.append(max(lo - u, u - c[t], 0.0))
            viol = np.array(viol)
            gen_err = np.abs(gen_lp - want[P - 1:])
        else:
            lr_o = want
        del m, z, lsm
        print(name, stats[name], flush=True)
    kl_err = np.abs(kl_g[P:] - (lp_o - lr_o)[P - 1:])
    print("8b bench configuration, row", row, stats, "cdf viol max", viol.max(), "frac>1e-3", np.mean(viol > 1e-3),
          "gen logp max", gen_err.max(), "kl max", kl_err.max())
    for name in stats:
        rms, frac, mx = stats[name]
        assert mx <= 2e-2, (name, stats[name])
    assert viol.max() < 1e-3                                 # every sampled token inside the oracle's CDF bracket
    assert gen_err.max() <= 2e-2
    assert kl_err.max() <= 2e-2
    assert np.all(kl_g[:P] == 0.0) and lp_g[0] == 0.0
