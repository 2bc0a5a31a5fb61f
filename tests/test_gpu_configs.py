"""GPU parity at the benchmark's real widths: the oracle runs at true width and depth on a
subset of rows / positions (it cannot finish the full batches in reasonable time)."""
import os

import numpy as np
import pytest
import torch

from oracle import rollout_oracle as O
from paper_2405_01481_amd import rollout as R
from paper_2405_01481_amd import synth
from tests.helpers import LazyModel, check_row, check_scores, verify_rollout

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
# The whole GPU suite has to fit a quarter of an hour of wall time, most of which is the float64 oracle on the
# host's cores.  By default the three full-size cases below take the oracle over part of their workload (stated in
# each docstring); ROLLOUT_FULL_PARITY=1 extends them to the whole of it (about a quarter of an hour more).
FULL = os.environ.get("ROLLOUT_FULL_PARITY", "") == "1"


def _conv(t, dt):
    """A torch tensor (device or host, bf16 / fp32) as a host numpy array of dtype dt: exact, cast on the GPU."""
    return t.to(DEV).to(torch.float64 if dt == np.float64 else torch.float32).cpu().numpy()


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


def _bench_run(wl, B, chunk=16384, ref_host=False, layers=None, gen=None):
    """The workload as bench.py runs it (captured decode graph on a side stream, chunks of 16384 tokens): generate,
    then score the rollouts under policy and reference.  Returns everything the oracle checks need."""
    s = wl.shape if layers is None else synth.scaled_shape(wl.shape, f"{wl.shape.name}_{layers}l", n_layers=layers)
    P, G = wl.prompt_max, gen or wl.gen
    wp = synth.make_weights(s, wl.policy_seed, DEV)
    cfg = R.make_cfg(s, B, P + G, max_chunk_tokens=max(P + G, chunk))
    if ref_host:
        # the reference never sits on the device in full: made a tensor at a time, kept in host memory (the first
        # 16 GB pinned) and streamed layer by layer while scoring
        pinned = [0]

        def host(t):
            h = t.cpu()
            nb = h.numel() * h.element_size()
            if pinned[0] + nb <= 16e9:
                pinned[0] += nb
                return h.pin_memory()
            return h
        wr = {k: host(v) for k, v in synth.make_globals(s, wl.ref_seed, DEV).items()}
        wr["layers"] = [{k: host(v) for k, v in synth.make_layer(s, wl.ref_seed, l, DEV).items()} for l in range(s.n_layers)]
        torch.cuda.empty_cache()
        staging = torch.empty(R.rollout_weight_staging_bytes(cfg), dtype=torch.uint8, device=DEV)
        Wp, Wr = R.Weights(wp), R.Weights(wr, staging=staging)
    else:
        wr = synth.make_weights(s, wl.ref_seed, DEV)
        Wp, Wr = R.Weights(wp), R.Weights(wr)
    ro = R.Rollout(cfg, Wp, DEV)
    ids, lens = synth.make_prompts(s.vocab, B, P, wl.prompt_min, wl.prompt_seed)
    out = torch.zeros(B, G, dtype=torch.int32, device=DEV)
    olp = torch.zeros(B, G, dtype=torch.float32, device=DEV)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ro.rollout_generate(R.sample_cfg(wl.sample_seed, wl.temperature), torch.tensor(ids, device=DEV), lens, G, out,
                            None, olp)
        side.synchronize()
    ro.rollout_check()
    g = out.cpu().numpy()
    full = np.zeros((B, P + G), np.int32)
    for b in range(B):
        full[b, :lens[b]] = ids[b, :lens[b]]
        full[b, lens[b]:lens[b] + G] = g[b]
    L = (lens + G).astype(np.int32)
    outs = [torch.zeros(B, P + G, dtype=torch.float32, device=DEV) for _ in range(4)]
    ro.score_logprobs_kl(Wp, Wr, torch.tensor(full, device=DEV), L, lens, 0.003, *outs)
    ro.rollout_check()
    got = [o.cpu().numpy() for o in outs]
    ro.close()
    del ro, outs
    torch.cuda.empty_cache()
    print("gpu done", flush=True)
    return s, wp, wr, full, L, lens, g, olp.cpu().numpy(), got


@pytest.mark.slow
def test_1b_bench_configuration_against_oracle():
    """Config 2 as stated (1B shape, 64 prompts of 256 tokens, 256 tokens sampled at temperature 1 with the shared
    uniforms, reference of the same shape from another seed), run whole on the GPU.  The oracle is teacher-forced
    over full rows under BOTH models: every position of log-probs and KL within 2e-2; on the first 8 of those rows
    every one of the 256 sampled tokens is verified along the GPU's trajectory.  Rows taken: 12 spread over the batch
    by default, all 64 with ROLLOUT_FULL_PARITY=1."""
    wl = synth.WORKLOADS["1b"]
    s, wp, wr, full, L, lens, g, glp, got = _bench_run(wl, wl.batch)
    mp = O.Model(s, synth.weights_for_oracle(wp))
    mr = O.Model(s, synth.weights_for_oracle(wr))
    rows = list(range(wl.batch)) if FULL else [int(r) for r in np.linspace(0, wl.batch - 1, 12).round()]
    worst = {"policy": 0.0, "ref": 0.0, "kl": 0.0, "gen": 0.0, "cdf": 0.0}
    for i, b in enumerate(rows):
        P = int(lens[b])
        verify = i < 8
        lp_o, st = check_row(mp, full[b, :L[b]], P, wl.sample_seed, b, got[0][b], g[b] if verify else None, glp[b])
        lr_o, st_r = check_row(mr, full[b, :L[b]], P, wl.sample_seed, b, got[1][b])
        kl_o = np.zeros(L[b])
        kl_o[P:] = (lp_o - lr_o)[P:]
        kl_err = float(np.abs(got[2][b, :L[b]] - kl_o).max())
        assert kl_err <= 2e-2, (b, kl_err)
        assert np.all(got[2][b, :P] == 0.0) and got[0][b, 0] == 0.0
        worst = {"policy": max(worst["policy"], st["max"]), "ref": max(worst["ref"], st_r["max"]),
                 "kl": max(worst["kl"], kl_err), "gen": max(worst["gen"], st["gen_max"]),
                 "cdf": max(worst["cdf"], st.get("cdf_viol_max", 0.0))}
        print("row", b, st, st_r, "kl max %.3e" % kl_err, flush=True)
    print("1b bench configuration:", len(rows), "rows, worst", worst)


@pytest.mark.slow
def test_8b_long_bench_configuration_against_oracle():
    """Config 4 as stated (8B shape at its full 32 layers, 32 ragged prompts of 1024-2048 tokens, 2048 sampled
    tokens: decode at contexts from 1 k to 4 k with split-KV attention, rotary positions up to 4095, scoring over
    rows of up to 4096 tokens), run whole on the GPU.  The row with the longest prompt (contexts pass 2048 and 4000)
    is checked over its full length under the policy: every log-prob within 2e-2, all 2048 sampled tokens inside the
    oracle's CDF bracket, generation log-probs within 2e-2.  The reference's log-probs and the KL term are checked
    on the row's first 1024 positions by default and on all of them with ROLLOUT_FULL_PARITY=1."""
    wl = synth.WORKLOADS["8b_long"]
    s, wp, wr, full, L, lens, g, glp, got = _bench_run(wl, wl.batch)
    b = int(np.argmax(lens))
    P, n = int(lens[b]), int(L[b])
    assert n > 4000 and P > 1500
    conv = _conv
    mp = LazyModel(s, wp, conv)
    lp_o, st = check_row(mp, full[b, :n], P, wl.sample_seed, b, got[0][b], g[b], glp[b])
    print("8b_long row", b, "prompt", P, "length", n, "policy", st, flush=True)
    del mp
    upto = n if FULL else 1024
    mr = LazyModel(s, wr, conv)
    lr_o, st_r = check_row(mr, full[b, :n], P, wl.sample_seed, b, got[1][b], upto=upto)
    print("reference on the first", upto, "positions", st_r, flush=True)
    if upto > P:
        kl_err = float(np.abs(got[2][b, P:upto] - (lp_o[P:upto] - lr_o[P:upto])).max())
        print("kl max %.3e" % kl_err)
        assert kl_err <= 2e-2
    assert np.all(got[2][b, :P] == 0.0) and np.all(got[2][b, n:] == 0.0)


@pytest.mark.slow
def test_70b_residency_full_depth_against_oracle():
    """Config 5's model and residency: 70B shape (d 8192, 64 query / 8 KV heads, FFN 28672, vocab 128256), the
    policy resident on the device for generation, the reference weights in host memory and streamed layer by layer
    while scoring.  Four prompts of 72 tokens, 24 sampled tokens; one row checked at every position under both
    models (95 scored positions, 24 verified sampled tokens), the oracle fed one layer at a time.  Depth: 16 of the
    80 layers by default, all 80 with ROLLOUT_FULL_PARITY=1."""
    layers = 80 if FULL else 16
    wl = synth.Workload(synth.L70B, 4, 72, 72, 24, 1.0)
    s, wp, wr, full, L, lens, g, glp, got = _bench_run(wl, wl.batch, ref_host=True, layers=layers)
    b = 2
    P, n = int(lens[b]), int(L[b])
    mp = LazyModel(s, wp, _conv)
    lp_o, st = check_row(mp, full[b, :n], P, wl.sample_seed, b, got[0][b], g[b], glp[b])
    print("70b shape,", layers, "layers, row", b, "policy", st, flush=True)
    del mp
    mr = LazyModel(s, wr, _conv)
    lr_o, st_r = check_row(mr, full[b, :n], P, wl.sample_seed, b, got[1][b])
    kl_err = float(np.abs(got[2][b, P:n] - (lp_o[P:n] - lr_o[P:n])).max())
    print("reference", st_r, "kl max %.3e" % kl_err)
    assert kl_err <= 2e-2


def test_exact_kl_and_values_at_8b_width():
    """score_kl_exact and score_values at the 8B width (d 4096, FFN 14336, 32 query / 8 KV heads of 128, vocab
    128256 -- 1002 column tiles and 2004 partial groups per row in the dual LM head) with two layers, so that the
    oracle's cost is the two LM heads: three ragged rows, every position against the oracle's full-vocabulary KL
    and its value head."""
    s = synth.scaled_shape(synth.L8B, "8b_2l", n_layers=2)
    B, Lmax = 3, 48
    wp, wr = synth.make_weights(s, 1, DEV), synth.make_weights(s, 2, DEV)
    Wp, Wr = R.Weights(wp), R.Weights(wr)
    ro = R.Rollout(R.make_cfg(s, B, Lmax), Wp, DEV)
    ids, lens, plens = synth.make_sequences(s.vocab, B, Lmax, 20, 0.4, 95)
    d_ids = torch.tensor(ids, device=DEV)
    klx = torch.full((B, Lmax), 9.0, dtype=torch.float32, device=DEV)
    ro.score_kl_exact(Wp, Wr, d_ids, lens, plens, klx)
    head = (torch.randn(s.d_model, generator=torch.Generator().manual_seed(96)) * 0.05).to(torch.bfloat16).to(DEV)
    val = torch.full((B, Lmax), 9.0, dtype=torch.float32, device=DEV)
    ro.score_values(Wr, head, d_ids, lens, val)
    ro.rollout_check()
    got_kl, got_v = klx.cpu().numpy(), val.cpu().numpy()
    ro.close()
    mp = O.Model(s, synth.weights_for_oracle(wp))
    mr = O.Model(s, synth.weights_for_oracle(wr))
    want_kl = np.zeros((B, Lmax))
    for b in range(B):
        L, P = int(lens[b]), max(int(plens[b]), 1)
        want_kl[b, P:L] = O.kl_full(mp, mr, ids[b, :L])[P:L]
    want_v = O.values_batch(mr, head.float().cpu().numpy().astype(np.float64), ids, lens)
    e_kl, e_v = np.abs(got_kl - want_kl).max(), np.abs(got_v - want_v).max()
    print("8b width, 2 layers: exact KL max", want_kl.max(), "err", e_kl, "| values err", e_v)
    assert e_kl <= 2e-2 and e_v <= 2e-2
    assert np.all(got_kl[want_kl == 0.0] == 0.0) and np.all(got_v[want_v == 0.0] == 0.0)
    assert want_kl.max() > 0.2
