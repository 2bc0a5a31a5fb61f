#!/usr/bin/env python3
"""Benchmark of the rollout hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic batch: rollout_generate
(prompt prefill + G decode steps over the paged KV cache) followed by
score_logprobs_kl (teacher-forced log-probs under policy and reference + KL).
Prints ONE JSON line.  `value` = generated tokens per second over the whole step,
inputs resident in HBM.  Extra keys give the decode-only and scoring-only rates,
the roofline of the dominant kernel class (HIP events on the launch stream, live in
the timed region) and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2405_01481_amd import rollout as R   # noqa: E402
from paper_2405_01481_amd import synth          # noqa: E402

HBM_PEAK_GBPS = 8000.0        # MI355X HBM3E
MFMA_PEAK_TFLOPS = 2500.0     # dense bf16 / fp16 MFMA


def decode_bytes(shape, plens, G):
    """Algorithmic HBM bytes of the G decode steps: weights once per step, plus per sequence the
    KV of every attended key read and the new token's KV written."""
    w = 2 * (shape.body_params() + shape.head_params())
    kvt = shape.kv_bytes_per_token()
    total = G * w
    for p in plens:
        for n in range(G):
            ctx = int(p) + n                       # keys attended at step n (prompt + n generated so far)
            total += (ctx + 1) * kvt               # read ctx keys/values, write one
    return total


def gemm_decode_bytes_per_step(shape, B):
    """Algorithmic bytes of the weight-streaming GEMMs of one decode step (weights + fp16 A rows in,
    fp16 / fp32 results out at their final width; split-K partials are overhead, not counted)."""
    d, F, V = shape.d_model, shape.d_ffn, shape.vocab
    qd = shape.n_q_heads * shape.head_dim
    per_layer_w = 2 * (shape.qkv_rows * d + d * qd + 2 * F * d + d * F)
    per_layer_act = 2 * B * (d + qd + d + F) + 2 * B * (shape.qkv_rows + F) + 4 * B * 2 * d
    return shape.n_layers * (per_layer_w + per_layer_act) + 2 * V * d + 2 * B * d + 4 * B * V


def attn_decode_bytes(shape, plens, G):
    kvt = shape.kv_bytes_per_token()
    return sum((int(p) + n) * kvt for p in plens for n in range(G))


def score_flops(shape, lens):
    """Algorithmic FLOP of one teacher-forced pass: 2*params per token (LM head only on scored
    positions) + causal attention (lower triangle only)."""
    f = 0.0
    for L in lens:
        L = int(L)
        f += 2.0 * shape.body_params() * L + 2.0 * shape.head_params() * max(L - 1, 0)
        f += shape.n_layers * 4.0 * shape.n_q_heads * shape.head_dim * (L * (L + 1) / 2.0)
    return f


def cpu_baseline(shape, wp, ids, prompt_len, seed, sample_P, sample_G, temperature, reps=5):
    """The CPU oracle, as it stands, on a bounded sample of the workload, both stages of the path: generation
    (row 0's first sample_P prompt tokens, sample_G generated tokens, with KV cache) and teacher-forced scoring of
    the resulting sample_P + sample_G tokens.  One warm-up and `reps` timed repetitions of each, mean and standard
    deviation.  Weights are handed over as float64 arrays (same values) so the timed regions hold the oracle's
    arithmetic only."""
    from oracle import rollout_oracle as O
    try:
        import threadpoolctl
        threads = max(int(i.get("num_threads", 1)) for i in threadpoolctl.threadpool_info()) or 1
    except Exception:
        threads = os.cpu_count() or 1
    w = {k: synth.to_numpy_f32(v).astype(np.float64) for k, v in wp.items() if k != "layers"}
    w["layers"] = [{k: synth.to_numpy_f32(v).astype(np.float64) for k, v in lw.items()} for lw in wp["layers"]]
    m = O.Model(shape, w)
    print("[bench] cpu oracle: weights converted, %d repetitions of generate + score" % (reps + 1), file=sys.stderr, flush=True)
    prompt = ids[0, :min(sample_P, int(prompt_len[0]))]
    tg, ts, toks = [], [], None
    for r in range(reps + 1):
        t0 = time.perf_counter()
        out, _ = O.generate(m, [prompt], sample_G, temperature, seed=seed)
        t1 = time.perf_counter()
        seq = np.concatenate([prompt, out[0]])
        O.score(m, seq)
        t2 = time.perf_counter()
        print("[bench] cpu oracle repetition %d: generate %.1f s, score %.1f s" % (r, t1 - t0, t2 - t1), file=sys.stderr, flush=True)
        if r > 0:                      # the first repetition is the warm-up
            tg.append(t1 - t0)
            ts.append(t2 - t1)
    n_sc = len(prompt) + sample_G
    gen_rate, sc_rate = sample_G / np.array(tg), n_sc / np.array(ts)
    return {"value": float(gen_rate.mean()), "unit": "generated tokens/s", "cores": threads, "kind": "oracle",
            "std": float(gen_rate.std()), "repetitions": reps,
            "scored_tok_s": float(sc_rate.mean()), "scored_tok_s_std": float(sc_rate.std()),
            "sample": f"row 0: first {len(prompt)} prompt tokens + {sample_G} generated tokens (float64 numpy oracle with "
                      f"KV cache, {np.mean(tg):.1f} s per repetition), then those {n_sc} tokens scored "
                      f"({np.mean(ts):.1f} s per repetition); 1 warm-up + {reps} repetitions each"}


def response_limits(Q, cap, seed):
    """Synthetic response lengths: log-normal body with a long tail, mean about 351 tokens (the mean the paper
    reports for its 70B actor's first PPO steps, Section 5.1's 405B paragraph), clipped to [16, cap]."""
    rng = np.random.default_rng(seed)
    x = rng.lognormal(mean=np.log(351.0) - 0.5 * 0.8 ** 2, sigma=0.8, size=Q)
    return np.clip(np.rint(x), 16, cap).astype(np.int32)


def queue_bench(args, wl, shape, ro, B, Pmax, Pmin, dev):
    """Useful generated tokens per second on a variable-length workload: dynamic slot refill against fixed
    batches of B that each run until their longest row is done (what a fixed-batch engine does)."""
    Q, Gcap = args.queue, args.gen or 1024
    ids_np, plen = synth.make_prompts(shape.vocab, Q, Pmax, Pmin, wl.prompt_seed)
    limit = response_limits(Q, Gcap, wl.sample_seed + 1)
    ids = torch.tensor(ids_np, device=dev)
    out = torch.zeros(Q, Gcap, dtype=torch.int32, device=dev)
    olen = torch.zeros(Q, dtype=torch.int32, device=dev)
    olp = torch.zeros(Q, Gcap, dtype=torch.float32, device=dev)
    sc = R.sample_cfg(wl.sample_seed, wl.temperature)
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    torch.cuda.set_stream(stream)
    useful = int(limit.sum())

    def run_queue():
        ro.rollout_generate_queue(sc, ids, plen, limit, Gcap, out, olen, olp)

    def run_fixed():
        for q0 in range(0, Q, B):
            n = min(B, Q - q0)
            G = int(limit[q0:q0 + n].max())
            sb = R.sample_cfg(wl.sample_seed, wl.temperature, -1, q0)
            ro.rollout_generate(sb, ids[q0:q0 + n], plen[q0:q0 + n], G, out[q0:q0 + n, :G].contiguous(), None, None)

    res = {}
    for name, fn in (("queue", run_queue), ("fixed_batches", run_fixed)):
        if args.warmup:
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        res[name] = (time.perf_counter() - t0) / args.steps
    ro.rollout_check()
    assert np.array_equal(olen.cpu().numpy(), limit)
    line = {
        "metric": "useful generated tokens/s, variable-length responses (1 GPU)",
        "value": useful / res["queue"], "unit": "generated tokens/s (prefill + decode, dynamic slot refill)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["queue"] * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 weights, fp16 activations/KV, fp32 accumulate", "data": "synthetic",
        "config": {"workload": args.workload + "_queue", "shape": shape.name, "layers": shape.n_layers, "prompts": Q,
                   "slots": B, "prompt": [int(plen.min()), int(plen.max())],
                   "response_limit": {"mean": float(limit.mean()), "p50": float(np.median(limit)),
                                      "max": int(limit.max()), "cap": Gcap}},
        "fixed_batches_tok_s": useful / res["fixed_batches"], "fixed_batches_s": res["fixed_batches"],
        "queue_s": res["queue"], "speedup_vs_fixed_batches": res["fixed_batches"] / res["queue"],
    }
    print(json.dumps(line))
    ro.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="8b", choices=sorted(synth.WORKLOADS))
    ap.add_argument("--layers", type=int, default=0, help="debug: fewer layers (marks the line reduced)")
    ap.add_argument("--batch", type=int, default=0, help="debug override")
    ap.add_argument("--prompt", type=int, default=0, help="debug override")
    ap.add_argument("--gen", type=int, default=0, help="debug override")
    ap.add_argument("--no-score", action="store_true", help="debug: skip scoring (marks the line reduced)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--impl", type=int, default=-1)
    ap.add_argument("--chunk", type=int, default=16384)
    ap.add_argument("--calib-copy", action="store_true",
                    help="first run three device copies of 1 GiB (read 1 GiB, write 1 GiB each): the known-size "
                         "kernel that HBM-traffic counters of a rocprofv3 --pmc run are scaled by")
    ap.add_argument("--kl-exact", action="store_true",
                    help="also time score_kl_exact (both bodies + the fused dual LM head) on the rollouts; extra key kl_exact_s")
    ap.add_argument("--queue", type=int, default=0, metavar="Q",
                    help="variable-length generation instead of the headline step: Q prompts with response limits "
                         "from a long-tailed distribution (mean about 351 tokens), run once through "
                         "rollout_generate_queue and once as fixed batches that wait for their longest row")
    ap.add_argument("--no-shadow", action="store_true",
                    help="do not give the policy a buffer for the library's fp16 copy (decode GEMMs then convert on the fly)")
    ap.add_argument("--decode-tile-rows", type=int, default=None,
                    help="measurement switch: decode GEMMs above this many rows use the 128 x 128 tile kernel (library default -1 = never)")
    ap.add_argument("--precise-layers", type=int, default=None,
                    help="measurement switch: layers carried as fp16 pairs (library default 1)")
    ap.add_argument("--no-large-gemm-copy", action="store_true",
                    help="measurement: the large-M GEMMs convert bf16 weights in the loop even where an fp16 copy exists")
    ap.add_argument("--separate-qkv-consumer", action="store_true",
                    help="measurement: a separate kernel sums, rotates and appends the decode QKV partial sums (default: decode attention does)")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="also time torch.matmul (the vendor library) on the layer's GEMM shapes, as context")
    ap.add_argument("--no-alt-decode", action="store_true",
                    help="skip the extra generation without the policy's fp16 copy (key decode_without_fp16_copy)")
    ap.add_argument("--progress", action="store_true", help="phase markers with elapsed time on stderr")
    ap.add_argument("--pin-gb", type=float, default=24.0, help="with --ref-host: most host memory to pin, in GB")
    ap.add_argument("--ref-host", action="store_true",
                    help="keep the reference weights in pinned host memory and stream them layer by layer while "
                         "scoring (the 70B configuration's residency); reported in config.reference")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)

    wl = synth.WORKLOADS[args.workload]
    shape = wl.shape
    reduced = False
    if args.layers:
        shape = synth.scaled_shape(shape, shape.name, n_layers=args.layers)
        reduced = True
    B = args.batch or wl.batch
    Pmax = args.prompt or wl.prompt_max
    Pmin = min(wl.prompt_min, Pmax) if not args.prompt else Pmax
    G = args.gen or wl.gen
    reduced = reduced or (B, Pmax, G) != (wl.batch, wl.prompt_max, wl.gen) or args.no_score
    dev = "cuda:0"
    torch.cuda.set_device(0)

    if args.calib_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    wp = synth.make_weights(shape, wl.policy_seed, dev)
    if args.queue and not args.gen:
        G = 1024                     # cap of the synthetic response lengths
    Lmax = Pmax + G
    cfg = R.make_cfg(shape, B, Lmax, max_chunk_tokens=max(Lmax, args.chunk))
    def policy_shadow(cfg):
        # a buffer for the library's fp16 copy of the policy, when a third of the free memory holds it (the KV pool,
        # the workspace and, without --ref-host, the reference weights are still to come)
        nb = R.rollout_weight_shadow_bytes(cfg)
        free, _ = torch.cuda.mem_get_info()
        if args.no_shadow or nb == 0 or nb > free // 3:
            return None
        return torch.empty(nb, dtype=torch.uint8, device=dev)

    if args.ref_host:
        # the reference never has to be device-resident: made one tensor at a time and moved to pinned host memory
        host_bytes = {"pinned": 0, "pageable": 0}

        def pin(t):
            # pinned up to --pin-gb (transfers from pinned memory overlap with compute); pageable beyond that:
            # a box may refuse to pin more, and a process does not reliably survive a refused allocation
            h = t.cpu()
            nb = h.numel() * h.element_size()
            if host_bytes["pinned"] + nb <= args.pin_gb * 1e9:
                host_bytes["pinned"] += nb
                return h.pin_memory()
            host_bytes["pageable"] += nb
            return h

        wr = {k: pin(v) for k, v in synth.make_globals(shape, wl.ref_seed, dev).items()}
        wr["layers"] = []
        for l in range(shape.n_layers):
            wr["layers"].append({k: pin(v) for k, v in synth.make_layer(shape, wl.ref_seed, l, dev).items()})
        torch.cuda.empty_cache()
        staging = torch.empty(R.rollout_weight_staging_bytes(cfg), dtype=torch.uint8, device=dev)
        Wp, Wr = R.Weights(wp, shadow=policy_shadow(cfg)), R.Weights(wr, staging=staging)
    else:
        wr = synth.make_weights(shape, wl.ref_seed, dev)
        # the frozen reference gets a copy of its own when there is room: its large-M GEMMs read it too
        Wp = R.Weights(wp, shadow=policy_shadow(cfg))
        Wr = R.Weights(wr, shadow=policy_shadow(cfg) if Wp.shadow is not None else None)
    if args.progress:
        print("[bench] weights ready", file=sys.stderr, flush=True)
    ro = R.Rollout(cfg, Wp, dev)
    if args.progress:
        torch.cuda.synchronize()
        print("[bench] context ready", file=sys.stderr, flush=True)
    if args.impl >= 0:
        ro.rollout_set_impl(args.impl)
    if args.decode_tile_rows is not None:
        R.rollout_set_decode_tile_rows(args.decode_tile_rows)
    if args.no_large_gemm_copy:
        R.rollout_set_large_gemm_copy(False)
    if args.precise_layers is not None:
        ro.rollout_set_precise_layers(args.precise_layers)
    if args.separate_qkv_consumer:
        ro.rollout_set_fused_qkv_consumer(False)
    if args.queue:
        return queue_bench(args, wl, shape, ro, B, Pmax, Pmin, dev)
    ids_np, plen = synth.make_prompts(shape.vocab, B, Pmax, Pmin, wl.prompt_seed)
    ids = torch.tensor(ids_np, device=dev)
    out_ids = torch.zeros(B, G, dtype=torch.int32, device=dev)
    out_lp = torch.zeros(B, G, dtype=torch.float32, device=dev)
    full = torch.zeros(B, Lmax, dtype=torch.int32, device=dev)
    seq_len = (plen + G).astype(np.int32)
    outs = [torch.zeros(B, Lmax, dtype=torch.float32, device=dev) for _ in range(4)]
    sc = R.sample_cfg(wl.sample_seed, wl.temperature)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]

    def assemble():
        # [prompt | generated] rows, ragged prompts packed to the left (device-side copies only)
        if Pmin == Pmax:
            full[:, :Pmax] = ids
            full[:, Pmax:] = out_ids
        else:
            for b in range(B):
                p = int(plen[b])
                full[b, :p] = ids[b, :p]
                full[b, p:p + G] = out_ids[b]

    t_start = time.perf_counter()

    def note(msg):
        # progress on stderr (the JSON line on stdout stays alone): long configurations are otherwise silent for minutes
        if args.progress:
            print("[bench %.0fs] %s" % (time.perf_counter() - t_start, msg), file=sys.stderr, flush=True)

    def one_step(timed):
        ev[0].record()
        if Wp.shadow is not None:
            ro.rollout_refresh_policy()      # a PPO step starts from updated weights: the fp16 copy is rebuilt, timed
            if args.progress:
                torch.cuda.synchronize()
                note("fp16 copy rebuilt")
        ro.rollout_generate(sc, ids, plen, G, out_ids, None, out_lp)
        ev[1].record()
        if args.progress:
            ev[1].synchronize()
            note("generated")
        if not args.no_score:
            assemble()
            ro.score_logprobs_kl(Wp, Wr, full, seq_len, plen, 0.003, *outs)
        ev[2].record()
        if args.progress:
            ev[2].synchronize()
            note("scored")

    # a non-default stream: rollout_generate then replays its decode step as a captured HIP graph
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    torch.cuda.set_stream(stream)

    def beat(msg):
        # one short line per step on stderr, always: a default run is otherwise silent for minutes (stdout keeps the JSON line alone)
        print("[bench %.0fs] %s" % (time.perf_counter() - t_start, msg), file=sys.stderr, flush=True)

    for i in range(args.warmup):
        one_step(False)
        ev[2].synchronize()
        beat("warm-up step %d of %d done" % (i + 1, args.warmup))
    torch.cuda.synchronize()
    ro.rollout_check()

    gen_ms, score_ms = [], []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step(True)
        ev[2].synchronize()
        gen_ms.append(ev[0].elapsed_time(ev[1]))
        score_ms.append(ev[1].elapsed_time(ev[2]))
        beat("step %d of %d: %.0f ms" % (i + 1, args.steps, gen_ms[-1] + score_ms[-1]))
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ro.rollout_check()

    # One more step of the same work with HIP events bracketing sampled kernel launches on the
    # launch stream (per-class average launch durations for the roofline).  With events on, the
    # decode step is launched kernel by kernel instead of as a captured graph, so this step is
    # kept out of `value`.
    prof_classes = {"gemm_decode": R.RL_K_GEMM_DECODE, "attn_decode": R.RL_K_ATTN_DECODE,
                    "gemm_prefill": R.RL_K_GEMM_PREFILL, "attn_prefill": R.RL_K_ATTN_PREFILL,
                    "lmhead_score": R.RL_K_LMHEAD_SCORE}
    launches_per_step = {"gemm_decode": G * (4 * shape.n_layers + 1), "attn_decode": G * shape.n_layers}
    import math
    for name, k in prof_classes.items():
        n = launches_per_step.get(name, 0)
        stride = max(1, -(-n // 6000))                           # sample evenly, stay under the event cap ...
        period = shape.n_layers if name == "attn_decode" else 4 * shape.n_layers + 1
        while math.gcd(stride, period) != 1:     # ... and visit every launch of a decode step equally often (the
            stride += 1                          # GEMM shapes differ, and so do the layers: the first carries fp16 pairs)
        ro.rollout_profile_enable(k, stride)
    one_step(False)
    torch.cuda.synchronize()
    prof = {}
    # an event pair with nothing between it does not read zero: that much is in every timed launch on top of the
    # kernel's own duration (which is what a tracer reports), so it is measured here and taken off
    event_overhead_ms = ro.rollout_profile_event_overhead(256)
    for name, k in prof_classes.items():
        ms, n = ro.rollout_profile_read(k)
        prof[name] = {"ms_timed_raw": ms, "ms_timed": max(ms - n * event_overhead_ms, 0.0), "launches_timed": n}
        ro.rollout_profile_enable(k, 0)

    # context for the MFMA-bound rooflines: what the matrix cores sustain on their own under this chip's power
    # management (random operands as in a real GEMM, and zeros), and optionally the vendor library's GEMM on the layer's
    # shapes with the same value distributions
    mfma_sustained = {"random_operands": ro.rollout_probe_mfma_rate(True), "zeros": ro.rollout_probe_mfma_rate(False)}
    vendor = None
    if args.vendor_gemm:
        vendor = {}
        Mv = min(args.chunk, 16384)
        nqkv = (shape.n_q_heads + 2 * shape.n_kv_heads) * shape.head_dim
        for name, (N_, K_) in {"qkv": (nqkv, shape.d_model), "o": (shape.d_model, shape.n_q_heads * shape.head_dim),
                               "gate_up": (2 * shape.d_ffn, shape.d_model), "down": (shape.d_model, shape.d_ffn)}.items():
            A_ = (torch.rand(Mv, K_, device=dev) * 2 - 1).to(torch.float16)
            W_ = ((torch.rand(N_, K_, device=dev) - 0.5) * 0.08).to(torch.float16)
            for _ in range(3):
                torch.matmul(A_, W_.t())
            e0_, e1_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0_.record()
            for _ in range(10):
                torch.matmul(A_, W_.t())
            e1_.record()
            e1_.synchronize()
            vendor[name] = {"M": Mv, "N": N_, "K": K_, "tflops": 2.0 * Mv * N_ * K_ * 10 / (e0_.elapsed_time(e1_) * 1e-3) / 1e12}
            del A_, W_

    # prompt prefill alone, to split generation time into prefill + decode loop
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ro.rollout_prefill(ids, plen)
    torch.cuda.synchronize()
    prefill_s = time.perf_counter() - t1

    ms_per_step = dt * 1e3 / args.steps
    gen_s = float(np.mean(gen_ms)) / 1e3
    score_s = float(np.mean(score_ms)) / 1e3
    decode_s = max(gen_s - prefill_s, 1e-9)
    dbytes = decode_bytes(shape, plen, G)
    decode_gbps = dbytes / decode_s / 1e9
    sflops = 2 * score_flops(shape, seq_len)
    score_tflops = sflops / score_s / 1e12 if not args.no_score else None

    kl_exact_s = None
    if args.kl_exact and not args.ref_host:
        klf = torch.zeros(B, Lmax, dtype=torch.float32, device=dev)
        ro.score_kl_exact(Wp, Wr, full, seq_len, plen, klf)       # warm
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ro.score_kl_exact(Wp, Wr, full, seq_len, plen, klf)
        torch.cuda.synchronize()
        kl_exact_s = time.perf_counter() - t1

    # The same generation without the policy's fp16 copy (the mode a policy that fills the device has to use): one
    # untimed-for-`value` run on a second context, reported beside the headline decode figures.
    no_copy = None
    if Wp.shadow is not None and not args.no_alt_decode:
        ro2 = R.Rollout(cfg, R.Weights(wp), dev)
        if args.precise_layers is not None:
            ro2.rollout_set_precise_layers(args.precise_layers)
        ro2.rollout_generate(sc, ids, plen, G, out_ids, None, out_lp)      # warm: captures the graph
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ro2.rollout_generate(sc, ids, plen, G, out_ids, None, out_lp)
        torch.cuda.synchronize()
        g2 = time.perf_counter() - t1
        d2 = max(g2 - prefill_s, 1e-9)
        no_copy = {"generate_s": g2, "decode_s": d2, "decode_tok_s": B * G / d2,
                   "decode_hbm_frac": dbytes / d2 / 1e9 / HBM_PEAK_GBPS}
        ro2.close()
        del ro2
        if not args.no_score and not args.no_large_gemm_copy:
            # and the scoring pass with the large-M GEMMs converting the bf16 weights themselves
            R.rollout_set_large_gemm_copy(False)
            assemble()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            ro.score_logprobs_kl(Wp, Wr, full, seq_len, plen, 0.003, *outs)
            torch.cuda.synchronize()
            s2 = time.perf_counter() - t1
            R.rollout_set_large_gemm_copy(True)
            no_copy["score_s"] = s2
            no_copy["score_mfma_frac"] = sflops / s2 / 1e12 / MFMA_PEAK_TFLOPS

    # ---- rooflines per kernel class: algorithmic work of the class in one step / time of its launches in one step
    def cls_ms(name):            # time of the class in one step: mean timed launch x launches per step
        p_ = prof[name]
        if not p_["launches_timed"]:
            return None, None
        avg = p_["ms_timed"] / p_["launches_timed"]
        n = launches_per_step.get(name, p_["launches_timed"])
        return avg, avg * n

    n_tok_scored = 2 * float(seq_len.sum()) if not args.no_score else 0.0
    n_tok_prefill = float(np.sum(plen - 1))
    attn_pairs = sum(int(L_) * (int(L_) + 1) / 2.0 for L_ in seq_len) * (2 if not args.no_score else 0) + \
        sum(int(p_ - 1) * int(p_) / 2.0 for p_ in plen)
    work = {
        "gemm_prefill": ("mfma", 2.0 * shape.body_params() * (n_tok_scored + n_tok_prefill) / 1e12, "TFLOP",
                         "large-M MFMA GEMMs of prefill and scoring (gemm_dma8_kernel 256x256 / gemm_mfma_kernel 128x128)"),
        "lmhead_score": ("mfma", 2.0 * shape.head_params() * max(n_tok_scored - 2 * B, 0) / 1e12, "TFLOP",
                         "LM head + log-sum-exp + target gather (MG_LSE epilogue)"),
        "attn_prefill": ("mfma", shape.n_layers * 4.0 * shape.n_q_heads * shape.head_dim * attn_pairs / 1e12, "TFLOP",
                         "causal prefill attention (attn_prefill_kernel)"),
        "gemm_decode": ("hbm", G * gemm_decode_bytes_per_step(shape, B) / 1e9, "GB",
                        "weight-streaming decode GEMMs (gemm_ring_kernel)"),
        "attn_decode": ("hbm", attn_decode_bytes(shape, plen, G) / 1e9, "GB",
                        "paged GQA decode attention (attn_decode_kernel)"),
    }
    traffic_db = {}
    try:
        traffic_db = json.load(open(os.path.join(ROOT, "profiles", "hbm_traffic.json")))
    except Exception:
        pass
    rl = []
    for name, (bound, amount, unit, desc) in work.items():
        avg, tot = cls_ms(name)
        if not tot or amount <= 0:
            continue
        peak = HBM_PEAK_GBPS if bound == "hbm" else MFMA_PEAK_TFLOPS
        achieved = amount / (tot * 1e-3)
        n = launches_per_step.get(name, prof[name]["launches_timed"])
        ent = {"kernel": desc, "class": name, "bound": bound, "achieved": achieved, "peak": peak,
               "unit": "GB/s" if bound == "hbm" else "TFLOP/s", "frac": achieved / peak,
               "avg_launch_ms": avg, "launches_per_step": n, "ms_per_step": tot,
               "algorithmic_per_launch": amount / n, "algorithmic_unit": unit, "traffic": None}
        if bound == "mfma":
            ent["frac_of_sustained_mfma"] = achieved / mfma_sustained["random_operands"]
        t = traffic_db.get(args.workload, {}).get(name)
        if t and not reduced and args.impl in (-1, 1) and not t.get("context_dependent"):
            # HBM-side bytes per launch from rocprofv3 counters (FETCH_SIZE + WRITE_SIZE, scaled by a copy of known
            # size), taken by the profile step that wrote profiles/hbm_traffic.json at the commit it names
            ent["traffic"] = t["bytes_per_launch"]
            ent["traffic_measured_at"] = traffic_db.get("commit")
        rl.append(ent)
    rl.sort(key=lambda e: -e["ms_per_step"])
    roofline = rl[0] if rl else None

    line = {
        "metric": "rollout gen tokens/s + decode HBM GB/s % peak, 8B shape batch 128 (1 GPU)",
        "value": B * G / (ms_per_step / 1e3),
        "unit": "generated tokens/s (whole step: generate + policy/reference scoring + KL)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 weights, fp16 activations/KV (fp16 pairs in layer 0), fp32 accumulate" if shape.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "shape": shape.name, "layers": shape.n_layers, "batch": B,
                   "prompt": [int(Pmin), int(Pmax)], "gen": G, "page_tokens": shape.page_tokens,
                   "temperature": wl.temperature, "reduced": reduced, "impl": args.impl,
                   "policy_fp16_copy": Wp.shadow is not None,
                   "reference_fp16_copy": getattr(Wr, "shadow", None) is not None,
                   "attention_consumes_qkv_partials": not args.separate_qkv_consumer,
                   "reference": ("host, streamed (%.0f GB pinned, %.0f GB pageable)" % (host_bytes["pinned"] / 1e9, host_bytes["pageable"] / 1e9)) if args.ref_host else "device"},
        "generate_s": gen_s, "prefill_s": prefill_s, "decode_s": decode_s, "score_s": score_s,
        "kl_exact_s": kl_exact_s,
        "decode_tok_s": B * G / decode_s, "generate_tok_s": B * G / gen_s,
        "decode_hbm_gbps": decode_gbps, "decode_hbm_frac": decode_gbps / HBM_PEAK_GBPS,
        "decode_without_fp16_copy": no_copy,
        "scored_tok_s": (2 * float(seq_len.sum()) / score_s) if not args.no_score else None,
        "score_tflops": score_tflops,
        "score_mfma_frac": (score_tflops / MFMA_PEAK_TFLOPS) if score_tflops else None,
        "kernel_classes": prof,
        "event_overhead_us": event_overhead_ms * 1e3,
        "mfma_sustained_tflops": mfma_sustained,
        "vendor_gemm": vendor,
        "roofline": roofline,
        "roofline_others": rl[1:],
        "host_cores": os.cpu_count(),
    }
    if not args.no_cpu:
        small = shape.body_params() < 5e9
        line["cpu_baseline"] = cpu_baseline(shape, wp, ids_np, plen, wl.sample_seed,
                                            64 if not small else 128, 8 if not small else 32, wl.temperature)
    else:
        line["cpu_baseline"] = None
    print(json.dumps(line))


if __name__ == "__main__":
    main()
