"""Shared test helpers: oracle-side verification of GPU rollouts along the GPU's own trajectory."""
import numpy as np

from oracle import rollout_oracle as O


def verify_rollout(model, prompts, gpu_ids, gpu_logp, temperature, seed, seq_base, cdf_delta, logp_tol,
                   rows=None, steps=None):
    """Teacher-force the oracle with each GPU sequence and check every emitted token.

    Greedy: the GPU token must be the oracle arg-max wherever the oracle's top-2 logit
    margin exceeds 1e-3, else one of the oracle's top two.  Sampling: with the shared
    uniform u and the oracle CDF C, require C(g-1) - delta <= u < C(g) + delta.
    Returns dict(max_logp_err, exact_match_rate, n_checked).
    """
    B, G = gpu_ids.shape
    rows = range(B) if rows is None else rows
    max_err, exact, checked = 0.0, 0, 0
    for b in rows:
        p = np.asarray(prompts[b], np.int64)
        P = len(p)
        full = np.concatenate([p, gpu_ids[b].astype(np.int64)])
        z_all = O.forward_logits(model, full[:-1])
        for n in (range(G) if steps is None else steps):
            z = z_all[P - 1 + n]
            g = int(gpu_ids[b, n])
            lsm = O.log_softmax(z)
            if temperature == 0.0:
                order = np.argsort(-z, kind="stable")
                margin = z[order[0]] - z[order[1]]
                if margin > 1e-3:
                    assert g == int(np.argmax(z)), f"row {b} step {n}: gpu {g} != oracle argmax {int(np.argmax(z))} (margin {margin:.3e})"
                else:
                    assert g in (int(order[0]), int(order[1])), f"row {b} step {n}: gpu {g} not in oracle top-2"
                exact += int(g == int(np.argmax(z)))
            else:
                c = np.cumsum(np.exp(O.log_softmax(z / temperature)))
                u = O.hash_uniform(seed, seq_base + b, n)
                lo = c[g - 1] if g > 0 else 0.0
                hi = c[g]
                assert lo - cdf_delta <= u < hi + cdf_delta, \
                    f"row {b} step {n}: token {g} CDF [{lo:.7f},{hi:.7f}) vs u={u:.7f}"
                exact += int(g == O.pick_token(z, temperature, u))
            if gpu_logp is not None:
                err = abs(float(gpu_logp[b, n]) - float(lsm[g]))
                max_err = max(max_err, err)
                assert err <= logp_tol, f"row {b} step {n}: logp err {err:.3e} > {logp_tol}"
            checked += 1
    return {"max_logp_err": max_err, "exact_match_rate": exact / max(1, checked), "n_checked": checked}


def check_scores(lp_gpu, lr_gpu, kl_gpu, pen_gpu, oracle_out, tol, kl_coef):
    lp, lr, kl, pen = oracle_out
    errs = {
        "logp_policy": float(np.abs(lp_gpu - lp).max()),
        "logp_ref": float(np.abs(lr_gpu - lr).max()),
        "kl": float(np.abs(kl_gpu - kl).max()),
    }
    for k, v in errs.items():
        assert v <= tol, f"{k}: max abs err {v:.3e} > {tol}"
    if pen_gpu is not None:
        assert np.abs(pen_gpu - pen).max() <= tol * max(1.0, kl_coef)
    # structure: exact zeros wherever nothing is scored (the oracle is exactly 0 only there)
    assert np.all(lp_gpu[lp == 0.0] == 0.0) and np.all(lr_gpu[lr == 0.0] == 0.0)
    assert np.all(kl_gpu[(lp == 0.0)] == 0.0)
    return errs
