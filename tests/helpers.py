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


def tick(msg="."):
    """Progress mark of a long comparison (tests/conftest.py points this at the real stderr)."""


class LazyModel(O.Model):
    """The oracle's model with its layers handed over one at a time (float64 arrays of the same values, made
    from the torch tensors the GPU path holds), so that an 80-layer model never has to sit in host memory as
    float64.  `conv` turns a torch tensor into such an array."""

    def __init__(self, shape, w_torch, conv):
        super().__init__(shape, {k: conv(v, np.float32) for k, v in w_torch.items() if k != "layers"})
        self._wt, self._conv, self._at, self._cur = w_torch["layers"], conv, -1, None

    def layer(self, l):
        if l != self._at:
            tick()
            self._cur = None
            self._cur = {k: self._conv(v, np.float64) for k, v in self._wt[l].items()}
            self._at = l
        return self._cur


def check_row(model, seq, P, seed, row, gpu_logp_row, gen_ids_row=None, gen_logp_row=None, tol=2e-2, cdf_delta=1e-3,
              upto=None):
    """One full row against the oracle, teacher-forced over the row's own tokens: every scored position of
    gpu_logp_row (positions 1 .. len-1, or 1 .. upto-1) within tol; if the row's generated tokens are given, each
    inside the oracle's CDF bracket for the shared uniform (temperature 1), and the generation log-probs within
    tol.  Returns (oracle log-probs, stats)."""
    seq = np.asarray(seq, np.int64)
    n = len(seq) if upto is None else upto
    z = O.forward_logits(model, seq[:n - 1])
    want = np.zeros(n)
    stats = {}
    viol = []
    for t in range(n - 1):
        lsm = O.log_softmax(z[t])
        want[t + 1] = lsm[seq[t + 1]]
        if gen_ids_row is not None and t >= P - 1 and t - (P - 1) < len(gen_ids_row):
            k = t - (P - 1)
            c = np.cumsum(np.exp(lsm))
            u = O.hash_uniform(seed, row, k)
            g = int(gen_ids_row[k])
            lo = c[g - 1] if g > 0 else 0.0
            viol.append(max(lo - u, u - c[g], 0.0))
    err = np.abs(np.asarray(gpu_logp_row[:n], np.float64) - want)
    stats["rms"] = float(np.sqrt(np.mean(err[1:] ** 2)))
    stats["max"] = float(err.max())
    assert err.max() <= tol, f"row {row}: log-prob error {err.max():.3e} at position {int(err.argmax())}"
    if viol:
        stats["cdf_viol_max"] = float(np.max(viol))
        assert np.max(viol) < cdf_delta, f"row {row}: sampled token outside the oracle's CDF bracket by {np.max(viol):.3e}"
    if gen_logp_row is not None:
        G = len(gen_logp_row)
        ge = np.abs(np.asarray(gen_logp_row, np.float64)[:max(0, n - P)] - want[P:P + G])
        stats["gen_max"] = float(ge.max(initial=0.0))
        assert ge.max(initial=0.0) <= tol, f"row {row}: generation log-prob error {ge.max():.3e}"
    return want, stats
