"""Estimator quality of the HIP path on synthetic attention, next to the paper's two reference
points: exact TopK attention (Sec. 2.1, Sec. 3.1) and oracle sampling estimation (Sec. 3.2), at
equal budget, and with / without the centering of Sec. 4.3 (the ablation of Sec. 5.3).

This reproduces the *shape* of the paper's error-versus-budget figures without its datasets: the
relative error |estimate - o| / |o| against exact attention o, averaged over query heads and over
independent random projectors.  The HIP path produces the LSH-sampled estimates; TopK, oracle
sampling and exact attention come from the CPU oracle.

    python -m tests.estimator_quality            (on a GPU machine; prints the tables)

Synthetic inputs (see paper_2410_16179_amd/workloads.py for the geometry): one query head per KV
head; "flat" heads take the workload's literal queries (attention nearly uniform), "peaked" heads
take queries aligned with a few centered keys (alpha = 24: a few keys hold most of the mass).
Values are either the workload's iid N(0, I) rows, or rows that depend on the attention score,
v_i = 0.3 g_i + 3 zscore(log w_i) 1/sqrt(d) (the situation of the paper's zoo example, where what
is averaged is correlated with how often it is drawn: the case in which TopK is biased).
"""
from __future__ import annotations

import math
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import magicpig_oracle as oracle  # noqa: E402
from paper_2410_16179_amd import workloads as wl  # noqa: E402


def make_heads(n, heads, shape, values, seed=0):
    """K, V [1, heads, n, 128], q [1, heads, 128], mu [1, heads, 128] (bf16-representable)."""
    w = wl.Workload("quality", 1, heads, heads, n, 8, 75, "bf16", (16,))
    Kc = np.empty((1, heads, n, 128), np.float32)
    Vc = np.empty_like(Kc)
    q = np.empty((1, heads, 128), np.float32)
    mu = np.empty((1, heads, 128), np.float32)
    for g in range(heads):
        Kc[0, g], Vc[0, g] = wl.keys_values(w, 0, g, seed)
        mu[0, g] = oracle.key_mean(Kc[0, g]).astype(np.float32)
        if shape == "flat":
            q[0, g] = wl.query(w, 0, g, Kc[0, g], seed)
        else:
            q[0, g] = wl.query(w, 0, g, Kc[0, g], seed, alpha=24.0, center=mu[0, g])
        if values == "score-correlated":
            z = np.log(oracle.attention_weights(q[0, g], Kc[0, g]))
            zs = (z - z.mean()) / z.std()
            Vc[0, g] = wl.store(0.3 * Vc[0, g] + 3.0 * np.outer(zs, np.full(128, 1.0 / math.sqrt(128))), "bf16")
    return w, Kc, Vc, q, mu


def hip_estimates(Kc, Vc, q, mu, K, L, seeds, use_mu=True):
    """The HIP path's outputs [seeds, heads, 128] and sample sizes [seeds, heads] over projector seeds."""
    import torch
    from tests.gpu_helpers import Session
    heads, n = Kc.shape[1], Kc.shape[2]
    outs, sizes = [], []
    for s in range(seeds):
        wcfg = wl.Workload("quality", 1, heads, heads, n, K, L, "bf16", (16,))
        W = wl.projector(wcfg, 1000 + s)
        ses = Session(K=K, L=L, dtype="bf16", Kc=Kc, Vc=Vc, q=q, W=W)
        ses.set_mu(mu if use_mu else None)
        ses.hash_keys()
        ses.hash_query()
        r = ses.attend(debug=True, cand_cap=1, with_counts=False)
        outs.append(r["out"][0])
        sizes.append(r["ncand"][0])
        del ses
        torch.cuda.empty_cache()
    return np.array(outs), np.array(sizes)


def study(n=16384, heads=4, seeds=6, pairs=((8, 75), (9, 120), (10, 150), (10, 220), (11, 300)),
          shapes=("flat", "peaked"), value_models=("iid", "score-correlated"), n_static=68, rng_seed=7):
    """Rows of {shape, values, K, L, budget, fraction, err_hip, err_topk, err_oracle_sampling, err_static}."""
    rng = np.random.default_rng(rng_seed)
    rows = []
    for shape in shapes:
        for values in value_models:
            w, Kc, Vc, q, mu = make_heads(n, heads, shape, values)
            exact = [oracle.exact_attention(q[0, g], Kc[0, g], Vc[0, g]) for g in range(heads)]
            for K, L in pairs:
                outs, sizes = hip_estimates(Kc, Vc, q, mu, K, L, seeds)
                e_hip, e_top, e_os, budgets = [], [], [], []
                for g in range(heads):
                    for s in range(seeds):
                        m = int(sizes[s, g]) + n_static            # keys whose K / V rows the step read
                        budgets.append(m)
                        e_hip.append(oracle.relative_error(outs[s, g], exact[g]))
                        e_top.append(oracle.relative_error(oracle.topk_attention(q[0, g], Kc[0, g], Vc[0, g], m)[0], exact[g]))
                        e_os.append(oracle.relative_error(
                            oracle.oracle_sampling_estimate(q[0, g], Kc[0, g], Vc[0, g], rng.random(m))[0], exact[g]))
                rows.append({"shape": shape, "values": values, "K": K, "L": L, "budget": float(np.mean(budgets)),
                             "fraction": float(np.mean(budgets)) / n, "err_hip": float(np.mean(e_hip)),
                             "err_topk": float(np.mean(e_top)), "err_oracle_sampling": float(np.mean(e_os))})
    return rows


def centering_ablation(n=16384, heads=4, seeds=8, K=10, L=150):
    """Sampled fraction and error of the HIP path with the keys centered (Sec. 4.3) and without."""
    out = {}
    w, Kc, Vc, q, mu = make_heads(n, heads, "flat", "score-correlated")
    exact = [oracle.exact_attention(q[0, g], Kc[0, g], Vc[0, g]) for g in range(heads)]
    for label, use_mu in (("centered", True), ("not centered", False)):
        outs, sizes = hip_estimates(Kc, Vc, q, mu, K, L, seeds, use_mu=use_mu)
        frac = sizes / float(n)
        err = [oracle.relative_error(outs[s, g], exact[g]) for g in range(heads) for s in range(seeds)]
        out[label] = {"fraction_mean": float(frac.mean()), "fraction_min": float(frac.min()),
                      "fraction_max": float(frac.max()), "share_below_0.1_percent": float((frac < 1e-3).mean()),
                      "err_hip": float(np.mean(err)), "expected_fraction_orthogonal": oracle.expected_budget(K, L)}
    return out


def format_rows(rows):
    lines = [f"{'attention':9s} {'values':17s} {'(K,L)':>9s} {'budget':>8s} {'fraction':>9s} {'HIP path':>9s} {'TopK':>8s} {'oracle smp':>10s}"]
    for r in rows:
        lines.append(f"{r['shape']:9s} {r['values']:17s} {'(%d,%d)' % (r['K'], r['L']):>9s} {r['budget']:8.0f} {r['fraction']:9.4f} "
                     f"{r['err_hip']:9.3f} {r['err_topk']:8.3f} {r['err_oracle_sampling']:10.3f}")
    return "\n".join(lines)


def main():
    rows = study()
    print("relative error against exact attention, 16384 keys, mean over 4 heads x 6 projectors;")
    print("TopK and oracle sampling at the budget (keys read) the HIP path used")
    print(format_rows(rows))
    ab = centering_ablation()
    print("\ncentering ablation, (K, L) = (10, 150), flat attention, 4 heads x 8 projectors")
    for label, v in ab.items():
        print(f"  {label:13s} sampled fraction mean {v['fraction_mean']:.4f} min {v['fraction_min']:.5f} max {v['fraction_max']:.4f}; "
              f"draws below 0.1 %: {v['share_below_0.1_percent']:.0%}; relative error {v['err_hip']:.3f}")
    print(f"  (App. E budget for orthogonal vectors: {ab['centered']['expected_fraction_orthogonal']:.4f})")


if __name__ == "__main__":
    main()
