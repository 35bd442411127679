"""The HIP path as an estimator (Sec. 4.1 "importance sampling"; Eq. "close form"): over
many independent projectors W the sampled-attention output scatters around exact attention,
its average over projectors is much closer to exact attention than a single draw (numerator
and denominator are unbiased, the ratio consistent), and more tables (a larger sample)
shrink the error.  Exact attention is the oracle's dense softmax; everything else runs on the
GPU through the C ABI."""
from __future__ import annotations

import numpy as np
import pytest
import torch

from paper_2410_16179_amd import binding as mp
from paper_2410_16179_amd import workloads as wl
from gpu_helpers import Session

pytestmark = pytest.mark.gpu


def estimator_errors(oracle, K, L, n_proj, alpha):
    w = wl.Workload("stat", 1, 8, 2, 4096, K, L, "bf16", (4,))
    data = wl.generate(w, seed=3, alpha=alpha)
    Kc, Vc, q = data["K"], data["V"], data["q"]
    mu = np.stack([[oracle.key_mean(Kc[0, g]) for g in range(2)]]).astype(np.float32)
    for h in range(w.n_q_heads):          # queries aligned with a few centered keys: peaked attention
        q[0, h] = wl.query(w, 0, h, Kc[0, h // w.group], 3, alpha, center=mu[0, h // w.group])
    exact = np.stack([oracle.exact_attention(q[0, h], Kc[0, h // w.group], Vc[0, h // w.group])
                      for h in range(w.n_q_heads)])
    s = Session(K=K, L=L, dtype="bf16", Kc=Kc, Vc=Vc, q=q, W=data["W"])
    s.set_mu(mu)
    outs, sizes = [], []
    for j in range(n_proj):
        W = wl.store(np.random.default_rng(1000 + j).standard_normal((128, K * L)), "bf16")
        s.W.copy_(torch.from_numpy(W).to(torch.bfloat16))
        s.hash_keys()
        s.hash_query()
        r = s.attend()
        outs.append(r["out"][0].astype(np.float64))
        sizes.append(r["ncand"][0].mean())
    outs = np.stack(outs)                                        # [n_proj, heads, 128]
    nrm = np.linalg.norm(exact, axis=1)
    single = np.linalg.norm(outs - exact[None], axis=2) / nrm    # relative error of each draw
    averaged = np.linalg.norm(outs.mean(axis=0) - exact, axis=1) / nrm
    return single.mean(), averaged.mean(), float(np.mean(sizes))


def test_average_over_projectors_approaches_exact_attention(oracle):
    n_proj = 48
    rows = []
    for K, L in ((8, 75), (8, 150), (8, 300)):
        single, averaged, size = estimator_errors(oracle, K, L, n_proj, alpha=16.0)
        rows.append((K, L, size, single, averaged))
        print(f"   (K,L)=({K},{L}): sample {size:.0f} of 4096 keys; relative error of one draw {single:.3f}, "
              f"of the average of {n_proj} draws {averaged:.3f}", flush=True)
    for K, L, size, single, averaged in rows:
        # independent unbiased draws average out like 1/sqrt(48) = 0.14; a systematic offset would not
        assert averaged < 0.3 * single
    # more tables at the same K: larger sample, smaller error
    assert rows[0][2] < rows[1][2] < rows[2][2]
    assert rows[2][3] < rows[0][3]
