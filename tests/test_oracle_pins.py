"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test is chosen so that a plausible mistake in the oracle (dropped term, wrong sign
or index, transposed operand, raw instead of centered keys) fails it.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.stats
import torch

HERE = os.path.dirname(os.path.abspath(__file__))


def golden():
    vals = {}
    with open(os.path.join(HERE, "golden", "paper_values.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split()
                vals[k] = float(v)
    return vals


def f32(rng, *shape):
    return rng.standard_normal(shape).astype(np.float32)


# ---- key centering vector, Sec. 4.3 "Data pre-processing" ------------------------------
def test_key_mean_hand_example_with_exact_rationals(oracle):
    # four keys of three coordinates; expected values written out by hand as exact fractions
    Kmat = np.array([[1.0, -2.0, 0.5],
                     [3.0, 4.0, 0.25],
                     [-1.0, 7.0, 0.125],
                     [5.0, -1.0, 0.0625]], np.float32)
    expected = [Fraction(8, 4), Fraction(8, 4), Fraction(15, 16) / 4]      # column sums / n
    got = oracle.key_mean(Kmat)
    assert got.dtype == np.float64 and got.shape == (3,)
    assert [Fraction(float(v)) for v in got] == expected                   # exact: dyadic values
    # one mean per coordinate over the keys, not one per key over the coordinates
    assert oracle.key_mean(np.ones((5, 2), np.float32) * np.array([1.0, 3.0], np.float32)).tolist() == [1.0, 3.0]


def test_key_mean_runs_over_every_key_with_divisor_n(oracle):
    # sink keys (first 4), the local window (last 64) and the keys in between all count, and the
    # divisor is the number of keys n: each alternative reading moves the expected value
    n, d, n_sink, n_local = 200, 4, 4, 64
    Kmat = np.zeros((n, d), np.float32)
    Kmat[:n_sink, 0] = 50.0                 # only the sink keys are non-zero in coordinate 0
    Kmat[n - n_local:, 1] = 25.0            # only the local window in coordinate 1
    Kmat[n_sink:n - n_local, 2] = 4.0       # only the LSH-eligible keys in coordinate 2
    Kmat[:, 3] = np.arange(n, dtype=np.float32)
    mu = oracle.key_mean(Kmat)
    assert mu[0] == 50.0 * n_sink / n       # would be 0 if sink keys were left out
    assert mu[1] == 25.0 * n_local / n      # would be 0 if the local window were left out
    assert mu[2] == 4.0 * (n - n_sink - n_local) / n    # would be 4 over the eligible keys only
    assert mu[3] == (n - 1) / 2.0           # (n-1)/2 with divisor n; n/2 with divisor n-1
    # against an independent routine on random data (math.fsum: correctly rounded column sums)
    rng = np.random.default_rng(7)
    R = f32(rng, 333, 5)
    ref = [math.fsum(float(x) for x in R[:, j]) / 333 for j in range(5)]
    np.testing.assert_allclose(oracle.key_mean(R), ref, rtol=1e-14)
    # float32 inputs are averaged in float64: a float32 running sum would lose the small terms
    big = np.array([[2.0 ** 24], [1.0], [1.0], [-(2.0 ** 24)]], np.float32)
    assert oracle.key_mean(big)[0] == 0.5


def test_key_mean_of_no_keys_is_zero(oracle):
    mu = oracle.key_mean(np.zeros((0, 128), np.float32))
    assert mu.shape == (128,) and not mu.any()


def test_decode_step_centers_with_the_mean_of_all_keys(oracle):
    # decode_step without an explicit mu must use key_mean over all n keys, rounded to float32
    rng = np.random.default_rng(11)
    Kc = f32(rng, 1, 1, 90, 8) + np.float32(3.0)
    Vc = f32(rng, 1, 1, 90, 8)
    q = f32(rng, 1, 1, 8)
    W = f32(rng, 8, 12)
    r = oracle.decode_step(q, Kc, Vc, W, 3, 4, n_sink=2, n_local=5)
    hand = (Kc[0, 0].astype(np.float64).sum(axis=0) / 90).astype(np.float32)
    np.testing.assert_array_equal(r["mu"][0, 0], hand)
    np.testing.assert_array_equal(r["key_codes"][0, 0], oracle.hash_keys(Kc[0, 0], W, hand, 3, 4))


# ---- TopK attention (Sec. 2.1) and oracle sampling estimation (Sec. 3.2) -----------------
def zoo():
    """The zoo example of App. "TopK vs. Sampling" as an attention problem: 73 keys whose attention
    scores are the probabilities of the kinds (head dimension 1, logit = log probability), values =
    daily food."""
    w = np.array([0.1, 0.1, 0.1] + [0.01] * 70)
    food = np.array([50.0, 20.0, 10.0] + [1.0] * 70)
    return np.ones(1), np.log(w)[:, None], food[:, None], w


def test_zoo_example_true_average_and_topk(oracle):
    g = golden()
    q, K, V, w = zoo()
    np.testing.assert_allclose(oracle.attention_weights(q, K), w, rtol=1e-12)
    assert abs(oracle.exact_attention(q, K, V)[0] - g["zoo_true_average"]) < 1e-12
    t10, sel10 = oracle.topk_attention(q, K, V, 10)
    t20, sel20 = oracle.topk_attention(q, K, V, 20)
    assert abs(t10[0] - 807.0 / 37.0) < 1e-12 and round(t10[0]) == g["zoo_topk_10"]
    assert abs(t20[0] - 817.0 / 47.0) < 1e-12 and round(t20[0]) == g["zoo_topk_20"]
    assert sel10.tolist() == list(range(10)) and sel20.size == 20      # ties: the lower indices
    # the whole context is exact attention; nothing selected is the zero vector
    assert abs(oracle.topk_attention(q, K, V, 73)[0][0] - g["zoo_true_average"]) < 1e-12
    assert oracle.topk_attention(q, K, V, 0)[0][0] == 0.0


def test_zoo_example_sampling_is_unbiased_with_the_printed_spread(oracle):
    g = golden()
    q, K, V, w = zoo()
    rng = np.random.default_rng(2024)
    trials = 200_000
    for budget, key in ((10, "zoo_sampling_std_10"), (20, "zoo_sampling_std_20")):
        est = np.array([oracle.oracle_sampling_estimate(q, K, V, rng.random(budget))[0][0] for _ in range(trials)])
        std = est.std()
        assert abs(est.mean() - g["zoo_true_average"]) < 4 * std / math.sqrt(trials)     # unbiased
        assert abs(std - g[key]) < 0.07                        # 4.7 / 3.4 as printed (two digits) + Monte-Carlo noise
        assert round(math.sqrt(oracle.oracle_sampling_trace_of_covariance(q, K, V, budget)), 1) == g[key]
        # Theorem on oracle sampling, proof: Tr Cov = (E|v|^2 - |o|^2) / B = 225.01 / B here
        assert abs(oracle.oracle_sampling_trace_of_covariance(q, K, V, budget) - 225.01 / budget) < 1e-9
        assert abs(std ** 2 - 225.01 / budget) < 0.02 * 225.01 / budget


def test_topk_against_a_sorted_brute_force(oracle):
    rng = np.random.default_rng(5)
    n, d = 57, 6
    q, K, V = f32(rng, d), f32(rng, n, d), f32(rng, n, d)
    z = [(sum(float(a) * float(b) for a, b in zip(K[i], q)) / math.sqrt(d), i) for i in range(n)]
    for m in (1, 2, 13, 56, 57, 80):
        best = sorted(z, key=lambda t: (-t[0], t[1]))[:min(m, n)]
        mx = max(t[0] for t in best)
        den = sum(math.exp(t[0] - mx) for t in best)
        want = [sum(math.exp(t[0] - mx) / den * float(V[t[1], j]) for t in best) for j in range(d)]
        got, sel = oracle.topk_attention(q, K, V, m)
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)
        assert sel.tolist() == sorted(t[1] for t in best)
    np.testing.assert_allclose(oracle.topk_attention(q, K, V, n)[0], oracle.exact_attention(q, K, V), rtol=1e-12)
    # the selection keeps the largest scores: every kept score >= every dropped one
    w = oracle.attention_weights(q, K)
    _, sel = oracle.topk_attention(q, K, V, 20)
    assert w[sel].min() >= np.delete(w, sel).max()


def test_oracle_sampling_draws_from_the_attention_distribution(oracle):
    # three keys with scores 0.2, 0.3, 0.5: the uniforms select by the cumulative distribution
    q = np.ones(1)
    K = np.log(np.array([0.2, 0.3, 0.5]))[:, None]
    V = np.array([[1.0, 0.0], [0.0, 1.0], [4.0, 4.0]])
    est, idx = oracle.oracle_sampling_estimate(q, K, V, [0.0, 0.19, 0.21, 0.49, 0.51, 0.999])
    assert idx.tolist() == [0, 0, 1, 1, 2, 2]
    np.testing.assert_allclose(est, [(1 + 1 + 4 + 4) / 6.0, (1 + 1 + 4 + 4) / 6.0])
    assert oracle.oracle_sampling_estimate(q, K, V, [])[0].tolist() == [0.0, 0.0]
    # unbiased in every coordinate; Tr Cov = (E|v|^2 - |o|^2) / B, falling as 1 / B; the number of
    # unique draws has mean n - sum (1 - w_i)^B <= 1 + B (1 - max w)  (both theorems of Sec. 3.2)
    rng = np.random.default_rng(9)
    n, d = 40, 3
    qq, KK, VV = f32(rng, d), 2.0 * f32(rng, n, d), f32(rng, n, d)
    w = oracle.attention_weights(qq, KK)
    o = oracle.exact_attention(qq, KK, VV)
    trials, last = 40_000, None
    for budget in (4, 16, 64):
        runs = [oracle.oracle_sampling_estimate(qq, KK, VV, rng.random(budget)) for _ in range(trials)]
        est = np.array([r[0] for r in runs])
        tr = est.var(axis=0).sum()
        want = oracle.oracle_sampling_trace_of_covariance(qq, KK, VV, budget)
        assert abs(want - (float(w @ (VV.astype(np.float64) ** 2).sum(axis=1)) - float(o @ o)) / budget) < 1e-12
        assert np.all(np.abs(est.mean(axis=0) - o) < 4 * est.std(axis=0) / math.sqrt(trials))
        assert abs(tr - want) < 0.05 * want
        assert last is None or tr < last
        last = tr
        uniq = np.mean([np.unique(r[1]).size for r in runs])
        expect = n - ((1.0 - w) ** budget).sum()
        assert abs(uniq - expect) < 0.02 * expect
        assert expect <= 1 + budget * (1 - w.max()) + 1e-12
    assert oracle.relative_error([3.0, 4.0], [0.0, 0.0 + 5.0]) == pytest.approx(math.sqrt(9 + 1) / 5)


# ---- P1: per-hyperplane agreement probability, Sec. 2.2 -------------------------------
@pytest.mark.parametrize("deg", [30, 60, 90, 120, 150])
def test_agreement_probability_matches_empirical_hyperplanes(oracle, deg):
    rng = np.random.default_rng(100 + deg)
    d, draws = 16, 1_000_000
    th = math.radians(deg)
    a = np.zeros(d, np.float32); a[0] = 1.0
    b = np.zeros(d, np.float32); b[0] = np.float32(math.cos(th)); b[1] = np.float32(math.sin(th))
    W = f32(rng, d, draws)
    bits = oracle.simhash_bits(np.stack([a, b]), W)
    freq = (bits[0] == bits[1]).mean()
    cos = float(np.dot(a.astype(np.float64), b.astype(np.float64)) /
                (np.linalg.norm(a.astype(np.float64)) * np.linalg.norm(b.astype(np.float64))))
    p = float(oracle.agreement_probability(cos))
    assert abs(p - (1 - th / math.pi)) < 1e-6          # closed form, float32-rounded b
    sigma = math.sqrt(p * (1 - p) / draws)
    assert abs(freq - p) < 4 * sigma


def test_agreement_value_printed_form(oracle):
    assert abs(float(oracle.agreement_probability(0.5)) - golden()["agreement_at_60deg"]) < 1e-15
    assert float(oracle.agreement_probability(1.0)) == 1.0
    assert float(oracle.agreement_probability(-1.0)) == 0.0
    assert float(oracle.agreement_probability(3.0)) == 1.0     # clamped


# ---- P2: inclusion probability, Eq. "lsh sampling probability" -------------------------
def exact_tail(x: float, L: int, tau: int) -> float:
    xf = Fraction(x)
    return float(sum(math.comb(L, j) * xf ** j * (1 - xf) ** (L - j) for j in range(tau, L + 1)))


@pytest.mark.parametrize("K,L", [(10, 150), (8, 75), (9, 120), (10, 170), (3, 7), (1, 1)])
def test_inclusion_probability_vs_exact_rational_and_scipy(oracle, K, L):
    cs = np.array([-1.0, -0.9, -0.5, -0.2, 0.0, 0.2, 0.5, 0.8, 0.95, 0.999, 1.0])
    p = oracle.agreement_probability(cs)
    for tau in (1, 2, 3):
        if tau > L:
            continue
        u = oracle.inclusion_probability(p, K, L, tau)
        ref = np.array([exact_tail(float(pi) ** K, L, tau) for pi in p])
        np.testing.assert_allclose(u, ref, rtol=1e-10, atol=1e-300)
        sf = scipy.stats.binom.sf(tau - 1, L, p ** K)
        np.testing.assert_allclose(u, sf, rtol=1e-8, atol=1e-300)


def test_inclusion_probability_equals_printed_formula_where_well_conditioned(oracle):
    for K, L in [(10, 150), (9, 120), (8, 75)]:
        p = np.linspace(0.5, 1.0, 101)
        x = p ** K
        printed = 1 - (1 - x) ** L - L * x * (1 - x) ** (L - 1)
        u = oracle.inclusion_probability(p, K, L, 2)
        ok = printed > 1e-3          # the printed form loses digits below that
        np.testing.assert_allclose(u[ok], printed[ok], rtol=1e-9)


def test_inclusion_probability_special_cases(oracle):
    p = np.array([0.0, 0.3, 0.7, 1.0])
    np.testing.assert_allclose(oracle.inclusion_probability(p, 1, 1, 1), p, rtol=1e-14)
    np.testing.assert_array_equal(oracle.inclusion_probability(p, 5, 9, 0), np.ones(4))
    # one table can never give two hits
    np.testing.assert_array_equal(oracle.inclusion_probability(p, 2, 1, 2), np.zeros(4))
    # monotone in p
    u = oracle.inclusion_probability(np.linspace(0, 1, 300), 10, 150, 2)
    assert np.all(np.diff(u) >= 0) and u[0] == 0.0 and u[-1] == 1.0


# ---- P3: budget for orthogonal vectors, App. E Eq. "budget" ----------------------------
def test_expected_budget_values(oracle):
    g = golden()
    for K, L in [(10, 150), (8, 75), (9, 120), (10, 170)]:
        assert abs(oracle.expected_budget(K, L) - g[f"budget_K{K}_L{L}"]) < 1e-12
        # cos = 0 gives p = 1/2, and the inclusion probability must reduce to the budget
        u = float(oracle.inclusion_probability(oracle.agreement_probability(0.0), K, L, 2))
        assert abs(u - g[f"budget_K{K}_L{L}"]) < 1e-12


@pytest.mark.parametrize("K,L,seeds", [(4, 20, 40), (8, 75, 24)])
def test_sampled_fraction_of_orthogonal_keys_matches_budget(oracle, K, L, seeds):
    d, n = 32, 3000
    rng = np.random.default_rng(7)
    q = np.zeros(d, np.float32); q[0] = 3.0
    keys = f32(rng, n, d); keys[:, 0] = 0.0          # exactly orthogonal to q
    hits = 0
    for s in range(seeds):
        W = f32(np.random.default_rng(1000 + s), d, K * L)
        kc = oracle.hash_keys(keys, W, None, K, L)
        qc = oracle.hash_query(q, W, K, L)[0]
        S = oracle.sample_set(oracle.collision_counts(qc, kc), 0, 0, 2)
        hits += S.size
    frac = hits / (n * seeds)
    bud = oracle.expected_budget(K, L)
    # keys under one projector share the query's code, so allow for that correlation:
    # the per-projector fraction has a standard deviation measured to be well under 30 %
    # of the budget at these sizes; the mean over `seeds` projectors is far tighter.
    assert abs(frac - bud) < 0.15 * bud


# ---- P4: every key sampled with u = 1 -> exact softmax attention -----------------------
def sdpa64(q, K, V):
    out = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q.astype(np.float64))[None, None, None, :],
        torch.from_numpy(K.astype(np.float64))[None, None],
        torch.from_numpy(V.astype(np.float64))[None, None])
    return out[0, 0, 0].numpy()


def test_exact_attention_is_textbook(oracle):
    rng = np.random.default_rng(3)
    q, K, V = f32(rng, 16), f32(rng, 50, 16), f32(rng, 50, 16)
    np.testing.assert_allclose(oracle.exact_attention(q, K, V), sdpa64(q, K, V), rtol=1e-12, atol=1e-14)


def test_min_hits_zero_recovers_exact_attention(oracle):
    rng = np.random.default_rng(4)
    d, n, K, L = 16, 200, 4, 12
    q = f32(rng, 1, 1, d); Kc = f32(rng, 1, 1, n, d) + 2.0; Vc = f32(rng, 1, 1, n, d)
    W = f32(rng, d, K * L)
    r = oracle.decode_step(q, Kc, Vc, W, K, L, min_hits=0, n_sink=4, n_local=16)
    np.testing.assert_allclose(r["out"][0, 0], sdpa64(q[0, 0], Kc[0, 0], Vc[0, 0]), rtol=1e-12, atol=1e-14)
    assert r["S"][0][0].size == n - 20


def test_keys_parallel_to_query_are_all_sampled_with_u_one(oracle):
    rng = np.random.default_rng(5)
    d, n, K, L = 16, 64, 6, 10
    q = f32(rng, d)
    scales = (2.0 ** rng.integers(-3, 4, size=n)).astype(np.float32)   # exact scalings
    Kmat = scales[:, None] * q[None, :]
    V = f32(rng, n, d)
    W = f32(rng, d, K * L)
    r = oracle.decode_step(q[None, None], Kmat[None, None], V[None, None], W, K, L,
                           mu=np.zeros((1, 1, d), np.float32), min_hits=2, n_sink=0, n_local=0)
    assert np.all(r["counts"][0, 0] == L)
    assert r["S"][0][0].size == n
    np.testing.assert_allclose(r["out"][0, 0], sdpa64(q, Kmat, V), rtol=1e-11, atol=1e-13)


def test_static_tokens_only_when_context_is_short(oracle):
    rng = np.random.default_rng(6)
    d, n, K, L = 8, 10, 3, 5
    q = f32(rng, 1, 1, d); Kc = f32(rng, 1, 1, n, d); Vc = f32(rng, 1, 1, n, d)
    r = oracle.decode_step(q, Kc, Vc, f32(rng, d, K * L), K, L, n_sink=4, n_local=64)
    assert r["S"][0][0].size == 0
    np.testing.assert_allclose(r["out"][0, 0], sdpa64(q[0, 0], Kc[0, 0], Vc[0, 0]), rtol=1e-12)
    # no keys at all: defined as the zero vector
    r0 = oracle.decode_step(q, Kc[:, :, :0], Vc[:, :, :0], f32(rng, d, K * L), K, L)
    assert np.all(r0["out"] == 0)


# ---- P5: Monte Carlo over projectors ----------------------------------------------------
def _mc_setup(K, L, seeds, with_mean, rng_seed=11):
    rng = np.random.default_rng(rng_seed)
    d, n = 8, 32
    keys = f32(rng, n, d)
    if with_mean:
        keys = (keys + np.float32(1.5) * f32(rng, 1, d)).astype(np.float32)
    q = f32(rng, d)
    V = f32(rng, n, d)
    W = f32(np.random.default_rng(rng_seed + 1), d, seeds * K * L)
    return d, n, keys, q, V, W


def _mc_indicators(oracle, K, L, seeds, keys, q, W, mu):
    n = keys.shape[0]
    kc = oracle.table_codes(oracle.simhash_bits(keys, W, mu), K, seeds * L).reshape(n, seeds, L)
    qc = oracle.table_codes(oracle.simhash_bits(q, W, None), K, seeds * L).reshape(seeds, L)
    ind = np.zeros((seeds, n), bool)
    for s in range(seeds):
        cnt = oracle.collision_counts(qc[s], kc[:, s, :])
        ind[s, oracle.sample_set(cnt, 0, 0, 2)] = True
    return ind


@pytest.mark.parametrize("K,L", [(2, 6), (3, 10)])
def test_inclusion_frequency_and_unbiased_sums(oracle, K, L):
    seeds = 60_000
    d, n, keys, q, V, W = _mc_setup(K, L, seeds, with_mean=True)
    mu = oracle.key_mean(keys).astype(np.float32)
    ind = _mc_indicators(oracle, K, L, seeds, keys, q, W, mu)
    freq = ind.mean(axis=0)
    kc64 = keys.astype(np.float64) - mu.astype(np.float64)
    u = oracle.inclusion_probability(
        oracle.agreement_probability(oracle.cosine_to_centered_keys(q, kc64)), K, L, 2)
    sigma = np.sqrt(u * (1 - u) / seeds)
    assert np.all(np.abs(freq - u) < 4.5 * sigma + 1e-12)
    # the same check with the *raw* keys' cosine must fail: the hashed vectors are the
    # centered ones, which is what decides how cos(theta) in u_i is to be read.
    u_raw = oracle.inclusion_probability(
        oracle.agreement_probability(oracle.cosine_to_centered_keys(q, keys.astype(np.float64))), K, L, 2)
    assert np.any(np.abs(freq - u_raw) > 8 * np.sqrt(u_raw * (1 - u_raw) / seeds))
    # numerator and denominator of the estimator are each unbiased (Horvitz-Thompson)
    wt = np.exp(keys.astype(np.float64) @ q.astype(np.float64) / math.sqrt(d))
    terms = wt / u                                     # [n]
    den = (ind * terms[None, :]).sum(axis=1)           # [seeds]
    num = (ind * terms[None, :]) @ V.astype(np.float64)  # [seeds, d]
    Z = wt.sum()
    assert abs(den.mean() - Z) < 4.5 * den.std() / math.sqrt(seeds)
    target = wt @ V.astype(np.float64)
    assert np.all(np.abs(num.mean(axis=0) - target) < 4.5 * num.std(axis=0) / math.sqrt(seeds))


def test_ratio_estimator_bias_shrinks_with_more_tables(oracle):
    K = 2
    errs = []
    for L in (4, 16, 64):
        seeds = 4000
        d, n, keys, q, V, W = _mc_setup(K, L, seeds, with_mean=False, rng_seed=21)
        ind = _mc_indicators(oracle, K, L, seeds, keys, q, W, None)
        exact = oracle.exact_attention(q, keys, V)
        T = np.zeros(0, np.int64)
        outs = [oracle.estimator_from_sample(q, keys, V, None, np.nonzero(ind[s])[0], T, K, L, 2)
                for s in range(seeds) if ind[s].any()]
        errs.append(np.linalg.norm(np.mean(outs, axis=0) - exact))
    assert errs[2] < errs[0] and errs[2] < 0.02 * np.linalg.norm(exact) + 1e-3


# ---- P6: brute force ----------------------------------------------------------------------
def test_counts_and_sample_against_brute_force(oracle):
    rng = np.random.default_rng(8)
    d, n, K, L, s, l, tau = 8, 90, 2, 9, 3, 7, 2
    keys = f32(rng, n, d); q = f32(rng, d); W = f32(rng, d, K * L)
    mu = oracle.key_mean(keys).astype(np.float32)
    kc = oracle.hash_keys(keys, W, mu, K, L)
    qc = oracle.hash_query(q, W, K, L)[0]
    counts = oracle.collision_counts(qc, kc)
    S = oracle.sample_set(counts, s, l, tau)
    Wd = W.astype(np.float64)
    exp_counts, exp_S = [], []
    for i in range(n):
        c = 0
        for t in range(L):
            same = True
            for b in range(K):
                col = Wd[:, t * K + b]
                kb = sum((float(keys[i, e]) - float(mu[e])) * col[e] for e in range(d)) >= 0
                qb = sum(float(q[e]) * col[e] for e in range(d)) >= 0
                same = same and (kb == qb)
            c += same
        exp_counts.append(c)
        if s <= i < n - l and c >= tau:
            exp_S.append(i)
    assert counts.tolist() == exp_counts
    assert S.tolist() == exp_S
    # canonical code integer: bit b of table t has weight 2^b, column index t*K + b
    bits = oracle.simhash_bits(keys[:1], W, mu)[0]
    assert kc[0, 4] == sum(int(bits[4 * K + b]) << b for b in range(K))


def test_estimator_against_hand_written_sum(oracle):
    rng = np.random.default_rng(9)
    d, n, K, L = 4, 12, 2, 5
    keys = f32(rng, n, d); V = f32(rng, n, d); q = f32(rng, d)
    mu = oracle.key_mean(keys).astype(np.float32)
    S = np.array([2, 5, 7]); T = np.array([0, 11])
    out = oracle.estimator_from_sample(q, keys, V, mu, S, T, K, L, 2)
    num = np.zeros(d); den = 0.0
    for i in list(S) + list(T):
        w = math.exp(sum(float(q[e]) * float(keys[i, e]) for e in range(d)) / math.sqrt(d))
        if i in S:
            kc = [float(keys[i, e]) - float(mu[e]) for e in range(d)]
            c = sum(float(q[e]) * kc[e] for e in range(d)) / (
                math.sqrt(sum(float(x) ** 2 for x in q)) * math.sqrt(sum(x * x for x in kc)))
            x = (1 - math.acos(c) / math.pi) ** K
            u = 1 - (1 - x) ** L - L * x * (1 - x) ** (L - 1)
            w /= u
        num += w * V[i].astype(np.float64); den += w
    np.testing.assert_allclose(out, num / den, rtol=1e-10)


# ---- exact sign ------------------------------------------------------------------------------
def test_sign_is_that_of_the_exact_sum(oracle):
    big, tiny = np.float32(2.0 ** 40), np.float32(2.0 ** -40)
    x = np.array([[-tiny, big, -big, 0], [tiny, big, -big, 0], [0, 0, 0, 0],
                  [big, -big, 0, -tiny]], np.float32)
    W = np.ones((4, 1), np.float32)
    assert oracle.simhash_bits(x, W).ravel().tolist() == [False, True, True, False]
    # centering is applied exactly too: x - mu = -2^-40 although fl(x.W) == fl(mu.W)
    x2 = np.array([[big, 0, 0, 0]], np.float32)
    mu = np.array([big, tiny, 0, 0], np.float32)
    assert oracle.simhash_bits(x2, W, mu).ravel().tolist() == [False]
    assert oracle.simhash_bits(x2, W, np.array([big, -tiny, 0, 0], np.float32)).ravel().tolist() == [True]


# ---- P7: invariants -------------------------------------------------------------------------------
def test_invariants(oracle):
    rng = np.random.default_rng(10)
    d, n, K, L = 16, 300, 4, 24
    q = f32(rng, 1, 1, d); Kc = f32(rng, 1, 1, n, d) + 1.0; Vc = f32(rng, 1, 1, n, d)
    W = f32(rng, d, K * L)
    mu = oracle.key_mean(Kc[0, 0]).astype(np.float32)[None, None]
    r = oracle.decode_step(q, Kc, Vc, W, K, L, mu=mu, n_sink=4, n_local=16)
    cnt, S = r["counts"][0, 0], r["S"][0][0]
    assert cnt.min() >= 0 and cnt.max() <= L
    T = oracle.static_set(n, 4, 16)
    assert not set(S.tolist()) & set(T.tolist())
    # positive power-of-two scaling of q leaves its codes unchanged; scaling k and mu too
    np.testing.assert_array_equal(oracle.hash_query(4 * q[0, 0], W, K, L), r["q_codes"][0])
    np.testing.assert_array_equal(oracle.hash_keys(2 * Kc[0, 0], W, 2 * mu[0, 0], K, L), r["key_codes"][0, 0])
    # permuting keys permutes counts; earlier codes do not depend on later keys
    perm = rng.permutation(n)
    np.testing.assert_array_equal(
        oracle.collision_counts(r["q_codes"][0, 0], r["key_codes"][0, 0][perm]), cnt[perm])
    np.testing.assert_array_equal(oracle.hash_keys(Kc[0, 0, :100], W, mu[0, 0], K, L), r["key_codes"][0, 0, :100])
    # adding a constant vector to V adds it to the output; output is a convex combination
    cvec = f32(rng, d)
    r2 = oracle.decode_step(q, Kc, (Vc + cvec).astype(np.float32), W, K, L, mu=mu, n_sink=4, n_local=16)
    Vshift = (Vc + cvec).astype(np.float32).astype(np.float64) - Vc.astype(np.float64)
    np.testing.assert_allclose(r2["out"][0, 0] - r["out"][0, 0], Vshift[0, 0, 0], rtol=0, atol=1e-6)
    used = np.concatenate([S, T])
    vmin, vmax = Vc[0, 0, used].min(axis=0), Vc[0, 0, used].max(axis=0)
    assert np.all(r["out"][0, 0] >= vmin - 1e-12) and np.all(r["out"][0, 0] <= vmax + 1e-12)
    # shifting every key by the same vector (and mu with it) changes neither sample nor output
    shift = np.float32(0.5) * np.ones(d, np.float32)
    r3 = oracle.decode_step(q, (Kc + shift).astype(np.float32), Vc, W, K, L,
                            mu=(mu + shift).astype(np.float32), n_sink=4, n_local=16)
    if np.array_equal((Kc + shift).astype(np.float64) - (mu + shift).astype(np.float64),
                      Kc.astype(np.float64) - mu.astype(np.float64)):
        np.testing.assert_array_equal(r3["counts"], r["counts"])
        np.testing.assert_allclose(r3["out"], r["out"], rtol=1e-9)


def test_gqa_heads_use_their_kv_head(oracle):
    rng = np.random.default_rng(12)
    d, n, K, L = 8, 80, 3, 12
    q = f32(rng, 1, 4, d); Kc = f32(rng, 1, 2, n, d); Vc = f32(rng, 1, 2, n, d)
    W = f32(rng, d, K * L)
    r = oracle.decode_step(q, Kc, Vc, W, K, L, n_sink=2, n_local=4)
    for h in range(4):
        g = h // 2
        single = oracle.decode_step(q[:, h:h + 1], Kc[:, g:g + 1], Vc[:, g:g + 1], W, K, L,
                                    n_sink=2, n_local=4)
        np.testing.assert_array_equal(single["counts"][0, 0], r["counts"][0, h])
        np.testing.assert_allclose(single["out"][0, 0], r["out"][0, h], rtol=1e-12)


def test_projector_size_matches_paper_table():
    g = golden()
    assert 128 * 10 * 150 * 2 == g["projector_bytes_K10_L150"]
    assert 128 * 11 * 300 * 2 // 1024 == g["projector_kib_K11_L300"]
