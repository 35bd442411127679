"""CPU oracle for LSH-sampled decode attention (MagicPIG, arXiv 2410.16179).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the HIP path is
checked against; only tests, the smoke check and the benchmark's CPU-baseline leg may
import it.  It shares no code with the HIP path and never calls it.  All floating point
is fp64 (numpy); hash bits are defined by the sign of the *exact* real-arithmetic
projection of the stored input values, so they do not depend on summation order.

Parity pins (tests/test_oracle_pins.py): per-bit agreement probability 1 - theta/pi
against empirical hyperplane draws (Sec. 2.2); inclusion probability against the
printed closed form and against scipy's binomial survival function (Eq. "lsh sampling
probability"); expected budget for orthogonal vectors (App. E, Eq. "budget"); exact
softmax attention recovered when every key is sampled with u = 1 (Sec. 2.1 definition,
checked against torch's scaled_dot_product_attention); Monte-Carlo inclusion frequency
and unbiasedness of numerator/denominator over random projectors (Eq. "importance
sampling unnormalized"); brute-force collision counting; invariants; the two comparison
estimators of Sec. 2.1 and Sec. 3.2 (TopK attention, oracle sampling estimation) against
the values the paper prints for its zoo example (App. "TopK vs. Sampling"), the closed
forms of its two theorems on oracle sampling, and brute force.  No function here is
"parity unpinned".

Notation follows the paper: K sign bits per table, L tables, p_i per-hyperplane
agreement probability, u_i inclusion probability, S the sample, T the static
(sink + local) set.
"""
from __future__ import annotations

import math

import numpy as np

_TINY_U = 1e-300


# --------------------------------------------------------------------------------------
# Sec. 2.1: the quantity being estimated
# --------------------------------------------------------------------------------------
def exact_attention(q, K, V):
    """o = softmax(q K^T / sqrt(d)) V for one query (Sec. 2.1, first equation)."""
    q = np.asarray(q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    if K.shape[0] == 0:
        return np.zeros(V.shape[1], np.float64)
    z = K @ q / math.sqrt(q.shape[0])
    w = np.exp(z - z.max())
    return (w / w.sum()) @ V


def attention_weights(q, K):
    """w = softmax(q K^T / sqrt(d)): the attention (score) distribution of Sec. 2.1."""
    q = np.asarray(q, np.float64)
    K = np.asarray(K, np.float64)
    z = K @ q / math.sqrt(q.shape[0])
    e = np.exp(z - z.max())
    return e / e.sum()


# --------------------------------------------------------------------------------------
# Sec. 2.1 / 3.1: TopK attention (the upper bound of search-based sparse attention)
# --------------------------------------------------------------------------------------
def topk_attention(q, K, V, m):
    """The m keys with the largest attention scores, renormalised among themselves:
    sum_{i in top} w_i v_i / sum_{i in top} w_i  (Sec. 2.1: Pi selects r_1..r_m, D = 1/sum w_{r_i}).
    Ties are broken towards the lower index.  Returns (out, sorted indices of the selection)."""
    V = np.asarray(V, np.float64)
    n = V.shape[0]
    m = int(min(max(m, 0), n))
    if m == 0:
        return np.zeros(V.shape[1], np.float64), np.zeros(0, np.int64)
    w = attention_weights(q, K)
    order = np.lexsort((np.arange(n), -w))          # descending score, then ascending index
    top = np.sort(order[:m])
    return (w[top] / w[top].sum()) @ V[top], top


# --------------------------------------------------------------------------------------
# Sec. 3.2: oracle sampling estimation
# --------------------------------------------------------------------------------------
def oracle_sampling_estimate(q, K, V, uniforms):
    """Definition "Oracle Sampling Estimation": B = len(uniforms) indices are drawn independently
    from the attention distribution w and the output is estimated as (1/B) sum_j v_{i_j}.  The
    randomness is passed in: `uniforms` are B numbers in [0, 1), turned into indices by
    inverting the cumulative distribution of w.  Returns (estimate, drawn indices); the
    computation cost of the estimate is the number of unique indices (Sec. 3.2)."""
    V = np.asarray(V, np.float64)
    u = np.asarray(uniforms, np.float64).reshape(-1)
    if u.size == 0:
        return np.zeros(V.shape[1], np.float64), np.zeros(0, np.int64)
    w = attention_weights(q, K)
    cdf = np.cumsum(w)
    idx = np.minimum(np.searchsorted(cdf, u * cdf[-1], side="right"), w.size - 1)
    return V[idx].mean(axis=0), idx.astype(np.int64)


def oracle_sampling_trace_of_covariance(q, K, V, budget):
    """Theorem "Oracle sampling estimation is unbiased ...", proof: Tr Cov = (E|v|^2 - |o|^2) / B."""
    V = np.asarray(V, np.float64)
    w = attention_weights(q, K)
    o = w @ V
    return float((w @ (V * V).sum(axis=1) - o @ o) / budget)


def relative_error(estimate, exact):
    """|estimate - exact| / |exact| (Euclidean norms): the estimation error of the paper's figures."""
    estimate = np.asarray(estimate, np.float64)
    exact = np.asarray(exact, np.float64)
    return float(np.linalg.norm(estimate - exact) / max(np.linalg.norm(exact), 1e-300))


# --------------------------------------------------------------------------------------
# Sec. 4.3 "Data pre-processing": centering
# --------------------------------------------------------------------------------------
def key_mean(K):
    """mu = (1/n) sum_i k_i over all n keys of one (batch, KV head)."""
    K = np.asarray(K, np.float64)
    return K.mean(axis=0) if K.shape[0] else np.zeros(K.shape[1], np.float64)


# --------------------------------------------------------------------------------------
# Sec. 2.2 / 4.3 "Hash function selection": SimHash bits
# --------------------------------------------------------------------------------------
def _exact_sign_nonneg(terms) -> bool:
    """[sum(terms) >= 0] with the sum taken exactly (math.fsum is correctly rounded)."""
    return math.fsum(terms) >= 0.0


def simhash_bits(X, W, mu=None, chunk=8192):
    """bits[i, t, b] = [ sum_d (x_{i,d} - mu_d) W_{d, t*K+b} >= 0 ]  as bool [m, L*K].

    Returned flat over columns j = t*K + b; use `table_codes` to fold into per-table
    integers.  The sign is that of the exact sum over the stored values of x, mu, W
    (sign(0) counts as non-negative).  X, mu, W must hold float32-representable values so
    that every product is exact in fp64; the fp64 matrix product decides all entries
    except those within a rigorous rounding bound of zero, which are re-summed exactly.
    The centered vector is never formed in floating point: the projection is expanded
    as x.W_j - mu.W_j.
    """
    X = np.atleast_2d(np.asarray(X))
    W = np.asarray(W)
    for a in (X, W) + (() if mu is None else (np.asarray(mu),)):
        a64 = np.asarray(a, np.float64)
        if not np.array_equal(a64.astype(np.float32).astype(np.float64), a64):
            raise ValueError("inputs must be float32-representable")
    X64 = X.astype(np.float64)
    W64 = W.astype(np.float64)
    m, d = X64.shape
    ncol = W64.shape[1]
    wn = np.linalg.norm(W64, axis=0)
    if mu is None:
        mu64 = None
        pm = np.zeros(ncol)
        mun = 0.0
    else:
        mu64 = np.asarray(mu, np.float64).reshape(d)
        pm = mu64 @ W64
        mun = float(np.linalg.norm(mu64))
    out = np.empty((m, ncol), dtype=bool)
    # |fl(x.W_j) - x.W_j| <= d * 2^-53 * sum|terms| <= d * 2^-53 * |x||W_j| (same for mu);
    # 2^-40 leaves three orders of magnitude of margin for d <= 1024.
    eps = 2.0 ** -40
    for lo in range(0, m, chunk):
        xs = X64[lo:lo + chunk]
        D = xs @ W64 - pm
        bound = eps * (np.linalg.norm(xs, axis=1)[:, None] + mun) * wn[None, :]
        bits = D >= 0.0
        ri, rj = np.nonzero(np.abs(D) <= bound)
        for i, j in zip(ri.tolist(), rj.tolist()):
            terms = [float(a) * float(b) for a, b in zip(xs[i], W64[:, j])]
            if mu64 is not None:
                terms += [-(float(a) * float(b)) for a, b in zip(mu64, W64[:, j])]
            bits[i, j] = _exact_sign_nonneg(terms)
        out[lo:lo + chunk] = bits
    return out


def table_codes(bits, K, L):
    """Canonical per-table integers code[i, t] = sum_b bits[i, t*K+b] * 2^b, int32 [m, L]."""
    bits = np.asarray(bits, dtype=bool).reshape(-1, L, K)
    weights = (1 << np.arange(K, dtype=np.int64))
    return (bits.astype(np.int64) * weights).sum(axis=2).astype(np.int32)


def hash_keys(Kmat, W, mu, K, L):
    """Codes of cached keys (centered by mu; mu=None means no centering)."""
    return table_codes(simhash_bits(Kmat, W, mu), K, L)


def hash_query(q, W, K, L):
    """Codes of queries; the query is not centered (only keys are)."""
    return table_codes(simhash_bits(q, W, None), K, L)


# --------------------------------------------------------------------------------------
# Sec. 4.3: collisions and the sample
# --------------------------------------------------------------------------------------
def collision_counts(q_code, key_codes):
    """count[i] = number of tables t with key_codes[i, t] == q_code[t]."""
    q_code = np.asarray(q_code).reshape(1, -1)
    key_codes = np.asarray(key_codes)
    return (key_codes == q_code).sum(axis=1).astype(np.int32)


def static_set(n, n_sink, n_local):
    """T = [0, n_sink) U [n - n_local, n); all of [0, n) when n <= n_sink + n_local."""
    if n <= n_sink + n_local:
        return np.arange(n, dtype=np.int64)
    return np.concatenate([np.arange(n_sink), np.arange(n - n_local, n)]).astype(np.int64)


def sample_set(counts, n_sink, n_local, min_hits):
    """S = { i in [n_sink, n - n_local) : count[i] >= min_hits }, sorted."""
    n = counts.shape[0]
    if n <= n_sink + n_local:
        return np.zeros(0, np.int64)
    idx = np.arange(n_sink, n - n_local, dtype=np.int64)
    return idx[counts[n_sink:n - n_local] >= min_hits]


# --------------------------------------------------------------------------------------
# Eq. "lsh sampling probability"
# --------------------------------------------------------------------------------------
def agreement_probability(cos_theta):
    """p = 1 - arccos(cos theta) / pi  (probability that one hyperplane gives equal signs)."""
    c = np.clip(np.asarray(cos_theta, np.float64), -1.0, 1.0)
    return 1.0 - np.arccos(c) / math.pi


def inclusion_probability(p, K, L, min_hits=2):
    """u = P[ Binomial(L, p^K) >= min_hits ]: a key is sampled iff it collides with the
    query in at least min_hits of the L tables, each colliding independently w.p. p^K.

    For min_hits = 2 this equals the printed 1 - (1-x)^L - L x (1-x)^(L-1), x = p^K; it is
    evaluated as the sum of the (positive) upper-tail terms, each in log space, because
    the printed form cancels catastrophically for small x.  min_hits <= 0 gives u = 1.
    """
    p = np.asarray(p, np.float64)
    if min_hits <= 0:
        return np.ones_like(p)
    x = p ** K
    u = np.zeros_like(x)
    interior = (x > 0.0) & (x < 1.0)
    xi = x[interior]
    if xi.size:
        lx, l1x = np.log(xi), np.log1p(-xi)
        acc = np.zeros_like(xi)
        for j in range(min_hits, L + 1):
            lc = math.lgamma(L + 1) - math.lgamma(j + 1) - math.lgamma(L - j + 1)
            acc += np.exp(lc + j * lx + (L - j) * l1x)
        u[interior] = acc
    u[x >= 1.0] = 1.0 if L >= min_hits else 0.0
    return np.minimum(u, 1.0)


def cosine_to_centered_keys(q, Kc):
    """cos between q and each centered key; 0 where either vector is the zero vector."""
    q = np.asarray(q, np.float64)
    Kc = np.asarray(Kc, np.float64)
    num = Kc @ q
    den = np.linalg.norm(q) * np.linalg.norm(Kc, axis=1)
    c = np.zeros_like(num)
    ok = den > 0
    c[ok] = num[ok] / den[ok]
    return np.clip(c, -1.0, 1.0)


# --------------------------------------------------------------------------------------
# Algorithm 1 / Eq. "close form": the estimator
# --------------------------------------------------------------------------------------
def estimator_from_sample(q, Kmat, V, mu, S, T, K, L, min_hits):
    """softmax([q k_S/sqrt(d) - log u_S, q k_T/sqrt(d)]) [V_S, V_T]  for one query head.

    Logits use the raw keys (softmax is invariant to the common shift q.mu/sqrt(d));
    u_i uses the centered keys, the vectors that were hashed.
    """
    q = np.asarray(q, np.float64)
    d = q.shape[0]
    S = np.asarray(S, np.int64)
    T = np.asarray(T, np.int64)
    if S.size + T.size == 0:
        return np.zeros(np.asarray(V).shape[1], np.float64)
    Ks = np.asarray(Kmat[S], np.float64)
    Kt = np.asarray(Kmat[T], np.float64)
    mu64 = np.zeros(d) if mu is None else np.asarray(mu, np.float64)
    zs = Ks @ q / math.sqrt(d)
    zt = Kt @ q / math.sqrt(d)
    if min_hits > 0 and S.size:
        c = cosine_to_centered_keys(q, Ks - mu64)
        u = np.maximum(inclusion_probability(agreement_probability(c), K, L, min_hits), _TINY_U)
        zs = zs - np.log(u)
    z = np.concatenate([zs, zt])
    w = np.exp(z - z.max())
    Vall = np.concatenate([np.asarray(V[S], np.float64), np.asarray(V[T], np.float64)])
    return (w / w.sum()) @ Vall


def sampled_attention_head(q, Kmat, V, mu, q_code, key_codes, K, L,
                           min_hits=2, n_sink=4, n_local=64):
    """One query head: counts -> S, T -> estimator.  Returns (out, counts, S)."""
    n = np.asarray(Kmat).shape[0]
    counts = collision_counts(q_code, key_codes) if n else np.zeros(0, np.int32)
    S = sample_set(counts, n_sink, n_local, min_hits)
    T = static_set(n, n_sink, n_local)
    out = estimator_from_sample(q, Kmat, V, mu, S, T, K, L, min_hits)
    return out, counts, S


def decode_step(q, Kc, Vc, W, K, L, mu=None, min_hits=2, n_sink=4, n_local=64,
                key_codes=None, heads=None):
    """Whole path for a batch with grouped-query attention.

    q [B, Hq, d]; Kc, Vc [B, Hkv, n, d]; W [d, K*L]; mu [B, Hkv, d] (None: computed by
    `key_mean` and rounded to float32, the form the boundary takes it in).  Each query
    head h samples independently against the codes of KV head h // (Hq/Hkv).
    Returns dict(out [B,Hq,d] fp64, counts [B,Hq,n], S list-of-lists, key_codes
    [B,Hkv,n,L], q_codes [B,Hq,L], mu [B,Hkv,d]).  `heads` restricts the (b, h) pairs
    evaluated (others are left zero / None); `key_codes` reuses precomputed codes.
    """
    q = np.asarray(q)
    B, Hq, d = q.shape
    Hkv, n = Kc.shape[1], Kc.shape[2]
    G = Hq // Hkv
    if mu is None:
        mu = np.stack([[key_mean(Kc[b, g]) for g in range(Hkv)] for b in range(B)])
        mu = mu.astype(np.float32)
    want = [(b, h) for b in range(B) for h in range(Hq)] if heads is None else list(heads)
    need_g = sorted({(b, h // G) for b, h in want})
    if key_codes is None:
        key_codes = np.zeros((B, Hkv, n, L), np.int32)
        for b, g in need_g:
            key_codes[b, g] = hash_keys(Kc[b, g], W, mu[b, g], K, L)
    q_codes = hash_query(q.reshape(B * Hq, d), W, K, L).reshape(B, Hq, L)
    out = np.zeros((B, Hq, d), np.float64)
    counts = np.zeros((B, Hq, n), np.int32)
    S = [[None] * Hq for _ in range(B)]
    for b, h in want:
        g = h // G
        out[b, h], counts[b, h], S[b][h] = sampled_attention_head(
            q[b, h], Kc[b, g], Vc[b, g], mu[b, g], q_codes[b, h], key_codes[b, g],
            K, L, min_hits, n_sink, n_local)
    return {"out": out, "counts": counts, "S": S, "key_codes": key_codes,
            "q_codes": q_codes, "mu": mu}


def expected_budget(K, L):
    """App. E, Eq. "budget": sampled fraction when every table collides w.p. 2^-K."""
    x = 0.5 ** K
    return 1.0 - (1.0 - x) ** L - L * x * (1.0 - x) ** (L - 1)
