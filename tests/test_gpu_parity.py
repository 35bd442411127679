"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Hash codes, collision counts and candidate sets must match bit for bit;
attention outputs within 2e-3 max relative error per head."""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2410_16179_amd import binding as mp
from paper_2410_16179_amd import workloads as wl
from tests.gpu_helpers import Session, TOL, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    mp.lib()


def oracle_mu(oracle, Kc, n):
    B, Hkv = Kc.shape[:2]
    return np.stack([[oracle.key_mean(Kc[b, g, :n]) for g in range(Hkv)] for b in range(B)]).astype(np.float32)


def run_case(oracle, w: wl.Workload, seed=0, alpha=0.8, use_mu=True, n_cap=None, check_codes=True,
             oracle_codes_too=True, heads=None, centered_query=False, say="", indexed=(), layout="dense",
             check_key_mean=False, random_rows=0):
    print(f"[case] {say or w.name} B={w.batch} Hq={w.n_q_heads} Hkv={w.n_kv_heads} n={w.n_ctx} "
          f"K={w.K} L={w.L} tau={w.min_hits} dtype={w.dtype} seed={seed}", flush=True)
    data = wl.generate(w, seed, alpha)
    Kc, Vc, q, W = data["K"], data["V"], data["q"], data["W"]
    n = w.n_ctx
    mu = oracle_mu(oracle, Kc, n) if use_mu else None
    if centered_query:
        for b in range(w.batch):
            for h in range(w.n_q_heads):
                q[b, h] = wl.query(w, b, h, Kc[b, h // w.group], seed, alpha, center=mu[b, h // w.group])
    if n_cap is not None and n_cap > n:          # cache with spare capacity behind the context
        pad = wl.store(np.random.default_rng(5).standard_normal((w.batch, w.n_kv_heads, n_cap - n, 128)), w.kv or w.dtype)
        Kc = np.concatenate([Kc, pad], axis=2)
        Vc = np.concatenate([Vc, pad], axis=2)
    ref = oracle.decode_step(q, Kc[:, :, :n], Vc[:, :, :n], W, w.K, w.L,
                             mu=mu if use_mu else np.zeros((w.batch, w.n_kv_heads, 128), np.float32),
                             min_hits=w.min_hits, n_sink=w.n_sink, n_local=w.n_local, heads=heads)
    s = Session(K=w.K, L=w.L, dtype=w.dtype, Kc=Kc, Vc=Vc, q=q, W=W, n_ctx=n,
                min_hits=w.min_hits, n_sink=w.n_sink, n_local=w.n_local, layout=layout, kv=w.kv)
    s.set_mu(mu)
    if check_key_mean:
        assert np.abs(s.key_mean() - oracle_mu(oracle, Kc, n)).max() <= 1e-5 * np.abs(Kc).max()
    s.hash_keys(0, n)
    if w.dtype == "bf16" and n >= 1000:
        st = mp.hash_keys_stats(s.params, s.ws)
        elems = w.batch * w.n_kv_heads * n * w.K * w.L
        # the matrix-core path did the work: nothing overflowed, and only a small fraction
        # of the projections was close enough to zero to need the exact re-evaluation
        assert not st["overflowed"], st
        assert 0 < st["rechecked"] < 2e-3 * elems, (st, elems)
        print(f"   rechecked {st['rechecked']} of {elems} projections ({st['rechecked'] / elems:.2e})", flush=True)
    s.hash_query()
    pairs = heads if heads is not None else [(b, h) for b in range(w.batch) for h in range(w.n_q_heads)]
    if check_codes:
        np.testing.assert_array_equal(s.query_table_codes(), ref["q_codes"])
        for b, g in sorted({(b, h // w.group) for b, h in pairs}):
            np.testing.assert_array_equal(s.key_table_codes_unit(b, g)[:n], ref["key_codes"][b, g])
        if random_rows > 0:
            # everywhere else: random keys of every (batch, KV head) against the oracle's hashing
            rng = np.random.default_rng(seed + 77)
            checked = 0
            for b in range(w.batch):
                for g in range(w.n_kv_heads):
                    rows = np.sort(rng.choice(n, size=min(random_rows, n), replace=False))
                    want = oracle.hash_keys(Kc[b, g][rows], W, mu[b, g] if use_mu else None, w.K, w.L)
                    np.testing.assert_array_equal(s.key_table_codes_unit(b, g, rows), want)
                    checked += rows.size
            print(f"   key codes: every key of {len({(b, h // w.group) for b, h in pairs})} (batch, KV head) units, and "
                  f"{checked} random keys ({checked / (w.batch * w.n_kv_heads * n):.2%}) over all "
                  f"{w.batch * w.n_kv_heads} units", flush=True)
    if check_codes and n > 0:
        # the same hashing from the prepared projector (matrix cores for bf16): queries, and the
        # newest keys coded into buffers of their own by both forms, which must then be equal
        s.prepare()
        qc = torch.full_like(s.q_codes, -1)
        s.hash_query_prepared(qc)
        nq = w.batch * w.n_q_heads * s.NQ
        assert torch.equal(qc[:nq], s.q_codes[:nq])
        cnt = min(n, max(1, 128 // (w.batch * w.n_kv_heads)))
        if w.batch * w.n_kv_heads <= 128:
            a, b_ = torch.full_like(s.key_codes, 0x5a5a5a5a), torch.full_like(s.key_codes, 0x5a5a5a5a)
            mp.magicpig_hash_keys(s.params, s.Kc, s.mu, s.W, n - cnt, cnt, a, s.ws)
            qc.fill_(-1)
            s.hash_keys_prepared(n - cnt, cnt, key_codes=b_, q_codes=qc)
            assert torch.equal(a, b_), "keys coded from the prepared projector differ"
            assert torch.equal(qc[:nq], s.q_codes[:nq])
            # ... and those are the codes the prefill wrote for these keys
            full = s.key_codes.clone()
            s.hash_keys_prepared(n - cnt, cnt)
            assert torch.equal(full, s.key_codes)
    res = s.attend()
    worst = 0.0
    for b, h in pairs:
        np.testing.assert_array_equal(res["counts"][b, h], ref["counts"][b, h])
        assert res["ncand"][b, h] == ref["S"][b][h].size
        np.testing.assert_array_equal(res["S"][b][h], ref["S"][b][h])
        worst = max(worst, rel_err(res["out"][b, h][None], ref["out"][b, h][None]))
    print(f"   worst output error against the oracle {worst:.2e} (tolerance {TOL:.0e})", flush=True)
    assert worst <= TOL, worst
    # production call (no debug outputs) gives the same result
    res2 = s.attend(debug=False)
    for b, h in pairs:
        np.testing.assert_array_equal(res2["out"][b, h], res["out"][b, h])
    # the same step through the bucketed hash tables: same counts, same sample, same output
    if mp.magicpig_table_bytes(s.params) > 0 and n > 0:
        s.build_tables()
        rt = s.attend(tables=True)
        for b, h in pairs:
            np.testing.assert_array_equal(rt["counts"][b, h], ref["counts"][b, h])
            np.testing.assert_array_equal(rt["S"][b][h], ref["S"][b][h])
            assert rel_err(rt["out"][b, h][None], ref["out"][b, h][None]) <= TOL
            # same sample, same arithmetic; only the grouping of the partial sums differs
            assert rel_err(rt["out"][b, h][None], res["out"][b, h][None]) <= 1e-5
        rt2 = s.attend(debug=False, tables=True)
        rt3 = s.attend(tables=True, with_counts=False)      # candidate lists from the production lookup
        for b, h in pairs:
            # (the production form looks up and gathers in one launch: other partial sums)
            assert rel_err(rt2["out"][b, h][None], rt["out"][b, h][None]) <= 1e-5
            assert rel_err(rt2["out"][b, h][None], ref["out"][b, h][None]) <= TOL
            np.testing.assert_array_equal(rt3["S"][b][h], ref["S"][b][h])
            np.testing.assert_array_equal(rt3["out"][b, h], rt2["out"][b, h])
        # tables over a prefix of the keys, the rest found by the scan of their codes
        for ni in indexed:
            s.build_tables(ni)
            rh = s.attend(tables=True)
            rh2 = s.attend(debug=False, tables=True)        # production form of the lookup
            for b, h in pairs:
                np.testing.assert_array_equal(rh["counts"][b, h], ref["counts"][b, h])
                np.testing.assert_array_equal(rh["S"][b][h], ref["S"][b][h])
                assert rel_err(rh["out"][b, h][None], res["out"][b, h][None]) <= 1e-5
                assert rel_err(rh2["out"][b, h][None], rh["out"][b, h][None]) <= 1e-5
                assert rel_err(rh2["out"][b, h][None], ref["out"][b, h][None]) <= TOL
    if oracle_codes_too and heads is None:       # scan fed with the oracle's own codes
        s.upload_codes(np.concatenate([ref["key_codes"], np.zeros((w.batch, w.n_kv_heads, Kc.shape[2] - n, w.L), np.int32)], axis=2),
                       ref["q_codes"])
        res3 = s.attend()
        np.testing.assert_array_equal(res3["counts"], ref["counts"])
    return ref, res, worst


def test_c1_full(oracle):
    ref, res, worst = run_case(oracle, wl.CONFIGS["C1"])
    frac = ref["S"][0][0].size / 4096
    assert 0.01 < frac < 0.15        # (8,75) samples a few per cent of the keys


@pytest.mark.parametrize("seed", [1, 2])
def test_c1_other_seeds(oracle, seed):
    run_case(oracle, wl.CONFIGS["C1"], seed=seed)


def test_c2_shape_ragged_context(oracle):
    # Llama-3.1-8B shapes, (10,150), context not a multiple of the 64-key block or the chunk
    run_case(oracle, wl.scaled(wl.CONFIGS["C2"], n_ctx=5003))


def test_c4_shape_peaked_and_flat_heads(oracle):
    run_case(oracle, wl.scaled(wl.CONFIGS["C4"], batch=2, n_ctx=3000))


def test_c5_shape_group_of_eight(oracle):
    run_case(oracle, wl.scaled(wl.CONFIGS["C5"], batch=2, n_ctx=2500))


def test_full_batches_many_query_vectors(oracle):
    # 512 query vectors per step: the few-vectors kernel walks several pairs per workgroup
    run_case(oracle, wl.scaled(wl.CONFIGS["C4"], n_ctx=200), oracle_codes_too=False)
    run_case(oracle, wl.scaled(wl.CONFIGS["C5"], n_ctx=150), oracle_codes_too=False)
    # 544 heads: beyond the number up to which the hash-table step looks up and gathers in one
    # launch, so its production form runs the lookup and the gather as separate launches
    run_case(oracle, wl.scaled(wl.CONFIGS["C4"], batch=17, n_ctx=300), oracle_codes_too=False,
             heads=[(0, 0), (9, 17), (16, 31)], indexed=(128,))


@pytest.mark.parametrize("K,L,Hq,Hkv,dtype", [(7, 65, 4, 2, "bf16"), (3, 33, 2, 2, "fp32"),
                                              (16, 40, 8, 1, "bf16"), (1, 1, 1, 1, "fp32"),
                                              (5, 512, 2, 1, "bf16"),
                                              # the larger tables of the paper's hyper-parameter study
                                              (11, 300, 8, 2, "bf16"), (10, 220, 8, 2, "bf16")])
def test_generic_table_shapes(oracle, K, L, Hq, Hkv, dtype):
    w = wl.Workload("gen", 1, Hq, Hkv, 1500, K, L, dtype, (8,))
    run_case(oracle, w)


def test_token_major_cache_with_padded_value_rows(oracle):
    # K and V caches laid out [batch, token, KV head, row], V rows padded to 160 elements: every
    # kernel that reads the caches (key mean, the three key-hashing paths, the gather) goes
    # through the stride arguments, with different strides for K and V
    w = wl.scaled(wl.CONFIGS["C2"], batch=2, n_ctx=1777, n_q_heads=8, n_kv_heads=2)
    run_case(oracle, w, layout="token_major", check_key_mean=True, oracle_codes_too=False, indexed=(1024,))
    w1 = wl.scaled(wl.CONFIGS["C1"], n_ctx=700)                     # float32 caches
    run_case(oracle, w1, layout="token_major", check_key_mean=True, oracle_codes_too=False)
    # a handful of keys appended behind the prefill: the few-vectors kernel reads strided rows too
    data = wl.generate(w)
    mu = oracle_mu(oracle, data["K"], 1700)
    s = Session(K=w.K, L=w.L, dtype=w.dtype, Kc=data["K"], Vc=data["V"], q=data["q"], W=data["W"], layout="token_major")
    s.set_mu(mu)
    s.hash_keys(0, 1700)
    s.hash_keys(1700, 40)                                            # 2 x 2 x 40 vectors: matrix cores
    for i in range(1740, 1777):
        s.hash_keys(i, 1)                                            # 4 vectors: few-vectors kernel
    for b in range(2):
        for g in range(2):
            ref = oracle.hash_keys(data["K"][b, g], data["W"], mu[b, g], w.K, w.L)
            np.testing.assert_array_equal(s.key_table_codes()[b, g], ref)


def test_quantised_kv_cache(oracle):
    # K and V caches of OCP e4m3 bytes (q and W bf16): every kernel that reads the caches decodes
    # them; codes, counts, samples and outputs are those of the decoded values, which is what the
    # oracle is given.  Llama-8B and 70B shapes, a ragged context, the token-major layout with
    # padded V rows, a cache with spare capacity, keys appended behind tables, other thresholds.
    run_case(oracle, wl.scaled(wl.CONFIGS["C2"], n_ctx=5003, kv="fp8"), check_key_mean=True, indexed=(2048,))
    run_case(oracle, wl.scaled(wl.CONFIGS["C5"], batch=2, n_ctx=2500, kv="fp8"), oracle_codes_too=False)
    run_case(oracle, wl.scaled(wl.CONFIGS["C2"], batch=2, n_ctx=1777, n_q_heads=8, n_kv_heads=2, kv="fp8"),
             layout="token_major", check_key_mean=True, oracle_codes_too=False, indexed=(1024,))
    run_case(oracle, wl.scaled(wl.CONFIGS["C4"], batch=1, n_ctx=1000, n_q_heads=8, n_kv_heads=2, kv="fp8", min_hits=3),
             n_cap=1500, oracle_codes_too=False)
    # generic (K, L) and all-zero keys (every projection re-evaluated; the list overflows: float64 fallback)
    w = wl.Workload("gen8", 1, 4, 2, 700, 7, 65, "bf16", (8,), kv="fp8")
    run_case(oracle, w, oracle_codes_too=False)
    data = wl.generate(w)
    Kz = np.zeros_like(data["K"])
    s = Session(K=w.K, L=w.L, dtype="bf16", Kc=Kz, Vc=data["V"], q=data["q"], W=data["W"], kv="fp8")
    s.hash_keys()
    assert mp.hash_keys_stats(s.params, s.ws)["overflowed"]
    np.testing.assert_array_equal(s.key_table_codes()[0, 0], oracle.hash_keys(Kz[0, 0], data["W"], None, w.K, w.L))


@pytest.mark.parametrize("base,changes", [("C4", dict(n_ctx=11003, kv="fp8")), ("C4", dict(n_ctx=11003, dtype="fp32")),
                                          ("C5", dict(n_ctx=20011))])
def test_several_rounds_of_workgroups_other_element_types(oracle, base, changes):
    # Batches whose scan + gather grid does not fit the chip at once at a moderate context: runs of
    # 24 key blocks, the instantiation for four workgroups per compute unit, the early touches of
    # the rows of a wavefront's last block - here with e4m3 caches, with float32 inputs, and with
    # groups of eight query heads; a ragged context; heads of the first, a middle and the last
    # sequence against the oracle, every head finite.
    w = wl.scaled(wl.CONFIGS[base], **changes)
    B, Hq = w.batch, w.n_q_heads
    heads = [(0, 0), (0, Hq - 1), (B // 2, Hq // 2 + 1), (B - 1, 2), (B - 1, Hq - 1)]
    ref, res, worst = run_case(oracle, w, heads=heads, oracle_codes_too=False)
    assert np.isfinite(res["out"]).all() and np.abs(res["out"]).max() < 6.0


@pytest.mark.parametrize("Hq,Hkv", [(24, 8), (6, 1), (5, 1), (7, 1)])
def test_group_sizes_that_are_not_powers_of_two(oracle, Hq, Hkv):
    w = wl.scaled(wl.CONFIGS["C2"], n_ctx=2100, n_q_heads=Hq, n_kv_heads=Hkv)
    run_case(oracle, w, oracle_codes_too=False, indexed=(1024,))


@pytest.mark.parametrize("tau", [0, 1, 3, 4, 5, 7])    # 5 and up: the term-by-term tail of the inclusion probability
def test_other_hit_thresholds(oracle, tau):
    w = wl.scaled(wl.CONFIGS["C2"], n_ctx=2000, n_q_heads=8, n_kv_heads=2, min_hits=tau)
    ref, res, _ = run_case(oracle, w)
    if tau == 0:        # every key sampled with u = 1: exact attention
        data = wl.generate(w, 0)
        for h in range(8):
            ex = oracle.exact_attention(data["q"][0, h], data["K"][0, h // 4], data["V"][0, h // 4])
            assert rel_err(res["out"][0, h][None], ex[None]) <= TOL


@pytest.mark.parametrize("n", [0, 1, 5, 64, 68, 69, 130, 257])
def test_short_contexts(oracle, n):
    w = wl.scaled(wl.CONFIGS["C2"], n_ctx=max(n, 1), n_q_heads=4, n_kv_heads=1)
    if n == 0:
        s = Session(K=w.K, L=w.L, dtype=w.dtype, Kc=np.zeros((1, 1, 64, 128), np.float32),
                    Vc=np.zeros((1, 1, 64, 128), np.float32), q=np.ones((1, 4, 128), np.float32),
                    W=wl.projector(w), n_ctx=0)
        s.hash_query()
        res = s.attend(debug=False)
        assert np.all(res["out"] == 0)
        return
    run_case(oracle, w)


def test_no_static_tokens_and_no_centering(oracle):
    w = wl.scaled(wl.CONFIGS["C2"], n_ctx=3000, n_q_heads=8, n_kv_heads=2, n_sink=0, n_local=0)
    run_case(oracle, w, use_mu=False)
    run_case(oracle, w, use_mu=True)


def test_spare_capacity_behind_the_context(oracle):
    w = wl.scaled(wl.CONFIGS["C2"], n_ctx=1000, n_q_heads=8, n_kv_heads=2)
    run_case(oracle, w, n_cap=1500, oracle_codes_too=False)


@pytest.mark.parametrize("alpha", [8.0, 24.0])
def test_queries_with_large_inclusion_probabilities(oracle, alpha):
    # queries aligned with (centered) planted keys: u_i spans (0, 1], exercising both
    # branches of the inclusion-probability evaluation
    w = wl.scaled(wl.CONFIGS["C2"], n_ctx=4000, n_q_heads=8, n_kv_heads=2, planted=(4,))
    ref, _, _ = run_case(oracle, w, alpha=alpha, centered_query=True)


def test_append_keys_with_frozen_mean(oracle):
    w = wl.scaled(wl.CONFIGS["C2"], n_ctx=700, n_q_heads=4, n_kv_heads=1)
    data = wl.generate(w)
    mu = oracle_mu(oracle, data["K"], 500)                    # frozen after 500 prefill keys
    s = Session(K=w.K, L=w.L, dtype=w.dtype, Kc=data["K"], Vc=data["V"], q=data["q"], W=data["W"])
    s.set_mu(mu)
    s.hash_keys(0, 500)
    s.hash_keys(500, 37)
    s.hash_keys(537, 163)
    ref = oracle.hash_keys(data["K"][0, 0], data["W"], mu[0, 0], w.K, w.L)
    np.testing.assert_array_equal(s.key_table_codes()[0, 0], ref)


def test_both_table_builds_give_the_same_buckets(oracle):
    # 40000 keys: three windows of the two-pass build, the last one partial; (9,120) has 32 tables per pass
    for cfg, n in (("C2", 40000), ("C4", 20011)):
        w = wl.scaled(wl.CONFIGS[cfg], batch=1, n_ctx=n, n_q_heads=8, n_kv_heads=2)
        data = wl.generate(w)
        s = Session(K=w.K, L=w.L, dtype=w.dtype, Kc=data["K"], Vc=data["V"], q=data["q"], W=data["W"])
        s.set_mu(oracle_mu(oracle, data["K"], n))
        s.hash_keys()
        codes = s.key_table_codes()                              # [B, Hkv, n, L]
        by_scan = s.attend(debug=False)["out"]
        s.build_tables(big_workspace=False)
        off1, idx1 = s.table_buckets()
        assert s.table_windows()[0] == 0                         # one-pass build: buckets in no order
        by_unordered_tables = s.attend(debug=False, tables=True)["out"]
        s.build_tables(big_workspace=True)
        off2, idx2 = s.table_buckets()
        by_window_ordered_tables = s.attend(debug=False, tables=True)["out"]
        # the decode step gives the same result whichever way the sample is retrieved
        for o in (by_unordered_tables, by_window_ordered_tables):
            assert rel_err(o.reshape(-1, 128), by_scan.reshape(-1, 128)) <= 1e-5
        windows, fill = s.table_windows()
        assert windows == (n + 16383) // 16384
        np.testing.assert_array_equal(off1, off2)
        nb = 1 << w.K
        for unit in range(2):
            # offsets are the exclusive prefix sums of the code histogram of every table
            for t in (0, 31, 32, w.L - 1):
                hist = np.bincount(codes[0, unit, :, t], minlength=nb)
                np.testing.assert_array_equal(np.diff(off1[unit, t]), hist)
            for t in (0, 33, w.L - 1):
                for c in (0, 1, 77, nb - 1):
                    lo, hi = off1[unit, t, c], off1[unit, t, c + 1]
                    ref = np.flatnonzero(codes[0, unit, :, t] == c)
                    np.testing.assert_array_equal(np.sort(idx1[unit, t, lo:hi]), ref)
                    np.testing.assert_array_equal(np.sort(idx2[unit, t, lo:hi]), ref)
                    # window-ordered build: the piece of window v holds exactly the bucket's keys of
                    # [16384 v, 16384 (v + 1)), and the fill levels say where it starts
                    for v in range(windows):
                        a = lo + fill[unit, t, v, c]
                        b = lo + fill[unit, t, v + 1, c] if v + 1 < windows else hi
                        np.testing.assert_array_equal(np.sort(idx2[unit, t, a:b]),
                                                      ref[(ref >= 16384 * v) & (ref < 16384 * (v + 1))])


def test_tables_over_a_prefix_and_scan_of_the_appended_keys(oracle):
    # 0: nothing indexed; 64: one block; 1984: most; 2944: what is left lies inside the local window
    w = wl.scaled(wl.CONFIGS["C2"], n_ctx=3000, n_q_heads=8, n_kv_heads=2)
    run_case(oracle, w, oracle_codes_too=False, indexed=(0, 64, 1984, 2944))
    w4 = wl.scaled(wl.CONFIGS["C4"], batch=2, n_ctx=1500)
    run_case(oracle, w4, oracle_codes_too=False, indexed=(1024,))
    # three build windows (the last one partial) and 25 appended code blocks, two runs of them, in
    # the one-launch lookup; 16384 indexed: one window, too many appended keys for that form
    w3 = wl.scaled(wl.CONFIGS["C2"], n_ctx=40000, n_q_heads=8, n_kv_heads=2)
    run_case(oracle, w3, oracle_codes_too=False, heads=[(0, 1), (0, 6)], indexed=(38400, 16384))


def test_decode_steps_append_keys_behind_the_tables(oracle):
    # prefill 1920 keys (mean frozen there, tables built there), then 80 decode steps each
    # hashing one new key per KV head; the last step is checked against the oracle
    w = wl.scaled(wl.CONFIGS["C2"], n_ctx=2000, n_q_heads=8, n_kv_heads=2)
    data = wl.generate(w)
    n0 = 1920
    mu = oracle_mu(oracle, data["K"], n0)
    s = Session(K=w.K, L=w.L, dtype=w.dtype, Kc=data["K"], Vc=data["V"], q=data["q"], W=data["W"])
    s.set_mu(mu)
    s.hash_keys(0, n0)
    s.build_tables(n0)
    for i in range(n0, w.n_ctx):
        if i % 2:
            s.hash_keys(i, 1)
        else:                                            # key and queries coded by one launch
            mp.magicpig_hash_decode_step(s.params, s.q, s.Kc, s.mu, s.W, i, 1, s.key_codes, s.q_codes, s.ws)
    qref = np.stack([oracle.hash_query(data["q"][b], data["W"], w.K, w.L) for b in range(w.batch)])
    np.testing.assert_array_equal(s.query_table_codes(), qref)
    s.q_codes.zero_()
    s.hash_query()
    ref = oracle.decode_step(data["q"], data["K"], data["V"], data["W"], w.K, w.L, mu=mu,
                             min_hits=w.min_hits, n_sink=w.n_sink, n_local=w.n_local)
    for b in range(w.batch):
        for g in range(w.n_kv_heads):
            np.testing.assert_array_equal(s.key_table_codes()[b, g], ref["key_codes"][b, g])
    for res in (s.attend(tables=True), s.attend()):
        for h in range(w.n_q_heads):
            np.testing.assert_array_equal(res["counts"][0, h], ref["counts"][0, h])
            np.testing.assert_array_equal(res["S"][0][h], ref["S"][0][h])
            assert rel_err(res["out"][0, h][None], ref["out"][0, h][None]) <= TOL


@pytest.mark.parametrize("nrows", [64, 320])     # few-vectors kernel / matrix-core and float64 kernels
def test_hash_bits_follow_the_exact_sum(oracle, nrows):
    # projections that cancel to (almost) nothing: the bit is the sign of the exact sum
    K, L = 2, 3
    big, tiny = 2.0 ** 40, 2.0 ** -40
    W = np.zeros((128, K * L), np.float32)
    W[:4, :] = 1.0
    W[4, 1] = 1.0
    rows = np.zeros((1, 1, nrows, 128), np.float32)
    rows[0, 0, 0, :3] = [-tiny, big, -big]
    rows[0, 0, 1, :3] = [tiny, big, -big]
    rows[0, 0, 2, :3] = [big, -big, 0]
    rows[0, 0, 3, :5] = [big, -big, 0, 0, -tiny]
    rows[0, 0, 4, :3] = [1.5, -1.5, 0]
    for dtype in ("fp32", "bf16"):
        for mu in (None, np.zeros((1, 1, 128), np.float32), None):
            s = Session(K=K, L=L, dtype=dtype, Kc=rows, Vc=rows, q=rows[:, :, 0], W=W, n_ctx=nrows)
            s.set_mu(mu)
            s.hash_keys()
            ref = oracle.hash_keys(rows[0, 0], W, None if mu is None else mu[0, 0], K, L)
            np.testing.assert_array_equal(s.key_table_codes()[0, 0], ref)
            # the prepared form on the same rows, taken as keys (64 at a time) and as queries
            s.prepare()
            s.key_codes.fill_(0x5a5a5a5a)
            for first in range(0, nrows, 64):
                s.hash_keys_prepared(first, 64)
            np.testing.assert_array_equal(s.key_table_codes()[0, 0], ref)
            sq = Session(K=K, L=L, dtype=dtype, Kc=rows, Vc=rows, q=rows[:, 0, :5][:, :, :], W=W, n_ctx=nrows)
            sq.prepare()
            sq.hash_query_prepared()
            np.testing.assert_array_equal(sq.query_table_codes()[0], oracle.hash_query(rows[0, 0, :5], W, K, L))
    # centering that matters only in exact arithmetic
    mu = np.zeros((1, 1, 128), np.float32)
    mu[0, 0, 0] = big
    mu[0, 0, 1] = tiny
    rows2 = np.zeros((1, 1, nrows, 128), np.float32)
    rows2[0, 0, :, 0] = big
    ref = oracle.hash_keys(rows2[0, 0], W, mu[0, 0], K, L)
    assert ref[0, 0] == 0          # x - mu = -2^-40 < 0 in both planes of table 0
    for dtype in ("fp32", "bf16"):
        s = Session(K=K, L=L, dtype=dtype, Kc=rows2, Vc=rows2, q=rows2[:, :, 0], W=W, n_ctx=nrows)
        s.set_mu(mu)
        s.hash_keys()
        np.testing.assert_array_equal(s.key_table_codes()[0, 0], ref)
        s.prepare()
        s.key_codes.fill_(0x5a5a5a5a)
        for first in range(0, nrows, 64):
            s.hash_keys_prepared(first, 64)
        np.testing.assert_array_equal(s.key_table_codes()[0, 0], ref)


@pytest.mark.parametrize("K,L", [(10, 150), (9, 120), (7, 65), (16, 40), (1, 1), (5, 512), (11, 300), (6, 64)])
def test_hashing_from_the_prepared_projector(oracle, K, L):
    # the few-vectors matrix-core kernel: 70 query vectors (a full group of 64 and a ragged one),
    # keys appended in batches that end inside and across 32-key groups, with and without centering;
    # an all-zero vector (every projection exactly zero: each one is re-evaluated exactly) and vectors
    # that are multiples of projector columns (the magnitude bound is tight there)
    w = wl.Workload("prep", 2, 35, 5, 300, K, L, "bf16", (8,))
    data = wl.generate(w)
    Kc, q, W = data["K"].copy(), data["q"].copy(), data["W"]
    q[0, 3] = 0.0
    q[1, 7] = wl.store(3.0 * W[:, (K * L) // 2], "bf16")
    q[1, 8] = wl.store(-0.5 * W[:, 0], "bf16")
    Kc[0, 1, 290] = 0.0
    Kc[1, 4, 299] = wl.store(2.0 * W[:, K * L - 1], "bf16")
    mu = oracle_mu(oracle, Kc, 250)
    mu[1, 4] = Kc[1, 4, 299]                                       # a key equal to its centering vector: projections exactly 0
    for use_mu in (True, False):
        s = Session(K=K, L=L, dtype="bf16", Kc=Kc, Vc=data["V"], q=q, W=W)
        s.set_mu(mu if use_mu else None)
        s.prepare()
        s.key_codes.fill_(0x5a5a5a5a)
        s.q_codes.fill_(0x5a5a5a5a)
        first = 0
        for cnt in (12, 1, 7, 3, 12, 12, 5, 12, 12, 12, 12, 12):      # 10 units x 12 keys = 120 vectors at most
            s.hash_keys_prepared(first, cnt, q_codes=s.q_codes if first == 0 else None)
            first += cnt
        while first < 300:
            cnt = min(12, 300 - first)
            s.hash_keys_prepared(first, cnt)
            first += cnt
        for b in range(2):
            np.testing.assert_array_equal(s.query_table_codes()[b], oracle.hash_query(q[b], W, K, L))
            for g in range(5):
                ref = oracle.hash_keys(Kc[b, g], W, mu[b, g] if use_mu else None, K, L)
                np.testing.assert_array_equal(s.key_table_codes_unit(b, g), ref)
    # float32: the prepared form is a copy of the projector behind the same calls
    w32 = wl.Workload("prep32", 1, 6, 2, 200, min(K, 8), min(L, 75), "fp32", (8,))
    d32 = wl.generate(w32)
    mu32 = oracle_mu(oracle, d32["K"], 200)
    s = Session(K=w32.K, L=w32.L, dtype="fp32", Kc=d32["K"], Vc=d32["V"], q=d32["q"], W=d32["W"])
    s.set_mu(mu32)
    s.prepare()
    for first in range(0, 200, 50):
        s.hash_keys_prepared(first, 50, q_codes=s.q_codes)
    np.testing.assert_array_equal(s.query_table_codes()[0], oracle.hash_query(d32["q"][0], d32["W"], w32.K, w32.L))
    for g in range(2):
        np.testing.assert_array_equal(s.key_table_codes_unit(0, g),
                                      oracle.hash_keys(d32["K"][0, g], d32["W"], mu32[0, g], w32.K, w32.L))


def test_matrix_core_key_hashing_on_adversarial_rows(oracle):
    # rows chosen against the error bound of the matrix-core path: multiples of projector columns
    # (Cauchy-Schwarz is tight: |k.W_j| = |k||W_j|), sums and differences of two columns, rows with
    # huge cancelling terms next to small ones, and keys equal to the centering vector up to one
    # element; with a large common mean, so that most of every projection cancels against mu.W_j
    K, L, n = 10, 150, 1024
    w = wl.Workload("adv", 1, 4, 1, n, K, L, "bf16", (8,))
    W = wl.projector(w, 3)
    rng = np.random.default_rng(17)
    rows = np.zeros((n, 128), np.float64)
    cols = rng.integers(0, K * L, size=(n, 2))
    c = np.exp2(rng.integers(-6, 7, size=n)).astype(np.float64)
    kind = np.arange(n) % 4
    rows[kind == 0] = (c[:, None] * W[:, cols[:, 0]].T)[kind == 0]
    rows[kind == 1] = (W[:, cols[:, 0]].T - W[:, cols[:, 1]].T)[kind == 1]
    big = np.zeros((n, 128)); big[:, 0] = 2.0 ** 30; big[:, 1] = -2.0 ** 30; big[:, 2:] = rng.standard_normal((n, 126)) * 2.0 ** -8
    rows[kind == 2] = big[kind == 2]
    mean = 6.0 * rng.standard_normal(128)
    rows[kind == 3] = mean + 2.0 ** -7 * rng.standard_normal((n, 128))[kind == 3]
    Kc = wl.store(rows, "bf16")[None, None]
    mu = wl.store(mean, "bf16").astype(np.float32)[None, None]
    Kc[0, 0, 3::64] = mu[0, 0]                                       # exactly the centering vector: every projection is 0
    for use_mu in (True, False):
        s = Session(K=K, L=L, dtype="bf16", Kc=Kc, Vc=Kc, q=Kc[:, :, :4].reshape(1, 4, 128), W=W)
        s.set_mu(mu if use_mu else None)
        s.hash_keys()
        st = mp.hash_keys_stats(s.params, s.ws)
        print(f"   adversarial rows, centering {use_mu}: {st}", flush=True)
        ref = oracle.hash_keys(Kc[0, 0], W, mu[0, 0] if use_mu else None, K, L)
        np.testing.assert_array_equal(s.key_table_codes()[0, 0], ref)
        s.hash_query()
        np.testing.assert_array_equal(s.query_table_codes()[0], oracle.hash_query(Kc[0, 0, :4], W, K, L))


def test_overflow_of_the_recheck_list_falls_back_to_the_float64_kernel(oracle):
    # all-zero keys: every matrix-core result is exactly zero, every projection is flagged,
    # the list overflows and the direct kernel must produce the codes (all ones: 0 >= 0)
    w = wl.scaled(wl.CONFIGS["C2"], n_ctx=512, n_q_heads=4, n_kv_heads=1)
    data = wl.generate(w)
    Kz = np.zeros_like(data["K"])
    s = Session(K=w.K, L=w.L, dtype="bf16", Kc=Kz, Vc=data["V"], q=data["q"], W=data["W"])
    s.hash_keys()
    assert mp.hash_keys_stats(s.params, s.ws)["overflowed"]
    ref = oracle.hash_keys(Kz[0, 0], data["W"], None, w.K, w.L)
    np.testing.assert_array_equal(s.key_table_codes()[0, 0], ref)
    assert np.all(ref == (1 << w.K) - 1)


def test_fallback_walks_every_key_when_its_grid_is_capped(oracle):
    # 512 all-zero keys overflow the list; the other keys are ordinary.  With more than 16384
    # rows the float64 kernel behind the matrix-core path runs on a capped grid and loops.
    w = wl.scaled(wl.CONFIGS["C2"], n_ctx=20000, n_q_heads=4, n_kv_heads=1)
    data = wl.generate(w)
    Kc = data["K"].copy()
    Kc[:, :, 3000:3512] = 0
    s = Session(K=w.K, L=w.L, dtype="bf16", Kc=Kc, Vc=data["V"], q=data["q"], W=data["W"])
    s.hash_keys()                                   # no centering: the zero keys project to exactly 0
    assert mp.hash_keys_stats(s.params, s.ws)["overflowed"]
    ref = oracle.hash_keys(Kc[0, 0], data["W"], None, w.K, w.L)
    np.testing.assert_array_equal(s.key_table_codes()[0, 0], ref)


def test_key_mean(oracle):
    w = wl.scaled(wl.CONFIGS["C2"], n_ctx=5003, n_q_heads=8, n_kv_heads=2, batch=2)
    data = wl.generate(w)
    s = Session(K=w.K, L=w.L, dtype=w.dtype, Kc=data["K"], Vc=data["V"], q=data["q"], W=data["W"])
    got = s.key_mean()
    ref = np.stack([[oracle.key_mean(data["K"][b, g]) for g in range(2)] for b in range(2)])
    # float32 partial sums over at most 64 rows, float64 beyond: error far below 1e-5 of |k|
    assert np.abs(got - ref).max() <= 1e-5 * np.abs(data["K"]).max()
    w1 = wl.CONFIGS["C1"]
    d1 = wl.generate(w1)
    s1 = Session(K=w1.K, L=w1.L, dtype="fp32", Kc=d1["K"], Vc=d1["V"], q=d1["q"], W=d1["W"])
    assert np.abs(s1.key_mean()[0, 0] - oracle.key_mean(d1["K"][0, 0])).max() <= 1e-5 * np.abs(d1["K"]).max()


def test_repeatable(oracle):
    w = wl.scaled(wl.CONFIGS["C2"], n_ctx=6000)
    data = wl.generate(w)
    s = Session(K=w.K, L=w.L, dtype=w.dtype, Kc=data["K"], Vc=data["V"], q=data["q"], W=data["W"])
    s.set_mu(oracle_mu(oracle, data["K"], w.n_ctx))
    s.hash_keys(); s.hash_query()
    a = s.attend(debug=False)["out"]
    codes = s.key_codes.clone()
    s.hash_keys()
    assert torch.equal(codes, s.key_codes)
    b = s.attend(debug=False)["out"]
    np.testing.assert_array_equal(a, b)
