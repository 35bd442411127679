"""The decode loop (Algorithm 1 used once per generated token; Sec. 4.4 (3), (4)): the context
grows by one key per step, the new key is coded behind the frozen mean and joins the hash
structure, the token that leaves the local window becomes eligible for sampling.  One HIP graph
is captured once and replayed for every token; the context length lives in device memory
(magicpig_params.n_ctx_dev) and is advanced inside the graph."""
import numpy as np
import pytest
import torch

from paper_2410_16179_amd import binding as mp
from paper_2410_16179_amd import workloads as wl
from tests.gpu_helpers import Session, TOL, rel_err, to_dev

pytestmark = pytest.mark.gpu


def _capture(fn):
    fn()                                     # eager once (also warms everything up)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            fn()
    torch.cuda.current_stream().wait_stream(side)
    return g


@pytest.mark.parametrize("cfg,Hq,Hkv,n0", [("C2", 8, 2, 1000), ("C4", 8, 2, 2019)])
def test_growing_context_one_graph_for_every_token(oracle, cfg, Hq, Hkv, n0):
    tokens = 150
    n_max = n0 + tokens
    w = wl.scaled(wl.CONFIGS[cfg], batch=2 if cfg == "C4" else 1, n_ctx=n_max, n_q_heads=Hq, n_kv_heads=Hkv)
    B = w.batch
    print(f"[case] decode loop {cfg} B={B} Hq={Hq} Hkv={Hkv} prefill {n0} + {tokens} tokens K={w.K} L={w.L}", flush=True)
    data = wl.generate(w)
    Kc, Vc, W = data["K"], data["V"], data["W"]
    # the mean is frozen at the prefill (reading r4); every later key is coded with it
    mu = np.stack([[oracle.key_mean(Kc[b, g, :n0]) for g in range(Hkv)] for b in range(B)]).astype(np.float32)
    all_codes = np.stack([[oracle.hash_keys(Kc[b, g], W, mu[b, g], w.K, w.L) for g in range(Hkv)] for b in range(B)])

    # device caches hold the prefill; the rows behind it are NaN until their token arrives
    nan_tail = lambda x: np.concatenate([x[:, :, :n0], np.full_like(x[:, :, n0:], 0.0)], axis=2)
    n_dev = torch.tensor([n0], dtype=torch.int64, device="cuda")
    s = Session(K=w.K, L=w.L, dtype=w.dtype, Kc=nan_tail(Kc), Vc=nan_tail(Vc), q=data["q"], W=W, n_ctx=n_max,
                n_ctx_dev=n_dev)
    s.Kc[:, :, n0:] = float("nan")
    s.Vc[:, :, n0:] = float("nan")
    K_all, V_all = to_dev(Kc, w.dtype), to_dev(Vc, w.dtype)
    s.set_mu(mu)
    prefill = mp.make_params(**{**s._pkw, "n_ctx_dev": None}, n_ctx=n0)
    mp.magicpig_hash_keys(prefill, s.Kc, s.mu, s.W, 0, n0, s.key_codes, s.ws)
    n_indexed = n0 // 64 * 64
    s.build_tables(n_indexed)

    counts = torch.full((B, Hq, n_max), -1, dtype=torch.int16, device="cuda")
    cand = torch.full((B, Hq, n_max), -1, dtype=torch.int32, device="cuda")
    ncand = torch.zeros((B, Hq), dtype=torch.int32, device="cuda")
    outs = {k: torch.full((B, Hq, 128), float("nan"), dtype=torch.float32, device="cuda")
            for k in ("scan_dbg", "scan", "tables_dbg", "tables", "noalloc")}
    cand_t = torch.full_like(cand, -1)
    ncand_t = torch.zeros_like(ncand)
    counts_t = torch.zeros_like(counts)
    state = {"n_indexed": n_indexed}

    def token_step():
        n_dev.add_(1)                        # the new token's key and value are in the cache: the context grew
        mp.magicpig_hash_decode_step(s.params, s.q, s.Kc, s.mu, s.W, 0, 1, s.key_codes, s.q_codes)
        ncand.zero_()
        ncand_t.zero_()
        mp.magicpig_sampled_attention(s.params, s.q, s.Kc, s.Vc, s.mu, s.key_codes, s.q_codes, outs["scan_dbg"],
                                      counts, cand, ncand, s.ws)
        mp.magicpig_sampled_attention(s.params, s.q, s.Kc, s.Vc, s.mu, s.key_codes, s.q_codes, outs["scan"],
                                      workspace=s.ws)
        mp.magicpig_sampled_attention_noalloc(s.params, s.q, s.Kc, s.Vc, s.mu, s.key_codes, s.q_codes, outs["noalloc"])
        mp.magicpig_sampled_attention_tables(s.params, s.q, s.Kc, s.Vc, s.mu, s.tables, state["n_indexed"],
                                             s.key_codes, s.q_codes, outs["tables_dbg"], counts_t, cand_t, ncand_t, s.ws)
        mp.magicpig_sampled_attention_tables(s.params, s.q, s.Kc, s.Vc, s.mu, s.tables, state["n_indexed"],
                                             s.key_codes, s.q_codes, outs["tables"], workspace=s.ws)

    # capture once.  The eager run and the capture run of _capture each advance the context by one
    # token: give them the rows of tokens n0 and n0 + 1 first, and start counting behind them.
    for i in (n0, n0 + 1):
        s.Kc[:, :, i] = K_all[:, :, i]
        s.Vc[:, :, i] = V_all[:, :, i]
    graph = _capture(token_step)             # eager step: context n0 + 1; capture itself runs nothing
    torch.cuda.synchronize()
    assert int(n_dev.item()) == n0 + 1
    checked, newly = 0, 0
    for t in range(2, tokens + 1):
        n_t = n0 + t
        if t == 80:
            # periodic rebuild of the tables over everything but the last partial block, then a
            # new graph (n_indexed is an argument of the call)
            state["n_indexed"] = (n_t - 1) // 64 * 64
            s.build_tables(state["n_indexed"])
            n_dev.fill_(n_t - 2)             # capture's eager run and nothing else moves it: back to n_t - 1 below
            graph = _capture(token_step)
            torch.cuda.synchronize()
            assert int(n_dev.item()) == n_t - 1
        # the token's K / V rows arrive, its query is new
        s.Kc[:, :, n_t - 1] = K_all[:, :, n_t - 1]
        s.Vc[:, :, n_t - 1] = V_all[:, :, n_t - 1]
        w_t = wl.scaled(w, n_ctx=n_t)
        q_t = np.stack([[wl.query(w_t, b, h, Kc[b, h // w.group, :n_t], seed=t) for h in range(Hq)] for b in range(B)])
        s.q.copy_(to_dev(q_t, w.dtype))
        graph.replay()
        if t % 16 and t != tokens and t not in (63, 64, 65, 80, 81):
            continue
        torch.cuda.synchronize()
        assert int(n_dev.item()) == n_t
        ref = oracle.decode_step(q_t, Kc[:, :, :n_t], Vc[:, :, :n_t], W, w.K, w.L, mu=mu, min_hits=w.min_hits,
                                 n_sink=w.n_sink, n_local=w.n_local, key_codes=all_codes[:, :, :n_t])
        np.testing.assert_array_equal(s.query_table_codes(), ref["q_codes"])
        for b in range(B):
            for g in range(Hkv):
                np.testing.assert_array_equal(s.key_table_codes_unit(b, g)[:n_t], all_codes[b, g, :n_t])
        cn, cnt_t = counts.cpu().numpy()[:, :, :n_t].astype(np.int32), counts_t.cpu().numpy()[:, :, :n_t].astype(np.int32)
        for name, cd, nc in (("scan", cand, ncand), ("tables", cand_t, ncand_t)):
            cdh, nch = cd.cpu().numpy(), nc.cpu().numpy()
            for b in range(B):
                for h in range(Hq):
                    np.testing.assert_array_equal(np.sort(cdh[b, h, :nch[b, h]]), ref["S"][b][h], err_msg=f"{name} t={t}")
        np.testing.assert_array_equal(cn, ref["counts"])
        np.testing.assert_array_equal(cnt_t, ref["counts"])
        o = {k: v.cpu().numpy() for k, v in outs.items()}
        assert rel_err(o["scan_dbg"], ref["out"]) <= TOL
        np.testing.assert_array_equal(o["scan"], o["scan_dbg"])
        np.testing.assert_array_equal(o["noalloc"], o["scan"])
        assert rel_err(o["tables_dbg"], ref["out"]) <= TOL and rel_err(o["tables"], ref["out"]) <= TOL
        # keys that were inside the local window at the prefill, or arrived later, are sampled now
        newly += sum(int((ref["S"][b][h] >= n0 - w.n_local).sum()) for b in range(B) for h in range(Hq))
        checked += 1
    assert checked >= 10 and newly > 0
    print(f"   {tokens - 1} graph replays, {checked} steps checked against the oracle (codes of every key, counts, "
          f"samples, outputs of all {B * Hq} heads); {newly} sampled keys had left the local window since the prefill",
          flush=True)
