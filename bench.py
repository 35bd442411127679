"""Benchmark of the LSH-sampled decode attention hot path on one MI355X.

One step = one decode step of one layer at the C3 workload (Llama-3.1-8B shapes, batch 1,
32 query / 8 KV heads, head_dim 128, context 98304, bf16, SimHash K=10 L=150, >= 2 hits,
4 sink + 64 local): magicpig_hash_query + magicpig_sampled_attention (query coding,
collision scan, compaction, gather, importance-weighted softmax.V).  Inputs, key codes and
the centering vector are resident in HBM before the timed region.  The one-time prefill
work (magicpig_key_mean + magicpig_hash_keys over all 786432 keys) is timed separately and
reported under "prefill_hash".  Steps rotate over several independent copies of (codes, K,
V) so that no step finds its data in the last-level cache, as in a real model where each
layer has its own cache.

Prints ONE JSON line.  `python bench.py --gpus 1 --steps K --warmup W`.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402
import torch  # noqa: E402

from paper_2410_16179_amd import binding as mp  # noqa: E402
from paper_2410_16179_amd import workloads as wl  # noqa: E402

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
METRIC = "LSH-sampled decode attn: query-heads/s at 96k ctx"


def build_workload(name: str, copies: int, seed: int):
    w = wl.CONFIGS[name]
    t0 = time.time()
    data = wl.generate(w, seed)
    gen_s = time.time() - t0
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    Kd = torch.from_numpy(data["K"]).to(tdt).cuda()
    Vd = torch.from_numpy(data["V"]).to(tdt).cuda()
    qd = torch.from_numpy(data["q"]).to(tdt).cuda()
    Wd = torch.from_numpy(data["W"]).to(tdt).cuda()
    params = mp.make_params(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, K=w.K,
                            L=w.L, n_ctx=w.n_ctx, dtype=w.dtype, min_hits=w.min_hits,
                            n_sink=w.n_sink, n_local=w.n_local)
    sets = []
    for c in range(copies):
        sets.append({
            "K": Kd if c == 0 else Kd.clone(), "V": Vd if c == 0 else Vd.clone(),
            "codes": mp.alloc_key_codes(params),
            "mu": torch.empty(w.batch, w.n_kv_heads, 128, dtype=torch.float32, device="cuda"),
        })
    return w, data, params, qd, Wd, sets, gen_s


def time_prefill(params, w, Wd, sets, ws):
    """key mean + key hashing of every copy; returns average ms per copy."""
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for s in sets:
        mp.magicpig_key_mean(params, s["K"], s["mu"], ws)
        mp.magicpig_hash_keys(params, s["K"], s["mu"], Wd, 0, w.n_ctx, s["codes"], ws)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / len(sets)


def cpu_baseline(w, data, seed):
    """The CPU oracle, as it stands, single-threaded, on the first batch element of the
    workload at its full context: the decode step (query coding, collision counts, sample,
    inclusion probabilities, estimator) of all its query heads.  The oracle first hashes the
    keys itself (timed and reported, not part of `value`, like the GPU's prefill hashing)."""
    from oracle import magicpig_oracle as oracle
    from threadpoolctl import threadpool_limits
    heads = [(0, h) for h in range(w.n_q_heads)]
    sub = {k: (v[:1] if k != "W" else v) for k, v in data.items()}
    with threadpool_limits(limits=1):
        mu = np.stack([[oracle.key_mean(sub["K"][0, g]) for g in range(w.n_kv_heads)]]).astype(np.float32)
        t0 = time.time()
        codes = np.zeros((1, w.n_kv_heads, w.n_ctx, w.L), np.int32)
        for g in range(w.n_kv_heads):
            codes[0, g] = oracle.hash_keys(sub["K"][0, g], sub["W"], mu[0, g], w.K, w.L)
        hash_s = time.time() - t0
        t0 = time.time()
        ref = oracle.decode_step(sub["q"], sub["K"], sub["V"], sub["W"], w.K, w.L, mu=mu,
                                 min_hits=w.min_hits, n_sink=w.n_sink, n_local=w.n_local,
                                 key_codes=codes, heads=heads)
        dec_s = time.time() - t0
    return {
        "value": len(heads) / dec_s, "unit": "query-heads/s", "cores": 1, "kind": "oracle",
        "sample": f"decode step of the {len(heads)} query heads of batch element 0 at the full "
                  f"{w.n_ctx}-key context: {dec_s:.2f} s; before it the oracle hashed those "
                  f"{w.n_kv_heads * w.n_ctx} keys in {hash_s:.1f} s "
                  f"({w.n_kv_heads * w.n_ctx / hash_s:.0f} keys/s, not in value)",
    }, ref, heads


def stored_traffic(workload: str):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary
    (FETCH_SIZE and WRITE_SIZE, calibrated on a copy of known size); None if absent."""
    path = os.path.join(ROOT, "profiles", f"scan_gather_{workload}_pmc.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch"):
                    return float(line.split()[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="C3")
    ap.add_argument("--copies", type=int, default=8)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-tables", action="store_true")
    ap.add_argument("--no-decode-loop", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path "
              "(the path shards by KV head without communication; see DESIGN.md)", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    mp.lib()

    w, data, params, qd, Wd, sets, gen_s = build_workload(args.workload, args.copies, args.seed)
    ws = mp.alloc_workspace(params)
    qcodes = mp.alloc_query_codes(params)
    out = torch.empty(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")

    prefill_ms = time_prefill(params, w, Wd, sets, ws)          # also produces codes and mu
    prefill_ms = time_prefill(params, w, Wd, sets, ws)          # second pass: warm

    def step(i):
        s = sets[i % len(sets)]
        mp.magicpig_hash_query(params, qd, Wd, qcodes, ws)
        mp.magicpig_sampled_attention(params, qd, s["K"], s["V"], s["mu"], s["codes"], qcodes, out,
                                      workspace=ws)

    # sample sizes for the algorithmic byte count (debug outputs, outside the timed region)
    ncand = torch.zeros(w.batch, w.n_q_heads, dtype=torch.int32, device="cuda")
    cand = torch.zeros(w.batch, w.n_q_heads, 1, dtype=torch.int32, device="cuda")
    mp.magicpig_hash_query(params, qd, Wd, qcodes, ws)
    mp.magicpig_sampled_attention(params, qd, sets[0]["K"], sets[0]["V"], sets[0]["mu"], sets[0]["codes"],
                                  qcodes, out, None, cand, ncand, ws)
    torch.cuda.synchronize()
    n_sampled = ncand.cpu().numpy().astype(np.int64)
    out0 = out.cpu().numpy().copy()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` decode steps, replayed from one HIP graph so that the
    # host's launch cost (python + ctypes, several microseconds per call) is not what is
    # measured.  If capture is unavailable the same steps are timed as eager launches.
    launch_mode = "hipgraph"
    graph = None
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                for i in range(args.steps):
                    step(i)
        torch.cuda.current_stream().wait_stream(side)
        graph.replay()                      # untimed: first replay uploads the graph
        torch.cuda.synchronize()
    except Exception as exc:  # noqa: BLE001
        print(f"graph capture failed ({exc}); timing eager launches", file=sys.stderr)
        graph, launch_mode = None, "eager"
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    if graph is not None:
        graph.replay()
    else:
        for i in range(args.steps):
            step(i)
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    gpu_ms_per_step = e0.elapsed_time(e1) / args.steps
    heads = w.batch * w.n_q_heads
    value = heads / (ms_per_step * 1e-3)

    # ---- per-kernel durations, live, with HIP events recorded between the kernels on the
    # stream they run on (same steps, eager launches)
    hip = ctypes.CDLL("libamdhip64.so")
    n_ev = min(args.steps, 100)
    evs = []
    for _ in range(n_ev):
        quad = []
        for _ in range(5):
            e = ctypes.c_void_p()
            assert hip.hipEventCreate(ctypes.byref(e)) == 0
            quad.append(e)
        evs.append(quad)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    for i in range(n_ev):
        s = sets[i % len(sets)]
        hip.hipEventRecord(evs[i][4], stream)
        mp.magicpig_hash_query(params, qd, Wd, qcodes, ws)
        mp.magicpig_profile_stage_events([e.value for e in evs[i][:4]])
        mp.magicpig_sampled_attention(params, qd, s["K"], s["V"], s["mu"], s["codes"], qcodes, out,
                                      workspace=ws)
    mp.magicpig_profile_stage_events(None)
    torch.cuda.synchronize()

    def span(a, b):
        ms = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
        return ms.value
    # (magicpig_sampled_attention scans and gathers in one kernel: events 0 / 1 are its begin /
    # end timestamps, event 3 the end of the merge kernel)
    stage_ms = {
        "hash_query": float(np.mean([span(q[4], q[0]) for q in evs])),
        "scan_gather": float(np.mean([span(q[0], q[1]) for q in evs])),
        "merge": float(np.mean([span(q[1], q[3]) for q in evs])),
    }
    for quad in evs:
        for e in quad:
            hip.hipEventDestroy(e)
    scan_ms = stage_ms["scan_gather"]

    # ---- the same decode step with the bucketed hash tables (the paper's Query(HT, q_code))
    # in place of the collision scan: same sample, same output, far fewer bytes
    tables_info = None
    if mp.magicpig_table_bytes(params) > 0 and not args.no_tables:
        for s_ in sets:
            s_["tables"] = mp.alloc_tables(params)
        b0, b1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        bws = mp.alloc_table_build_workspace(params)          # room for the two-pass build
        mp.magicpig_build_tables(params, sets[0]["codes"], sets[0]["tables"], bws)     # warm-up
        torch.cuda.synchronize()
        b0.record()
        for s_ in sets:
            mp.magicpig_build_tables(params, s_["codes"], s_["tables"], bws)
        b1.record()
        torch.cuda.synchronize()

        def tstep(i):
            s_ = sets[i % len(sets)]
            mp.magicpig_hash_query(params, qd, Wd, qcodes, ws)
            mp.magicpig_sampled_attention_tables(params, qd, s_["K"], s_["V"], s_["mu"], s_["tables"], w.n_ctx,
                                                 s_["codes"], qcodes, out, workspace=ws)
        for i in range(args.warmup):
            tstep(i)
        torch.cuda.synchronize()
        out_t = out.cpu().numpy().copy()
        side2 = torch.cuda.Stream()
        side2.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side2):
            g2 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g2, stream=side2):
                for i in range(args.steps):
                    tstep(i)
        torch.cuda.current_stream().wait_stream(side2)
        g2.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        g2.replay()
        torch.cuda.synchronize()
        t_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        tables_info = {"value": heads / (t_ms * 1e-3), "unit": "query-heads/s", "ms_per_step": t_ms,
                       "build_ms": b0.elapsed_time(b1) / len(sets),
                       "table_bytes": mp.magicpig_table_bytes(params),
                       "build_workspace_bytes": mp.magicpig_table_build_workspace_bytes(params),
                       "what": "magicpig_hash_query + magicpig_sampled_attention_tables, HIP graph; "
                               "build = magicpig_build_tables per cache copy (one-time)"}

    # ---- one generated token of a 32-layer model, the loop this path sits in: per layer the
    # token's key is coded behind the frozen mean (magicpig_hash_keys, one key per KV head), the
    # query is coded and the attention runs.  Layers cycle over the cache copies; the whole
    # token is one HIP graph.  In the table form the tables were built `appended` keys ago, so
    # those keys are found by the scan of their codes.
    loop_info = None
    if not args.no_decode_loop:
        layers, appended, reps = 32, 2048, 10
        n_idx = max(0, (w.n_ctx - appended) // 64 * 64)

        def token(form):
            for l in range(layers):
                s_ = sets[l % len(sets)]
                mp.magicpig_hash_decode_step(params, qd, s_["K"], s_["mu"], Wd, w.n_ctx - 1, 1, s_["codes"], qcodes,
                                             ws)
                if form == "tables":
                    mp.magicpig_sampled_attention_tables(params, qd, s_["K"], s_["V"], s_["mu"], s_["tables"],
                                                         n_idx, s_["codes"], qcodes, out, workspace=ws)
                else:
                    mp.magicpig_sampled_attention(params, qd, s_["K"], s_["V"], s_["mu"], s_["codes"], qcodes,
                                                  out, workspace=ws)

        def time_token(form):
            token(form)
            torch.cuda.synchronize()
            side3 = torch.cuda.Stream()
            side3.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side3):
                g3 = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g3, stream=side3):
                    token(form)
            torch.cuda.current_stream().wait_stream(side3)
            g3.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                g3.replay()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / reps

        loop_info = {"layers": layers, "tokens_timed": reps,
                     "scan_ms_per_token": time_token("scan"),
                     "what": "per layer: magicpig_hash_decode_step (the token's key, 1 per KV head, and the queries) "
                             "+ attention; 32 layers in one HIP graph"}
        if tables_info is not None:
            p_idx = mp.make_params(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, K=w.K, L=w.L,
                                   n_ctx=n_idx, n_cap=w.n_ctx, dtype=w.dtype, min_hits=w.min_hits,
                                   n_sink=w.n_sink, n_local=w.n_local)
            for s_ in sets:
                mp.magicpig_build_tables(p_idx, s_["codes"], s_["tables"], bws)
            loop_info["tables_ms_per_token"] = time_token("tables")
            loop_info["keys_appended_since_table_build"] = w.n_ctx - n_idx
            loop_info["max_abs_diff_tables_vs_scan_output"] = float(np.abs(out.cpu().numpy() - out0).max())

    n_static = min(w.n_ctx, w.n_sink + w.n_local)
    scan_bytes = w.batch * w.n_kv_heads * max(w.n_ctx - n_static, 0) * w.K * w.L / 8.0
    gather_bytes = float((n_sampled + n_static).sum()) * 2 * 128 * (2 if w.dtype == "bf16" else 4)
    out_bytes = heads * 128 * 4
    alg_bytes = scan_bytes + gather_bytes + out_bytes
    # the dominant kernel streams the codes of the eligible keys and gathers the K and V rows
    # of the attended ones: both are its algorithmic bytes
    kernel_bytes = scan_bytes + gather_bytes
    achieved = kernel_bytes / (scan_ms * 1e-3) / 1e9
    path_gbs = alg_bytes / (ms_per_step * 1e-3) / 1e9

    hash_flops = 2.0 * w.batch * w.n_kv_heads * w.n_ctx * 128 * w.K * w.L
    result = {
        "metric": METRIC, "value": value, "unit": "query-heads/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: batch {w.batch}, {w.n_q_heads} query / {w.n_kv_heads} KV heads, "
                               f"head_dim 128, context {w.n_ctx}, K={w.K} L={w.L}, min_hits {w.min_hits}, "
                               f"{w.n_sink} sink + {w.n_local} local, {args.copies} rotating cache copies",
                   "step": "magicpig_hash_query + magicpig_sampled_attention"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": stored_traffic(w.name),
                     "kernel": "scan_gather_kernel (dominant kernel of magicpig_sampled_attention)",
                     "avg_launch_ms": scan_ms, "algorithmic_bytes": kernel_bytes,
                     "code_bytes": scan_bytes, "row_bytes": gather_bytes,
                     "whole_step": {"algorithmic_bytes": alg_bytes, "achieved": path_gbs,
                                    "frac": path_gbs / HBM_PEAK_GBS,
                                    "what": "all kernels of the step (query hashing, scan_gather, merge): "
                                            "bytes / ms_per_step of the timed graph replay"},
                     "mean_sampled_per_head": float(n_sampled.mean())},
        "stage_ms": stage_ms, "launch": launch_mode, "gpu_ms_per_step": gpu_ms_per_step,
        "prefill_hash": {"ms": prefill_ms, "keys": w.batch * w.n_kv_heads * w.n_ctx,
                         "tflops": hash_flops / (prefill_ms * 1e-3) / 1e12,
                         "frac_of_bf16_mfma_peak": hash_flops / (prefill_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                         "what": "magicpig_key_mean + magicpig_hash_keys over the whole cache (one-time)"},
        "input_generation_s": gen_s,
    }
    if tables_info is not None:
        tables_info["max_abs_diff_vs_scan_output"] = float(np.abs(out_t - out0).max())
        result["hash_tables"] = tables_info
    if loop_info is not None:
        result["decode_loop"] = loop_info
    if not args.no_cpu_baseline:
        cb, ref, ref_heads = cpu_baseline(w, data, args.seed)
        result["cpu_baseline"] = cb
        err = max(float(np.abs(out0[b, h] - ref["out"][b, h]).max() / np.abs(ref["out"][b, h]).max())
                  for b, h in ref_heads)
        result["parity_vs_oracle_max_rel_err"] = err
        same_sets = all(int(n_sampled[b, h]) == ref["S"][b][h].size for b, h in ref_heads)
        result["parity_sample_sizes_equal"] = bool(same_sets)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
