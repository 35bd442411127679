"""Benchmark of the LSH-sampled decode attention hot path on one MI355X.

One step = one decode step of one layer at the C3 workload (Llama-3.1-8B shapes, batch 1,
32 query / 8 KV heads, head_dim 128, context 98304, bf16, SimHash K=10 L=150, >= 2 hits,
4 sink + 64 local): magicpig_hash_query_prepared + magicpig_sampled_attention (query coding,
collision scan, compaction, gather, importance-weighted softmax.V).  Inputs, key codes, the
centering vector and the prepared projector (a one-time, per-model re-layout of W) are resident
in HBM before the timed region.  The one-time prefill work (magicpig_key_mean +
magicpig_hash_keys over all 786432 keys) is timed separately and reported under
"prefill_hash".  Steps rotate over several independent copies of (codes, K,
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


def build_workload(w, data, copies: int):
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    kvt = torch.float8_e4m3fn if w.kv == "fp8" else tdt     # (the generator already rounded the values to the type)
    Kd = torch.from_numpy(data["K"]).to(kvt).cuda()
    Vd = torch.from_numpy(data["V"]).to(kvt).cuda()
    qd = torch.from_numpy(data["q"]).to(tdt).cuda()
    Wd = torch.from_numpy(data["W"]).to(tdt).cuda()
    params = mp.make_params(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, K=w.K,
                            L=w.L, n_ctx=w.n_ctx, dtype=w.dtype, min_hits=w.min_hits,
                            n_sink=w.n_sink, n_local=w.n_local, kv_dtype=w.kv)
    sets = []
    for c in range(copies):
        sets.append({
            "K": Kd if c == 0 else Kd.clone(), "V": Vd if c == 0 else Vd.clone(),
            "codes": mp.alloc_key_codes(params),
            "mu": torch.empty(w.batch, w.n_kv_heads, 128, dtype=torch.float32, device="cuda"),
        })
    return params, qd, Wd, sets


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
    # the same decode step with the host's cores: one process per core, each a share of the
    # heads (the oracle itself is unchanged; numpy threads held to one per process)
    ncores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    nproc = max(1, min(ncores, len(heads), 16))
    all_cores = None
    try:
        import multiprocessing as mpc
        chunks = [heads[i::nproc] for i in range(nproc)]
        ctx = mpc.get_context("fork")
        global _CPU_JOB
        _CPU_JOB = (sub, mu, codes, w)
        with ctx.Pool(nproc) as pool:
            pool.map(_cpu_heads, [[] for _ in range(nproc)])     # workers started and warm (not timed)
            reps = 5
            t0 = time.time()
            for _ in range(reps):
                pool.map(_cpu_heads, chunks)
            par_s = (time.time() - t0) / reps
        all_cores = {"value": len(heads) / par_s, "unit": "query-heads/s", "cores": nproc,
                     "host_cores_available": ncores, "seconds": par_s,
                     "sample": f"the same decode step, its {len(heads)} heads dealt over {nproc} worker processes "
                               f"(started beforehand), mean of {reps} passes"}
    except Exception as exc:  # noqa: BLE001
        all_cores = {"error": str(exc), "host_cores_available": ncores}
    return {
        "value": len(heads) / dec_s, "unit": "query-heads/s", "cores": 1, "kind": "oracle",
        "sample": f"decode step of the {len(heads)} query heads of batch element 0 at the full "
                  f"{w.n_ctx}-key context: {dec_s:.2f} s; before it the oracle hashed those "
                  f"{w.n_kv_heads * w.n_ctx} keys in {hash_s:.1f} s "
                  f"({w.n_kv_heads * w.n_ctx / hash_s:.0f} keys/s, not in value)",
        "all_cores": all_cores,
    }, ref, heads


_CPU_JOB = None


def _cpu_heads(heads):
    """Worker of the all-cores oracle leg: the decode step of some heads (forked: inputs are shared)."""
    from oracle import magicpig_oracle as oracle
    from threadpoolctl import threadpool_limits
    sub, mu, codes, w = _CPU_JOB
    if not heads:
        return 0
    with threadpool_limits(limits=1):
        oracle.decode_step(sub["q"], sub["K"], sub["V"], sub["W"], w.K, w.L, mu=mu, min_hits=w.min_hits,
                           n_sink=w.n_sink, n_local=w.n_local, key_codes=codes, heads=heads)
    return len(heads)


def stored_traffic(workload: str):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary
    (FETCH_SIZE and WRITE_SIZE, calibrated on a copy of known size): (bytes, file) or (None,
    None).  Counters cannot be read from inside this process: the figure is a stored one."""
    rel = os.path.join("profiles", f"scan_gather_{workload}_pmc.txt")
    try:
        with open(os.path.join(ROOT, rel)) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch"):
                    return float(line.split()[1]), rel
    except OSError:
        pass
    return None, None


def capture(fn):
    """One HIP graph of fn(), captured on a side stream."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            fn()
    torch.cuda.current_stream().wait_stream(side)
    g.replay()                              # untimed: the first replay uploads the graph
    torch.cuda.synchronize()
    return g


def timed_replays(graph, replays):
    """Wall-clock seconds of each of `replays` replays, synchronised on both sides."""
    out = []
    for _ in range(replays):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        graph.replay()
        torch.cuda.synchronize()
        out.append(time.perf_counter() - t0)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="C3")
    ap.add_argument("--copies", type=int, default=8)
    ap.add_argument("--replays", type=int, default=11, help="timed replays of the graph of `steps` steps (median reported)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-tables", action="store_true")
    ap.add_argument("--no-decode-loop", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path "
              "(the path shards by KV head without communication; see DESIGN.md)", file=sys.stderr)
        sys.exit(2)
    if torch.cuda.device_count() < 1:
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    mp.lib()

    w = wl.CONFIGS[args.workload]
    t0 = time.time()
    data = wl.generate(w, args.seed)
    gen_s = time.time() - t0
    # the CPU oracle leg runs first, before this process touches the GPU (it forks workers)
    cpu = None if args.no_cpu_baseline else cpu_baseline(w, data, args.seed)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    params, qd, Wd, sets = build_workload(w, data, args.copies)
    ws = mp.alloc_workspace(params)
    qcodes = mp.alloc_query_codes(params)
    out = torch.empty(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")

    prefill_ms = time_prefill(params, w, Wd, sets, ws)          # also produces codes and mu
    prefill_ms = time_prefill(params, w, Wd, sets, ws)          # second pass: warm

    # one-time, per model: the projector in the layout the few-vectors hashing reads
    prepared = mp.alloc_prepared_projector(params)
    mp.magicpig_prepare_projector(params, Wd, prepared)
    for s_ in sets:                         # per sequence: thresholds of the frozen centering vector
        s_["centering"] = mp.alloc_centering(params)
        mp.magicpig_prepare_centering(params, s_["mu"], prepared, s_["centering"])

    def step(i):
        s = sets[i % len(sets)]
        mp.magicpig_hash_query_prepared(params, qd, prepared, qcodes)
        mp.magicpig_sampled_attention(params, qd, s["K"], s["V"], s["mu"], s["codes"], qcodes, out,
                                      workspace=ws)

    # sample sizes for the algorithmic byte count (debug outputs, outside the timed region)
    ncand = torch.zeros(w.batch, w.n_q_heads, dtype=torch.int32, device="cuda")
    cand_cap = max(4096, w.n_ctx // 16)
    cand = torch.zeros(w.batch, w.n_q_heads, cand_cap, dtype=torch.int32, device="cuda")
    mp.magicpig_hash_query(params, qd, Wd, qcodes, ws)
    qcodes_plain = qcodes.clone()
    mp.magicpig_hash_query_prepared(params, qd, prepared, qcodes)
    assert torch.equal(qcodes, qcodes_plain), "prepared and plain query hashing disagree"
    mp.magicpig_sampled_attention(params, qd, sets[0]["K"], sets[0]["V"], sets[0]["mu"], sets[0]["codes"],
                                  qcodes, out, None, cand, ncand, ws)
    torch.cuda.synchronize()
    n_sampled = ncand.cpu().numpy().astype(np.int64)
    cand_host = cand.cpu().numpy()
    out0 = out.cpu().numpy().copy()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` decode steps, captured in one HIP graph so that the host's
    # launch cost (python + ctypes, several microseconds per call) is not what is measured; the
    # graph is replayed `replays` times, each replay timed on its own by the wall clock between
    # two synchronisations, and the median replay gives ms_per_step.  If capture is unavailable
    # the same steps are timed as eager launches.
    launch_mode = "hipgraph"
    try:
        graph = capture(lambda: [step(i) for i in range(args.steps)])
    except Exception as exc:  # noqa: BLE001
        print(f"graph capture failed ({exc}); timing eager launches", file=sys.stderr)
        graph, launch_mode = None, "eager"
    if graph is not None:
        walls = timed_replays(graph, args.replays)
    else:
        walls = []
        for _ in range(args.replays):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(args.steps):
                step(i)
            torch.cuda.synchronize()
            walls.append(time.perf_counter() - t0)
    wall = float(np.median(walls))
    ms_per_step = wall * 1e3 / args.steps
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    if graph is not None:
        graph.replay()
    else:
        for i in range(args.steps):
            step(i)
    e1.record()
    torch.cuda.synchronize()
    gpu_ms_per_step = e0.elapsed_time(e1) / args.steps
    heads = w.batch * w.n_q_heads
    value = heads / (ms_per_step * 1e-3)

    # ---- per-kernel durations, live: HIP events attached to the kernels of the same steps (eager
    # launches on torch's current stream), which carry each kernel's own begin / end timestamps
    hip = ctypes.CDLL("libamdhip64.so")
    n_ev = min(max(args.steps, 20), 100)
    evs = []
    for _ in range(n_ev):
        group = []
        for _ in range(7):
            e = ctypes.c_void_p()
            assert hip.hipEventCreate(ctypes.byref(e)) == 0
            group.append(e)
        evs.append(group)
    for i in range(n_ev):
        mp.magicpig_profile_stage_events([e.value for e in evs[i]])
        step(i)
    mp.magicpig_profile_stage_events(None)
    torch.cuda.synchronize()

    def span(a, b):
        ms = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
        return ms.value
    # events 5 / 6: begin / end of the query-hashing kernel; 0 / 1: of scan_gather_kernel; 4 / 3: of
    # the merge kernel
    stage_ms = {
        "hash_query": float(np.median([span(g[5], g[6]) for g in evs])),
        "scan_gather": float(np.mean([span(g[0], g[1]) for g in evs])),
        "merge": float(np.median([span(g[4], g[3]) for g in evs])),
        "what": "kernel begin-to-end timestamps (hipExtLaunchKernel events) over eager launches of the same steps; "
                "scan_gather is the average the roofline uses, the others medians",
    }
    for group in evs:
        for e in group:
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
            mp.magicpig_hash_query_prepared(params, qd, prepared, qcodes)
            mp.magicpig_sampled_attention_tables(params, qd, s_["K"], s_["V"], s_["mu"], s_["tables"], w.n_ctx,
                                                 s_["codes"], qcodes, out, workspace=ws)
        for i in range(args.warmup):
            tstep(i)
        torch.cuda.synchronize()
        out_t = out.cpu().numpy().copy()
        g2 = capture(lambda: [tstep(i) for i in range(args.steps)])
        t_ms = float(np.median(timed_replays(g2, args.replays))) * 1e3 / args.steps
        tables_info = {"value": heads / (t_ms * 1e-3), "unit": "query-heads/s", "ms_per_step": t_ms,
                       "build_ms": b0.elapsed_time(b1) / len(sets),
                       "table_bytes": mp.magicpig_table_bytes(params),
                       "build_workspace_bytes": mp.magicpig_table_build_workspace_bytes(params),
                       "what": "magicpig_hash_query_prepared + magicpig_sampled_attention_tables, HIP graph; "
                               "build = magicpig_build_tables per cache copy (one-time)"}

    # ---- the decode loop this path sits in: tokens generated one after the other by a 32-layer
    # model.  Per token the context grows by one key (its length lives in device memory and is
    # advanced inside the graph); per layer the token's key of every KV head is coded behind the
    # frozen mean together with the queries (magicpig_hash_decode_step_prepared) and the attention
    # runs.  Layers cycle over the cache copies; one HIP graph, captured once, is replayed for
    # every token.  In the table form the tables are rebuilt every `rebuild_period` tokens; the
    # timed tokens are the last ones before a rebuild, when the most keys (found by the scan of
    # their codes) lie behind the tables.
    loop_info = None
    if not args.no_decode_loop:
        layers, rebuild_period, tokens = 32, 2048, 48
        n0 = w.n_ctx - tokens - 2                           # context before the first timed token
        n_idx = max(0, (w.n_ctx - rebuild_period) // 64 * 64)
        n_dev = torch.zeros(1, dtype=torch.int64, device="cuda")
        live = mp.make_params(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, K=w.K, L=w.L,
                              n_ctx=w.n_ctx, dtype=w.dtype, min_hits=w.min_hits, n_sink=w.n_sink,
                              n_local=w.n_local, n_ctx_dev=n_dev, kv_dtype=w.kv)

        def token(form):
            n_dev.add_(1)
            for l in range(layers):
                s_ = sets[l % len(sets)]
                mp.magicpig_hash_decode_step_prepared(live, qd, s_["K"], s_["mu"], s_["centering"], prepared, 0, 1,
                                                      s_["codes"], qcodes)
                if form == "tables":
                    mp.magicpig_sampled_attention_tables(live, qd, s_["K"], s_["V"], s_["mu"], s_["tables"],
                                                         n_idx, s_["codes"], qcodes, out, workspace=ws)
                else:
                    mp.magicpig_sampled_attention(live, qd, s_["K"], s_["V"], s_["mu"], s_["codes"], qcodes,
                                                  out, workspace=ws)

        def time_tokens(form):
            n_dev.fill_(n0 - 2)
            token(form)                                     # eager warm-up token
            g3 = capture(lambda: token(form))               # (capture + its first replay: one more token)
            assert int(n_dev.item()) == n0
            per_token = timed_replays(g3, tokens)           # the context grows by one key per replay
            assert int(n_dev.item()) == n0 + tokens
            return float(np.median(per_token)) * 1e3

        codes_before = sets[0]["codes"].clone()
        loop_info = {"layers": layers, "tokens_timed": tokens, "context": [n0 + 1, n0 + tokens],
                     "scan_ms_per_token": time_tokens("scan"),
                     "what": "per token: context length + 1 (device memory, inside the graph); per layer: "
                             "magicpig_hash_decode_step_prepared (the token's key of each KV head + the queries) "
                             "+ attention; 32 layers in one HIP graph captured once and replayed per token; "
                             "median over the tokens"}
        # (the keys the loop coded are keys the prefill had coded with the same mean: nothing changed)
        loop_info["codes_unchanged_by_the_loop"] = bool(torch.equal(codes_before, sets[0]["codes"]))
        if tables_info is not None:
            p_idx = mp.make_params(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, K=w.K, L=w.L,
                                   n_ctx=n_idx, n_cap=w.n_ctx, dtype=w.dtype, min_hits=w.min_hits,
                                   n_sink=w.n_sink, n_local=w.n_local, kv_dtype=w.kv)
            for s_ in sets:
                mp.magicpig_build_tables(p_idx, s_["codes"], s_["tables"], bws)
            loop_info["tables_ms_per_token"] = time_tokens("tables")
            loop_info["table_rebuild_period_tokens"] = rebuild_period
            loop_info["keys_behind_the_tables"] = [n0 + 1 - n_idx, n0 + tokens - n_idx]
            loop_info["table_rebuild_ms_per_layer"] = tables_info["build_ms"]
            # the last token of either form attended the same context: same sample, same output
            o_t = out.cpu().numpy().copy()
            n_dev.fill_(n0 + tokens - 1)
            token("scan")
            torch.cuda.synchronize()
            loop_info["max_abs_diff_tables_vs_scan_output"] = float(np.abs(o_t - out.cpu().numpy()).max())

    n_static = min(w.n_ctx, w.n_sink + w.n_local)
    scan_bytes = w.batch * w.n_kv_heads * max(w.n_ctx - n_static, 0) * w.K * w.L / 8.0
    kv_elem_bytes = 1 if w.kv == "fp8" else (2 if w.dtype == "bf16" else 4)
    gather_bytes = float((n_sampled + n_static).sum()) * 2 * 128 * kv_elem_bytes
    out_bytes = heads * 128 * 4
    alg_bytes = scan_bytes + gather_bytes + out_bytes
    # the dominant kernel streams the codes of the eligible keys and gathers the K and V rows
    # of the attended ones: both are its algorithmic bytes
    kernel_bytes = scan_bytes + gather_bytes
    achieved = kernel_bytes / (scan_ms * 1e-3) / 1e9
    path_gbs = alg_bytes / (ms_per_step * 1e-3) / 1e9

    hash_flops = 2.0 * w.batch * w.n_kv_heads * w.n_ctx * 128 * w.K * w.L
    traffic, traffic_src = stored_traffic(w.name)
    if traffic_src is not None:
        traffic_src += " (stored rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE summary, not measured in this run)"
    result = {
        "metric": METRIC, "value": value, "unit": "query-heads/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("bf16" if w.dtype == "bf16" else "f32") + (" (K / V cache: fp8 e4m3)" if w.kv == "fp8" else ""),
        "data": "synthetic",
        "config": {"workload": f"{w.name}: batch {w.batch}, {w.n_q_heads} query / {w.n_kv_heads} KV heads, "
                               f"head_dim 128, context {w.n_ctx}, K={w.K} L={w.L}, min_hits {w.min_hits}, "
                               f"{w.n_sink} sink + {w.n_local} local, {args.copies} rotating cache copies",
                   "step": "magicpig_hash_query_prepared + magicpig_sampled_attention",
                   "timing": f"median of {args.replays} replays of one HIP graph of {args.steps} steps"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_src,
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
    if cpu is not None:
        cb, ref, ref_heads = cpu
        result["cpu_baseline"] = cb
        err = max(float(np.abs(out0[b, h] - ref["out"][b, h]).max() / np.abs(ref["out"][b, h]).max())
                  for b, h in ref_heads)
        result["parity_vs_oracle_max_rel_err"] = err
        same_sets = all(int(n_sampled[b, h]) == ref["S"][b][h].size and n_sampled[b, h] <= cand_cap and
                        np.array_equal(np.sort(cand_host[b, h, :n_sampled[b, h]]), ref["S"][b][h]) for b, h in ref_heads)
        result["parity_sample_sets_equal"] = bool(same_sets)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
