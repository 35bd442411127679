"""GPU parity at the full sizes of the named configurations, through the same calls and
launch configuration that bench.py times.  Where the oracle cannot cover everything in
seconds, it covers every key of some (batch, KV head) units and all their query heads."""
import numpy as np
import pytest
import torch

from paper_2410_16179_amd import binding as mp
from paper_2410_16179_amd import workloads as wl
from tests.test_gpu_parity import run_case

pytestmark = pytest.mark.gpu


def test_c2_full_all_heads(oracle):
    ref, res, worst = run_case(oracle, wl.CONFIGS["C2"], oracle_codes_too=False)
    frac = np.mean([ref["S"][0][h].size for h in range(32)]) / 16384
    assert 0.005 < frac < 0.04           # (10,150): a per cent or two of the keys
    print(f"   C2 sampled fraction {frac:.4f}, worst output error {worst:.2e}", flush=True)


def test_c3_full_two_kv_heads(oracle):
    # 96k context, the benchmark workload: every key code of KV heads 0 and 5, and the eight
    # query heads that use them (counts, sample sets, outputs)
    heads = [(0, h) for h in (0, 1, 2, 3, 20, 21, 22, 23)]
    ref, res, worst = run_case(oracle, wl.CONFIGS["C3"], heads=heads, oracle_codes_too=False)
    print(f"   C3 worst output error {worst:.2e}", flush=True)
    # properties that hold for all heads at any size: output finite, inside the value range
    assert np.isfinite(res["out"]).all()
    assert np.abs(res["out"]).max() < 6.0


def test_c4_one_sequence_peaked_and_flat_heads(oracle):
    # one of the 16 sequences at the full 65536 context; peaked (8 planted) and flat (512) heads
    w = wl.scaled(wl.CONFIGS["C4"], batch=1)
    heads = [(0, h) for h in (0, 3, 16, 19, 28, 31)]
    run_case(oracle, w, heads=heads, oracle_codes_too=False)


def test_c5_one_sequence_group_of_eight(oracle):
    # 70B shapes (8 query heads per KV head, L = 170) at the full 131072 context, one sequence
    w = wl.scaled(wl.CONFIGS["C5"], batch=1)
    heads = [(0, h) for h in range(8, 16)]
    run_case(oracle, w, heads=heads, oracle_codes_too=False)


def _finite_and_bounded(res, B, Hq):
    # properties that hold for every head at any size: finite, inside the range of the values
    out = res["out"]
    assert out.shape == (B, Hq, 128) and np.isfinite(out).all() and np.abs(out).max() < 6.0


def test_c4_whole_batch_at_full_context(oracle):
    # batch 16 x 65536 keys, the launch shape the benchmark times for this workload (many rounds of
    # workgroups in the scan + gather, separate lookup and gather launches through the tables, the
    # 16-wavefront merge).  The GPU runs all 512 heads; the oracle checks every key code of seven
    # (batch, KV head) units in the first, a middle and the last sequence, random keys of every
    # unit, and counts, samples and outputs of seven heads there, peaked (h < 16) and flat.
    w = wl.CONFIGS["C4"]
    heads = [(0, 0), (0, 17), (7, 5), (7, 30), (15, 3), (15, 16), (15, 31)]
    ref, res, worst = run_case(oracle, w, heads=heads, oracle_codes_too=False, random_rows=700)
    _finite_and_bounded(res, w.batch, w.n_q_heads)
    print(f"   C4 whole batch: {len(heads)} of {w.batch * w.n_q_heads} heads checked against the oracle, "
          f"worst output error {worst:.2e}", flush=True)


def test_c5_whole_batch_at_full_context(oracle):
    # batch 8 x 131072 keys, 64 query heads (groups of eight), (10,170)
    w = wl.CONFIGS["C5"]
    heads = [(0, 7), (0, 40), (3, 21), (3, 63), (7, 0), (7, 33), (7, 58)]
    ref, res, worst = run_case(oracle, w, heads=heads, oracle_codes_too=False, random_rows=1400)
    _finite_and_bounded(res, w.batch, w.n_q_heads)
    print(f"   C5 whole batch: {len(heads)} of {w.batch * w.n_q_heads} heads checked against the oracle, "
          f"worst output error {worst:.2e}", flush=True)


@pytest.mark.parametrize("name", ["C3_K10_L220", "C3_K11_L300"])
def test_larger_tables_of_the_hyperparameter_study_at_long_context(oracle, name):
    # (10,220) and (11,300) of App. E at 65536 keys: their own scan instantiations (69 and 104 code
    # words per key) and, for 300 tables, the table path beyond 255 tables (16-bit hit counters in
    # the counting lookup); every key code of two KV heads, four query heads
    w = wl.scaled(wl.CONFIGS[name], n_ctx=65536)
    heads = [(0, 5), (0, 6), (0, 30), (0, 31)]
    ref, res, worst = run_case(oracle, w, heads=heads, oracle_codes_too=False, indexed=(61440,))
    frac = np.mean([ref["S"][0][h].size for _, h in heads]) / w.n_ctx
    print(f"   {name}: sampled fraction {frac:.4f} (App. E budget for orthogonal vectors: {oracle.expected_budget(w.K, w.L):.4f}), "
          f"worst output error {worst:.2e}", flush=True)
    assert 0.5 * oracle.expected_budget(w.K, w.L) < frac < 4 * oracle.expected_budget(w.K, w.L)


def test_c3_ragged_context_in_a_larger_cache(oracle):
    # the benchmark shape with a context that ends inside a code block and inside a run of
    # blocks (the last workgroup of a KV head scans fewer blocks than the others and a part of its
    # last one), in a cache with spare capacity; the last KV head, all four of its query heads
    w = wl.scaled(wl.CONFIGS["C3"], n_ctx=98304 - 4 * 64 - 37)
    heads = [(0, h) for h in (28, 29, 30, 31)]
    ref, res, worst = run_case(oracle, w, heads=heads, n_cap=98304, oracle_codes_too=False)
    assert np.isfinite(res["out"]).all()


def test_100000_keys_runs_of_twenty_blocks(oracle):
    # 8 KV heads x 100000 keys: runs of 16 key blocks would leave a few workgroups for a second
    # round, so the scan + gather takes runs of 20 (five per wavefront), the last one partial
    w = wl.scaled(wl.CONFIGS["C3"], n_ctx=100000)
    heads = [(0, h) for h in (12, 13, 14, 15)]
    ref, res, worst = run_case(oracle, w, heads=heads, oracle_codes_too=False)
    assert np.isfinite(res["out"]).all()
