"""The decode step through the entry point that allocates nothing and takes no workspace
(magicpig_sampled_attention_noalloc: partial results in the library's static device array)
against magicpig_sampled_attention on the same inputs: same kernels, so the outputs must be
equal bit for bit; the workspace form is also held to the oracle."""
import numpy as np
import pytest
import torch

from paper_2410_16179_amd import binding as mp
from paper_2410_16179_amd import workloads as wl
from tests.gpu_helpers import Session, TOL, rel_err

pytestmark = pytest.mark.gpu


def _one_call(oracle, w, seed):
    print(f"[case] noalloc B={w.batch} Hq={w.n_q_heads} Hkv={w.n_kv_heads} n={w.n_ctx} K={w.K} L={w.L} seed={seed}",
          flush=True)
    data = wl.generate(w, seed)
    mu = np.stack([[oracle.key_mean(data["K"][b, g]) for g in range(w.n_kv_heads)]
                   for b in range(w.batch)]).astype(np.float32)
    s = Session(K=w.K, L=w.L, dtype=w.dtype, Kc=data["K"], Vc=data["V"], q=data["q"], W=data["W"])
    s.set_mu(mu)
    s.hash_keys()
    s.hash_query()
    with_workspace = s.attend(debug=False)["out"]
    out = torch.full((w.batch, w.n_q_heads, 128), float("nan"), dtype=torch.float32, device="cuda")
    mp.magicpig_sampled_attention_noalloc(s.params, s.q, s.Kc, s.Vc, s.mu, s.key_codes, s.q_codes, out)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.cpu().numpy(), with_workspace)
    heads = [(0, 0), (w.batch - 1, w.n_q_heads - 1)]
    ref = oracle.decode_step(data["q"], data["K"], data["V"], data["W"], w.K, w.L, mu=mu, heads=heads)
    for b, h in heads:
        assert rel_err(out.cpu().numpy()[b, h][None], ref["out"][b, h][None]) <= TOL


def test_two_calls_in_a_row_the_second_smaller(oracle):
    assert torch.cuda.is_available()
    # 32 heads x 20000 keys (79 runs of key blocks per head), then 8 heads x 3001 keys: the second
    # call finds the first call's partial results in the array and must not be disturbed by them
    _one_call(oracle, wl.scaled(wl.CONFIGS["C2"], n_ctx=20000), seed=3)
    _one_call(oracle, wl.scaled(wl.CONFIGS["C2"], n_ctx=3001, n_q_heads=8, n_kv_heads=2), seed=4)
    # and a float32 problem of another table shape
    _one_call(oracle, wl.scaled(wl.CONFIGS["C1"], n_ctx=1500), seed=5)


def test_a_step_beyond_the_static_array_is_refused():
    p = mp.make_params(batch=8, n_q_heads=64, n_kv_heads=8, K=10, L=170, n_ctx=131072, dtype="bf16")
    t = torch.zeros(64, dtype=torch.int32, device="cuda")
    with pytest.raises(mp.MagicpigError, match="static"):
        mp.magicpig_sampled_attention_noalloc(p, t, t, t, None, t, t, t)
