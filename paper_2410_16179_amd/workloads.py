"""Seeded synthetic inputs for LSH-sampled decode attention.

This module only *draws numbers*: it contains none of the method's arithmetic (no
hashing, no key mean, no probabilities, no attention).  It serves the HIP path, the
tests and the benchmark alike, so that every side sees identical bits.  Everything is
generated on the host with numpy's counter-based Philox generator; arrays are returned
as float32 whose values are exactly representable in the configuration's storage type
(bf16 values are float32 numbers with the low 16 mantissa bits cleared by
round-to-nearest-even), so any consumer converts them without rounding.

Geometry (stand-in for real LLM activations, which show keys packed in a narrow cone
with a large shared mean and queries lying away from it): per (batch, KV head) a shared
offset m ~ N(0, 4 I), keys k_i = m + N(0, I), values v_i ~ N(0, I); per query head
q = 0.8 * normalize(sum of P "planted" keys drawn from the LSH-eligible range) +
N(0, 0.25 I); projector W with iid N(0, 1) entries, one for all heads.
"""
from __future__ import annotations

import dataclasses
import zlib

import numpy as np


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    n_ctx: int
    K: int            # sign bits per table
    L: int            # tables
    dtype: str        # "bf16" | "fp32": storage type of q, K, V, W
    planted: tuple    # planted keys per query head: one int, or (first half, second half)
    head_dim: int = 128
    min_hits: int = 2
    n_sink: int = 4
    n_local: int = 64
    kv: str = ""      # storage type of the K / V cache when it differs from dtype: "fp8" (OCP e4m3)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def planted_for_head(self, h: int) -> int:
        if len(self.planted) == 1:
            return self.planted[0]
        return self.planted[0] if h < self.n_q_heads // 2 else self.planted[1]


# The five named configurations (C1..C5).
CONFIGS = {
    "C1": Workload("C1", 1, 1, 1, 4096, 8, 75, "fp32", (16,)),
    "C2": Workload("C2", 1, 32, 8, 16384, 10, 150, "bf16", (32,)),
    "C3": Workload("C3", 1, 32, 8, 98304, 10, 150, "bf16", (32,)),
    "C4": Workload("C4", 16, 32, 8, 65536, 9, 120, "bf16", (8, 512)),
    "C5": Workload("C5", 8, 64, 8, 131072, 10, 170, "bf16", (32,)),
}
# The benchmark shape (C3) with the larger table sets of the paper's (K, L) study (App. E).
CONFIGS["C3_K10_L220"] = Workload("C3_K10_L220", 1, 32, 8, 98304, 10, 220, "bf16", (32,))
CONFIGS["C3_K11_L300"] = Workload("C3_K11_L300", 1, 32, 8, 98304, 11, 300, "bf16", (32,))
# The benchmark shape with a quantised (e4m3) K / V cache (App. "Limitations and future work").
CONFIGS["C3_fp8kv"] = Workload("C3_fp8kv", 1, 32, 8, 98304, 10, 150, "bf16", (32,), kv="fp8")


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest bf16 value (ties to even), returned as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def round_to_e4m3(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest OCP e4m3 value (4 exponent bits, bias 7; 3 mantissa bits; subnormals in
    steps of 2^-9; largest value 448, larger magnitudes are clamped to it; ties to even), as float32."""
    x = np.clip(np.ascontiguousarray(x, dtype=np.float32), -448.0, 448.0)
    mag = np.abs(x).astype(np.float64)
    e = np.floor(np.log2(np.maximum(mag, 2.0 ** -20)))
    step = 2.0 ** (np.maximum(e, -6.0) - 3.0)               # spacing of the values around |x|
    y = np.minimum(np.rint(mag / step) * step, 448.0)
    return (np.sign(x) * y).astype(np.float32)


def store(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "fp8":
        return round_to_e4m3(x)
    return round_to_bf16(x) if dtype == "bf16" else x


def _rng(seed: int, wl: Workload, tag: str, *idx: int) -> np.random.Generator:
    words = [seed & 0xFFFFFFFF, zlib.crc32(wl.name.encode()), zlib.crc32(tag.encode())]
    words += [int(i) & 0xFFFFFFFF for i in idx]
    return np.random.Generator(np.random.Philox(np.random.SeedSequence(words)))


def projector(wl: Workload, seed: int = 0) -> np.ndarray:
    """W [head_dim, K*L]; column t*K + b is hyperplane b of table t."""
    g = _rng(seed, wl, "W")
    return store(g.standard_normal((wl.head_dim, wl.K * wl.L), dtype=np.float32), wl.dtype)


def keys_values(wl: Workload, b: int, g: int, seed: int = 0):
    """(K, V) of one (batch, KV head): two [n_ctx, head_dim] float32 arrays."""
    r = _rng(seed, wl, "KV", b, g)
    m = 2.0 * r.standard_normal(wl.head_dim, dtype=np.float32)
    K = r.standard_normal((wl.n_ctx, wl.head_dim), dtype=np.float32)
    K += m
    V = r.standard_normal((wl.n_ctx, wl.head_dim), dtype=np.float32)
    return store(K, wl.kv or wl.dtype), store(V, wl.kv or wl.dtype)


def query(wl: Workload, b: int, h: int, K_g: np.ndarray, seed: int = 0,
          alpha: float = 0.8, center: np.ndarray | None = None) -> np.ndarray:
    """q [head_dim] of query head h, built from its KV head's keys K_g.

    alpha and center are test knobs: alpha scales the planted direction (0.8 in every
    reported configuration) and center, if given, is subtracted from the planted keys
    before they are summed (used only to produce queries with large inclusion
    probabilities for numerical coverage).
    """
    r = _rng(seed, wl, "Q", b, h)
    lo, hi = wl.n_sink, max(wl.n_ctx - wl.n_local, wl.n_sink + 1)
    hi = min(hi, wl.n_ctx)
    P = min(wl.planted_for_head(h), max(hi - lo, 1))
    idx = r.choice(np.arange(lo, hi), size=P, replace=False) if hi > lo else np.zeros(1, np.int64)
    rows = K_g[idx].astype(np.float64)
    if center is not None:
        rows = rows - np.asarray(center, dtype=np.float64)
    s = rows.sum(axis=0)
    nrm = np.linalg.norm(s)
    direction = s / nrm if nrm > 0 else s
    noise = 0.5 * r.standard_normal(wl.head_dim, dtype=np.float32)
    return store(alpha * direction + noise, wl.dtype)


def generate(wl: Workload, seed: int = 0, alpha: float = 0.8):
    """All tensors of a workload: dict with K, V [B,Hkv,n,d], q [B,Hq,d], W [d,K*L]."""
    B, Hq, Hkv, n, d = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.n_ctx, wl.head_dim
    K = np.empty((B, Hkv, n, d), np.float32)
    V = np.empty((B, Hkv, n, d), np.float32)
    q = np.empty((B, Hq, d), np.float32)
    for b in range(B):
        for g in range(Hkv):
            K[b, g], V[b, g] = keys_values(wl, b, g, seed)
            for h in range(g * wl.group, (g + 1) * wl.group):
                q[b, h] = query(wl, b, h, K[b, g], seed, alpha)
    return {"K": K, "V": V, "q": q, "W": projector(wl, seed)}


def scaled(wl: Workload, **changes) -> Workload:
    """A copy of a named workload with some fields changed (test sizes)."""
    return dataclasses.replace(wl, **changes)
