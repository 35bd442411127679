"""Shared plumbing of the GPU parity tests: upload inputs, run the HIP path through the
binding, bring results back in the oracle's canonical forms."""
from __future__ import annotations

import numpy as np
import torch

from paper_2410_16179_amd import binding as mp

TOL = 2e-3   # max relative error of attention outputs (fp32 accumulate, bf16 K/V)


def to_dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    if dtype == "bf16":
        t16 = t.to(torch.bfloat16)
        assert torch.equal(t16.to(torch.float32), t), "inputs must be bf16-representable"
        t = t16
    elif dtype == "fp8":
        t8 = t.to(torch.float8_e4m3fn)
        assert torch.equal(t8.to(torch.float32), t), "inputs must be e4m3-representable"
        t = t8
    return t.cuda()


def pack_table_codes(codes: np.ndarray, K: int, L: int, pad_bit: int) -> np.ndarray:
    """[..., L] canonical integers -> [..., K*ceil(L/32)] plane words (inverse of table_codes_from_words)."""
    Wd = (L + 31) // 32
    codes = np.asarray(codes).astype(np.uint32)
    full = np.zeros(codes.shape[:-1] + (Wd * 32,), np.uint32)
    full[..., :L] = codes
    if pad_bit:
        full[..., L:] = (1 << K) - 1
    full = full.reshape(codes.shape[:-1] + (Wd, 32))
    words = np.zeros(codes.shape[:-1] + (Wd, K), np.uint32)
    for b in range(K):
        bits = (full >> np.uint32(b)) & np.uint32(1)
        words[..., b] = (bits << np.arange(32, dtype=np.uint32)).sum(axis=-1, dtype=np.uint64).astype(np.uint32)
    return words.reshape(codes.shape[:-1] + (Wd * K,))


class Session:
    """Device buffers of one problem instance."""

    def __init__(self, *, K, L, dtype, Kc, Vc, q, W, n_ctx=None, min_hits=2, n_sink=4, n_local=64,
                 layout="dense", n_ctx_dev=None, kv=""):
        """layout "dense": K and V caches [B, Hkv, n_cap, 128]; "token_major": both caches stored
        [B, n_cap, Hkv, row] with the heads of a token next to each other, K rows of 128 elements
        and V rows padded to 160, handed to the library through its stride arguments."""
        B, Hkv, n_cap, d = Kc.shape
        self.B, self.Hq, self.Hkv, self.K, self.L = B, q.shape[1], Hkv, K, L
        self.n_cap = n_cap
        self.n = n_cap if n_ctx is None else n_ctx
        self.dtype = dtype
        self._pkw = dict(batch=B, n_q_heads=self.Hq, n_kv_heads=Hkv, K=K, L=L, n_cap=n_cap, dtype=dtype,
                         min_hits=min_hits, n_sink=n_sink, n_local=n_local, n_ctx_dev=n_ctx_dev, kv_dtype=kv)
        self.Kc, self.Vc = (to_dev(x, kv or dtype) for x in (Kc, Vc))     # kv = "fp8": caches of e4m3 bytes
        self.q, self.W = (to_dev(x, dtype) for x in (q, W))
        if layout == "token_major":
            vrow = 160
            kt = self.Kc.permute(0, 2, 1, 3).contiguous()                       # [B, n_cap, Hkv, 128]
            vt = torch.full((B, n_cap, Hkv, vrow), float("nan"), dtype=torch.bfloat16, device="cuda").to(self.Vc.dtype)
            vt[..., :d] = self.Vc.permute(0, 2, 1, 3)
            self.Kc, self.Vc = kt, vt
            self._pkw["k_strides"] = (n_cap * Hkv * d, d, Hkv * d)
            self._pkw["v_strides"] = (n_cap * Hkv * vrow, vrow, Hkv * vrow)
        else:
            assert layout == "dense"
        self.params = mp.make_params(n_ctx=self.n, **self._pkw)
        self.key_codes = mp.alloc_key_codes(self.params)
        self.q_codes = mp.alloc_query_codes(self.params)
        self.ws = mp.alloc_workspace(self.params)
        self.mu = None
        self.NW = mp.magicpig_code_words_per_key(self.params)
        self.NQ = mp.magicpig_code_words_per_query(self.params)

    def set_mu(self, mu: np.ndarray | None):
        self.mu = None if mu is None else torch.from_numpy(np.ascontiguousarray(mu, np.float32)).cuda()

    def key_mean(self) -> np.ndarray:
        out = torch.empty(self.B, self.Hkv, 128, dtype=torch.float32, device="cuda")
        mp.magicpig_key_mean(self.params, self.Kc, out, self.ws)
        torch.cuda.synchronize()
        return out.cpu().numpy()

    def hash_keys(self, first=0, count=None):
        count = self.n_cap - first if count is None else count
        mp.magicpig_hash_keys(self.params, self.Kc, self.mu, self.W, first, count, self.key_codes, self.ws)

    def hash_query(self):
        mp.magicpig_hash_query(self.params, self.q, self.W, self.q_codes, self.ws)

    def prepare(self):
        """Prepared projector (once per model) and, if there is a centering vector, its thresholds."""
        self.prepared = mp.alloc_prepared_projector(self.params)
        mp.magicpig_prepare_projector(self.params, self.W, self.prepared)
        self.centering = None
        if self.mu is not None:
            self.centering = mp.alloc_centering(self.params)
            mp.magicpig_prepare_centering(self.params, self.mu, self.prepared, self.centering)

    def hash_query_prepared(self, q_codes=None):
        mp.magicpig_hash_query_prepared(self.params, self.q, self.prepared, self.q_codes if q_codes is None else q_codes)

    def hash_keys_prepared(self, first, count, key_codes=None, q_codes=None):
        """Keys [first, first + count) (and the queries, if q_codes is given) through the prepared form."""
        mp.magicpig_hash_decode_step_prepared(self.params, self.q, self.Kc, self.mu, self.centering, self.prepared,
                                              first, count, self.key_codes if key_codes is None else key_codes, q_codes)

    def key_table_codes(self) -> np.ndarray:
        """[B, Hkv, n_cap, L] canonical codes read back from the packed buffer."""
        torch.cuda.synchronize()
        raw = self.key_codes.cpu().numpy().view(np.uint32)
        words = raw[mp.key_code_gather_index(self.params)]
        return mp.table_codes_from_words(mp.key_plane_words(words, self.K, self.L), self.K, self.L)

    def key_table_codes_unit(self, b: int, g: int, rows=None) -> np.ndarray:
        """[n_cap, L] (or [len(rows), L]) canonical codes of one (batch, KV head): reads only that
        unit's part of the packed buffer."""
        torch.cuda.synchronize()
        one = mp.make_params(**{**self._pkw, "batch": 1, "n_kv_heads": 1, "n_q_heads": 1,
                                "k_strides": None, "v_strides": None, "n_ctx_dev": None, "kv_dtype": 0}, n_ctx=self.n)
        idx = mp.key_code_gather_index(one)[0, 0]                       # [n_cap, NW] inside the unit
        per_unit = (self.n_cap + 63) // 64 * 64 * self.NW
        u = b * self.Hkv + g
        raw = self.key_codes[u * per_unit:(u + 1) * per_unit].cpu().numpy().view(np.uint32)
        words = raw[idx if rows is None else idx[np.asarray(rows)]]
        return mp.table_codes_from_words(mp.key_plane_words(words, self.K, self.L), self.K, self.L)

    def query_table_codes(self) -> np.ndarray:
        torch.cuda.synchronize()
        raw = self.q_codes.cpu().numpy().view(np.uint32)[: self.B * self.Hq * self.NQ]
        return mp.table_codes_from_words(raw.reshape(self.B, self.Hq, self.NQ), self.K, self.L)

    def upload_codes(self, key_codes: np.ndarray, q_codes: np.ndarray):
        """Install oracle codes ([B,Hkv,n_cap,L], [B,Hq,L]) in the packed device layout."""
        idx = mp.key_code_gather_index(self.params)
        raw = np.zeros(self.key_codes.numel(), np.uint32)
        raw[idx.ravel()] = mp.key_words_from_planes(pack_table_codes(key_codes, self.K, self.L, 0),
                                                    self.K, self.L).ravel()
        self.key_codes.copy_(torch.from_numpy(raw.view(np.int32)))
        qw = pack_table_codes(q_codes, self.K, self.L, 1).ravel()
        self.q_codes[: qw.size].copy_(torch.from_numpy(qw.view(np.int32)))

    def build_tables(self, n_indexed=None, big_workspace=True):
        """Tables over the keys [0, n_indexed) (default: all); later keys are left to the scan.
        big_workspace: the two-pass build (codes per table in the workspace) or the one-pass scatter."""
        self.n_indexed = self.n if n_indexed is None else n_indexed
        self.tables = mp.alloc_tables(self.params)
        pb = mp.make_params(n_ctx=self.n_indexed, **self._pkw)
        ws = mp.alloc_table_build_workspace(pb) if big_workspace else None
        mp.magicpig_build_tables(pb, self.key_codes, self.tables, ws)
        torch.cuda.synchronize()

    def table_buckets(self):
        """offsets [units, L, 2^K + 1] and indices [units, L, n_cap] of the built tables (host copies)."""
        units, L, nb = self.B * self.Hkv, self.L, 1 << self.K
        raw = self.tables.cpu().numpy().view(np.uint32)
        noff = units * L * (nb + 1)
        o0 = 256 // 4                                     # behind the header
        off = raw[o0:o0 + noff].reshape(units, L, nb + 1)
        start = o0 + (noff * 4 + 255) // 256 * 256 // 4
        idx = raw[start:start + units * L * self.n_cap].reshape(units, L, self.n_cap)
        return off, idx

    def table_windows(self):
        """Header word 0 of the tables and the fill levels [units, L, windows, 2^K] behind the indices."""
        units, L, nb = self.B * self.Hkv, self.L, 1 << self.K
        raw = self.tables.cpu().numpy().view(np.uint32)
        windows = int(raw[0])
        start = 256 // 4 + (units * L * (nb + 1) * 4 + 255) // 256 * 256 // 4 + (units * L * self.n_cap * 4 + 255) // 256 * 256 // 4
        return windows, raw[start:start + units * L * max(windows, 0) * nb].reshape(units, L, max(windows, 0), nb)

    def attend(self, debug=True, cand_cap=None, tables=False, with_counts=True):
        B, Hq, n = self.B, self.Hq, self.n
        out = torch.full((B, Hq, 128), float("nan"), dtype=torch.float32, device="cuda")
        if debug:
            cap = max(n, 1) if cand_cap is None else cand_cap
            counts = torch.full((B, Hq, max(n, 1)), -1 if not tables else 0, dtype=torch.int16, device="cuda")
            cand = torch.full((B, Hq, cap), -1, dtype=torch.int32, device="cuda")
            ncand = torch.zeros((B, Hq), dtype=torch.int32, device="cuda")
            if not with_counts:
                counts = None
        else:
            counts = cand = ncand = None
        if tables:
            mp.magicpig_sampled_attention_tables(self.params, self.q, self.Kc, self.Vc, self.mu, self.tables,
                                                 self.n_indexed, self.key_codes, self.q_codes, out, counts, cand,
                                                 ncand, self.ws)
        else:
            mp.magicpig_sampled_attention(self.params, self.q, self.Kc, self.Vc, self.mu, self.key_codes,
                                          self.q_codes, out, counts, cand, ncand, self.ws)
        torch.cuda.synchronize()
        res = {"out": out.cpu().numpy()}
        if debug:
            if counts is not None:
                res["counts"] = counts.cpu().numpy()[:, :, :n].astype(np.int32)
            nc = ncand.cpu().numpy()
            cd = cand.cpu().numpy()
            res["ncand"] = nc
            res["S"] = [[np.sort(cd[b, h, : min(nc[b, h], cd.shape[-1])]) for h in range(Hq)] for b in range(B)]
        return res


def rel_err(out: np.ndarray, ref: np.ndarray) -> float:
    """Per head: max_j |o_j - ref_j| / max_j |ref_j|; returns the worst head."""
    out = np.asarray(out, np.float64).reshape(-1, out.shape[-1])
    ref = np.asarray(ref, np.float64).reshape(-1, ref.shape[-1])
    scale = np.maximum(np.abs(ref).max(axis=1), 1e-30)
    return float((np.abs(out - ref).max(axis=1) / scale).max())
