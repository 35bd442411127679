"""Thin ctypes binding of libmagicpig.so: argument marshalling only.

Every function has the name and argument order of its C entry point (include/magicpig.h)
and takes torch tensors where the C call takes device pointers.  Work is enqueued on
torch's current HIP stream.  There is no fallback: if the library is missing, loading
raises; if a call returns a negative status, MagicpigError is raised.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
# (MAGICPIG_LIB names another build of the library, e.g. one compiled with other options)
LIB_PATH = os.environ.get("MAGICPIG_LIB") or os.path.join(_PKG, "libmagicpig.so")

MAGICPIG_BF16, MAGICPIG_FP32 = 0, 1
MAGICPIG_KV_SAME, MAGICPIG_KV_FP8_E4M3 = 0, 1


class MagicpigError(RuntimeError):
    pass


class magicpig_params(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("K", ctypes.c_int32), ("L", ctypes.c_int32),
        ("min_hits", ctypes.c_int32), ("n_sink", ctypes.c_int32), ("n_local", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("n_ctx", ctypes.c_int64), ("n_cap", ctypes.c_int64),
        ("k_stride_b", ctypes.c_int64), ("k_stride_h", ctypes.c_int64), ("k_stride_n", ctypes.c_int64),
        ("v_stride_b", ctypes.c_int64), ("v_stride_h", ctypes.c_int64), ("v_stride_n", ctypes.c_int64),
        ("n_ctx_dev", ctypes.c_void_p),
        ("kv_dtype", ctypes.c_int32),
    ]


EXPORTS = (
    "magicpig_code_words_per_key", "magicpig_code_words_per_query", "magicpig_key_code_bytes",
    "magicpig_query_code_bytes",
    "magicpig_key_code_index", "magicpig_workspace_bytes", "magicpig_key_mean",
    "magicpig_hash_keys", "magicpig_hash_query", "magicpig_sampled_attention",
    "magicpig_status_string", "magicpig_last_hip_error", "magicpig_profile_stage_events",
    "magicpig_hash_keys_stats_offset", "magicpig_table_bytes", "magicpig_build_tables",
    "magicpig_sampled_attention_tables", "magicpig_hash_decode_step", "magicpig_table_build_workspace_bytes",
    "magicpig_sampled_attention_noalloc",
    "magicpig_prepared_projector_bytes", "magicpig_prepare_projector", "magicpig_centering_bytes",
    "magicpig_prepare_centering", "magicpig_hash_query_prepared", "magicpig_hash_decode_step_prepared",
)

_lib = None


def lib() -> ctypes.CDLL:
    """Loads libmagicpig.so (built in-tree by paper_2410_16179_amd.build); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise MagicpigError(f"{LIB_PATH} is not built; run `python -m paper_2410_16179_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER(magicpig_params)
    vp, sz, i32, i64 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int64
    for name in ("magicpig_code_words_per_key", "magicpig_code_words_per_query", "magicpig_key_code_bytes",
                 "magicpig_query_code_bytes", "magicpig_workspace_bytes",
                 "magicpig_hash_keys_stats_offset", "magicpig_table_bytes", "magicpig_table_build_workspace_bytes",
                 "magicpig_prepared_projector_bytes", "magicpig_centering_bytes"):
        getattr(L, name).restype, getattr(L, name).argtypes = sz, [P]
    L.magicpig_key_code_index.restype = sz
    L.magicpig_key_code_index.argtypes = [P, i32, i32, i64, i32]
    L.magicpig_key_mean.restype = ctypes.c_int
    L.magicpig_key_mean.argtypes = [P, vp, vp, vp, sz, vp]
    L.magicpig_hash_keys.restype = ctypes.c_int
    L.magicpig_hash_keys.argtypes = [P, vp, vp, vp, i64, i64, vp, vp, sz, vp]
    L.magicpig_hash_query.restype = ctypes.c_int
    L.magicpig_hash_query.argtypes = [P, vp, vp, vp, vp, sz, vp]
    L.magicpig_hash_decode_step.restype = ctypes.c_int
    L.magicpig_hash_decode_step.argtypes = [P, vp, vp, vp, vp, i64, i64, vp, vp, vp, sz, vp]
    L.magicpig_sampled_attention.restype = ctypes.c_int
    L.magicpig_sampled_attention.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, vp, sz, vp]
    L.magicpig_sampled_attention_noalloc.restype = ctypes.c_int
    L.magicpig_sampled_attention_noalloc.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp]
    L.magicpig_prepare_projector.restype = ctypes.c_int
    L.magicpig_prepare_projector.argtypes = [P, vp, vp, vp]
    L.magicpig_prepare_centering.restype = ctypes.c_int
    L.magicpig_prepare_centering.argtypes = [P, vp, vp, vp, vp]
    L.magicpig_hash_query_prepared.restype = ctypes.c_int
    L.magicpig_hash_query_prepared.argtypes = [P, vp, vp, vp, vp]
    L.magicpig_hash_decode_step_prepared.restype = ctypes.c_int
    L.magicpig_hash_decode_step_prepared.argtypes = [P, vp, vp, vp, vp, vp, i64, i64, vp, vp, vp]
    L.magicpig_build_tables.restype = ctypes.c_int
    L.magicpig_build_tables.argtypes = [P, vp, vp, vp, sz, vp]
    L.magicpig_sampled_attention_tables.restype = ctypes.c_int
    L.magicpig_sampled_attention_tables.argtypes = [P, vp, vp, vp, vp, vp, i64, vp, vp, vp, vp, vp, vp, i64, vp, sz, vp]
    L.magicpig_status_string.restype, L.magicpig_status_string.argtypes = ctypes.c_char_p, [ctypes.c_int]
    L.magicpig_last_hip_error.restype, L.magicpig_last_hip_error.argtypes = ctypes.c_char_p, []
    L.magicpig_profile_stage_events.restype = None
    L.magicpig_profile_stage_events.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    _lib = L
    return L


def _check(status: int) -> None:
    if status != 0:
        msg = lib().magicpig_status_string(status).decode()
        if status == -4:
            msg += ": " + lib().magicpig_last_hip_error().decode()
        raise MagicpigError(f"magicpig status {status}: {msg}")


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def make_params(*, batch, n_q_heads, n_kv_heads, K, L, n_ctx, dtype, n_cap=None, min_hits=2,
                n_sink=4, n_local=64, head_dim=128, k_strides=None, v_strides=None,
                n_ctx_dev=None, kv_dtype=0) -> magicpig_params:
    """Parameter block; strides default to a contiguous [batch, n_kv_heads, n_cap, 128] cache.
    n_ctx_dev: an int64 device tensor holding the live context length, or None.
    kv_dtype: 0 (caches hold `dtype`), 1 or "fp8" (caches hold OCP e4m3 bytes)."""
    kv_dtype = {"fp8": MAGICPIG_KV_FP8_E4M3, "": 0, None: 0}.get(kv_dtype, kv_dtype)
    n_cap = n_ctx if n_cap is None else n_cap
    dense = (n_kv_heads * n_cap * head_dim, n_cap * head_dim, head_dim)
    ks = dense if k_strides is None else tuple(k_strides)
    vs = dense if v_strides is None else tuple(v_strides)
    code = {"bf16": MAGICPIG_BF16, "fp32": MAGICPIG_FP32, torch.bfloat16: MAGICPIG_BF16,
            torch.float32: MAGICPIG_FP32}.get(dtype, dtype)
    return magicpig_params(batch, n_q_heads, n_kv_heads, head_dim, K, L, min_hits, n_sink, n_local,
                           code, n_ctx, n_cap, ks[0], ks[1], ks[2], vs[0], vs[1], vs[2],
                           None if n_ctx_dev is None else n_ctx_dev.data_ptr(), kv_dtype)


def magicpig_code_words_per_key(params) -> int:
    return lib().magicpig_code_words_per_key(ctypes.byref(params))


def magicpig_code_words_per_query(params) -> int:
    return lib().magicpig_code_words_per_query(ctypes.byref(params))


def magicpig_key_code_bytes(params) -> int:
    return lib().magicpig_key_code_bytes(ctypes.byref(params))


def magicpig_query_code_bytes(params) -> int:
    return lib().magicpig_query_code_bytes(ctypes.byref(params))


def magicpig_workspace_bytes(params) -> int:
    return lib().magicpig_workspace_bytes(ctypes.byref(params))


def magicpig_hash_keys_stats_offset(params) -> int:
    return lib().magicpig_hash_keys_stats_offset(ctypes.byref(params))


def hash_keys_stats(params, workspace) -> dict:
    """Reads the statistics a bf16 magicpig_hash_keys call left in its workspace (synchronises)."""
    off = magicpig_hash_keys_stats_offset(params)
    raw = workspace[off:off + 16].cpu().numpy().view(np.uint32)
    return {"w_max_norm": float(raw[:1].view(np.float32)[0]), "spilled": int(raw[1]),
            "overflowed": bool(raw[2]), "rechecked": int(raw[3])}


def magicpig_key_code_index(params, b, g, key, word) -> int:
    return lib().magicpig_key_code_index(ctypes.byref(params), b, g, key, word)


def magicpig_key_mean(params, K_cache, mu_out, workspace) -> None:
    _check(lib().magicpig_key_mean(ctypes.byref(params), _ptr(K_cache), _ptr(mu_out), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream()))


def magicpig_hash_keys(params, K_cache, mu, W, first_key, n_keys, key_codes, workspace) -> None:
    _check(lib().magicpig_hash_keys(ctypes.byref(params), _ptr(K_cache), _ptr(mu), _ptr(W), first_key,
                                    n_keys, _ptr(key_codes), _ptr(workspace),
                                    workspace.numel() * workspace.element_size(), _stream()))


def magicpig_hash_query(params, q, W, q_codes, workspace=None) -> None:
    _check(lib().magicpig_hash_query(ctypes.byref(params), _ptr(q), _ptr(W), _ptr(q_codes),
                                     _ptr(workspace), _nbytes(workspace), _stream()))


def magicpig_hash_decode_step(params, q, K_cache, mu, W, first_key, n_keys, key_codes, q_codes, workspace=None) -> None:
    _check(lib().magicpig_hash_decode_step(ctypes.byref(params), _ptr(q), _ptr(K_cache), _ptr(mu), _ptr(W),
                                           first_key, n_keys, _ptr(key_codes), _ptr(q_codes), _ptr(workspace),
                                           _nbytes(workspace), _stream()))


def magicpig_prepared_projector_bytes(params) -> int:
    return lib().magicpig_prepared_projector_bytes(ctypes.byref(params))


def magicpig_centering_bytes(params) -> int:
    return lib().magicpig_centering_bytes(ctypes.byref(params))


def magicpig_prepare_projector(params, W, prepared) -> None:
    _check(lib().magicpig_prepare_projector(ctypes.byref(params), _ptr(W), _ptr(prepared), _stream()))


def magicpig_prepare_centering(params, mu, prepared, centering) -> None:
    _check(lib().magicpig_prepare_centering(ctypes.byref(params), _ptr(mu), _ptr(prepared), _ptr(centering), _stream()))


def magicpig_hash_query_prepared(params, q, prepared, q_codes) -> None:
    _check(lib().magicpig_hash_query_prepared(ctypes.byref(params), _ptr(q), _ptr(prepared), _ptr(q_codes), _stream()))


def magicpig_hash_decode_step_prepared(params, q, K_cache, mu, centering, prepared, first_key, n_keys, key_codes,
                                       q_codes) -> None:
    _check(lib().magicpig_hash_decode_step_prepared(ctypes.byref(params), _ptr(q), _ptr(K_cache), _ptr(mu),
                                                    _ptr(centering), _ptr(prepared), first_key, n_keys,
                                                    _ptr(key_codes), _ptr(q_codes), _stream()))


def magicpig_sampled_attention(params, q, K_cache, V_cache, mu, key_codes, q_codes, out,
                               dbg_counts=None, dbg_cand=None, dbg_ncand=None, workspace=None) -> None:
    cap = 0 if dbg_cand is None else dbg_cand.shape[-1]
    _check(lib().magicpig_sampled_attention(
        ctypes.byref(params), _ptr(q), _ptr(K_cache), _ptr(V_cache), _ptr(mu), _ptr(key_codes),
        _ptr(q_codes), _ptr(out), _ptr(dbg_counts), _ptr(dbg_cand), _ptr(dbg_ncand), cap,
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def magicpig_sampled_attention_noalloc(params, q, K_cache, V_cache, mu, key_codes, q_codes, out) -> None:
    _check(lib().magicpig_sampled_attention_noalloc(
        ctypes.byref(params), _ptr(q), _ptr(K_cache), _ptr(V_cache), _ptr(mu), _ptr(key_codes),
        _ptr(q_codes), _ptr(out), _stream()))


def magicpig_table_bytes(params) -> int:
    return lib().magicpig_table_bytes(ctypes.byref(params))


def magicpig_build_tables(params, key_codes, tables, workspace=None) -> None:
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().magicpig_build_tables(ctypes.byref(params), _ptr(key_codes), _ptr(tables), _ptr(workspace),
                                       nbytes, _stream()))


def magicpig_sampled_attention_tables(params, q, K_cache, V_cache, mu, tables, n_indexed, key_codes, q_codes,
                                      out, dbg_counts=None, dbg_cand=None, dbg_ncand=None, workspace=None) -> None:
    cap = 0 if dbg_cand is None else dbg_cand.shape[-1]
    _check(lib().magicpig_sampled_attention_tables(
        ctypes.byref(params), _ptr(q), _ptr(K_cache), _ptr(V_cache), _ptr(mu), _ptr(tables),
        int(n_indexed), _ptr(key_codes), _ptr(q_codes), _ptr(out), _ptr(dbg_counts), _ptr(dbg_cand), _ptr(dbg_ncand), cap,
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def magicpig_profile_stage_events(events) -> None:
    """events: None, or seven hipEvent_t handles (ints) attached to the decode kernels."""
    if events is None:
        lib().magicpig_profile_stage_events(None)
    else:
        assert len(events) == 7
        arr = (ctypes.c_void_p * 7)(*events)
        lib().magicpig_profile_stage_events(arr)


# ---- buffer helpers (allocation and layout only) ---------------------------------------------
def alloc_key_codes(params, device="cuda") -> torch.Tensor:
    return torch.zeros(max(magicpig_key_code_bytes(params) // 4, 4), dtype=torch.int32, device=device)


def alloc_query_codes(params, device="cuda") -> torch.Tensor:
    return torch.zeros(max(magicpig_query_code_bytes(params) // 4, 4), dtype=torch.int32, device=device)


def alloc_tables(params, device="cuda") -> torch.Tensor:
    nbytes = magicpig_table_bytes(params)
    if nbytes == 0:
        raise MagicpigError("hash tables are not supported for these parameters")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def magicpig_table_build_workspace_bytes(params) -> int:
    return lib().magicpig_table_build_workspace_bytes(ctypes.byref(params))


def alloc_table_build_workspace(params, device="cuda") -> torch.Tensor:
    return torch.empty(max(magicpig_table_build_workspace_bytes(params), 256), dtype=torch.uint8, device=device)


def alloc_prepared_projector(params, device="cuda") -> torch.Tensor:
    return torch.empty(max(magicpig_prepared_projector_bytes(params), 256), dtype=torch.uint8, device=device)


def alloc_centering(params, device="cuda") -> torch.Tensor:
    return torch.empty(max(magicpig_centering_bytes(params), 256), dtype=torch.uint8, device=device)


def alloc_workspace(params, device="cuda") -> torch.Tensor:
    return torch.empty(max(magicpig_workspace_bytes(params), 256), dtype=torch.uint8, device=device)


def key_code_gather_index(params) -> np.ndarray:
    """u32 index of every (b, g, key < n_cap, word) in the key-code buffer, built from
    magicpig_key_code_index on one block and the block stride it implies."""
    NW = magicpig_code_words_per_key(params)
    n_cap = params.n_cap
    slot = np.array([[magicpig_key_code_index(params, 0, 0, r, x) for x in range(NW)]
                     for r in range(min(64, n_cap))], dtype=np.int64)
    nblk = (n_cap + 63) // 64
    keys = np.arange(n_cap)
    per_unit = (keys // 64)[:, None] * (64 * NW) + slot[keys % 64]          # [n_cap, NW]
    units = np.arange(params.batch * params.n_kv_heads, dtype=np.int64) * (nblk * 64 * NW)
    idx = units[:, None, None] + per_unit[None]
    return idx.reshape(params.batch, params.n_kv_heads, n_cap, NW)


def key_plane_words(words: np.ndarray, K: int, L: int) -> np.ndarray:
    """[..., NW] words of key codes -> [..., K*ceil(L/32)] plane words: the last table group,
    stored as one bit string of K planes, is spread out again (tables >= L read 0)."""
    words = np.asarray(words).astype(np.uint32)
    Wd = (L + 31) // 32
    Lt, xs = L - 32 * (Wd - 1), K * (Wd - 1)
    out = np.zeros(words.shape[:-1] + (K * Wd,), np.uint32)
    out[..., :xs] = words[..., :xs]
    tail = words[..., xs:].astype(np.uint64)
    for b in range(K):
        pos = b * Lt
        wi, sh = pos // 32, pos % 32
        v = tail[..., wi] >> np.uint64(sh)
        if sh + Lt > 32:
            v = v | (tail[..., wi + 1] << np.uint64(32 - sh))
        out[..., xs + b] = (v & np.uint64((1 << Lt) - 1)).astype(np.uint32)
    return out


def key_words_from_planes(planes: np.ndarray, K: int, L: int) -> np.ndarray:
    """Inverse of key_plane_words: [..., K*ceil(L/32)] plane words -> [..., NW] key-code words."""
    planes = np.asarray(planes).astype(np.uint32)
    Wd = (L + 31) // 32
    Lt, xs = L - 32 * (Wd - 1), K * (Wd - 1)
    nt = (K * Lt + 31) // 32
    out = np.zeros(planes.shape[:-1] + (xs + nt,), np.uint32)
    out[..., :xs] = planes[..., :xs]
    acc = np.zeros(planes.shape[:-1] + (nt + 1,), np.uint64)
    for b in range(K):
        pos = b * Lt
        wi, sh = pos // 32, pos % 32
        v = (planes[..., xs + b].astype(np.uint64) & np.uint64((1 << Lt) - 1)) << np.uint64(sh)
        acc[..., wi] |= v & np.uint64(0xffffffff)
        acc[..., wi + 1] |= v >> np.uint64(32)
    out[..., xs:] = acc[..., :nt].astype(np.uint32)
    return out


def table_codes_from_words(words: np.ndarray, K: int, L: int) -> np.ndarray:
    """[..., K*ceil(L/32)] plane words (word w*K+b, bit beta <-> table 32w+beta) -> [..., L]
    integers sum_b bit_b 2^b, the canonical per-table form."""
    words = np.asarray(words).astype(np.uint32)
    Wd = (L + 31) // 32
    w = words.reshape(*words.shape[:-1], Wd, K)
    beta = np.arange(32, dtype=np.uint32)
    bits = (w[..., None] >> beta) & np.uint32(1)                 # [..., Wd, K, 32]
    weights = (np.uint32(1) << np.arange(K, dtype=np.uint32))[:, None]
    codes = (bits * weights).sum(axis=-2)                        # [..., Wd, 32]
    return codes.reshape(*words.shape[:-1], Wd * 32)[..., :L].astype(np.int32)
