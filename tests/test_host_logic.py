"""Host-side checks that need no GPU: the library loads and exports what the header
declares, argument validation, sizes and the packed-code layout."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2410_16179_amd import binding as mp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def params(**kw):
    base = dict(batch=1, n_q_heads=32, n_kv_heads=8, K=10, L=150, n_ctx=1000, dtype="bf16")
    base.update(kw)
    return mp.make_params(**base)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "magicpig.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(magicpig_[a-z_]+)\s*\(", header))
    assert declared == set(mp.EXPORTS)
    lib = mp.lib()
    for name in declared:
        assert hasattr(lib, name), name


def test_library_exports_nothing_but_the_declared_symbols():
    # the dynamic symbol table of the built library: every function it defines and exports is an
    # entry point of the header (kernels' host stubs, launch helpers and the rest stay hidden)
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", mp.LIB_PATH], check=True, capture_output=True, text=True).stdout
    exported = {line.split()[-1] for line in out.splitlines() if line.split()[-2] in ("T", "t", "W", "w")}
    # (code-object bookkeeping the HIP toolchain emits itself is not the library's interface)
    exported = {name for name in exported if not name.startswith(("__hip_", "_init", "_fini"))}
    assert exported == set(mp.EXPORTS), sorted(exported ^ set(mp.EXPORTS))


def test_struct_layout_matches_header():
    assert ctypes.sizeof(mp.magicpig_params) == 10 * 4 + 8 * 8 + 8 + 8       # (kv_dtype and padding)
    assert mp.magicpig_params.n_ctx_dev.offset == 10 * 4 + 8 * 8
    assert mp.magicpig_params.kv_dtype.offset == 10 * 4 + 8 * 8 + 8


def test_sizes_and_paper_projector_size():
    p = params()
    # 1500 sign bits: 4 complete groups of 32 tables (40 plane words) + 10 planes x 22 tables = 220 bits
    assert mp.magicpig_code_words_per_key(p) == 40 + 7
    assert mp.magicpig_code_words_per_query(p) == 10 * 5
    assert mp.magicpig_query_code_bytes(p) == 32 * 50 * 4
    assert mp.magicpig_key_code_bytes(p) == 8 * 1024 * 47 * 4     # capacity rounded to 64 keys
    assert mp.magicpig_code_words_per_key(params(K=9, L=120)) == 27 + 7
    assert mp.magicpig_code_words_per_key(params(K=10, L=170)) == 50 + 4
    assert mp.magicpig_code_words_per_key(params(K=8, L=75)) == 16 + 3
    assert mp.magicpig_code_words_per_key(params(K=6, L=64)) == 12     # whole groups: nothing to pack
    assert mp.magicpig_workspace_bytes(p) >= 256
    # hash tables: header, offsets [units][L][2^K + 1], indices [units][L][n_cap], fill levels
    # [units][L][windows of 16384 keys][2^K], each part rounded up to 256 bytes
    up = lambda x: (x + 255) // 256 * 256
    units, nb = p.batch * p.n_kv_heads, 1 << p.K
    for n_cap in (1000, 16384, 16385, 40000):
        pt = params(n_ctx=min(1000, n_cap), n_cap=n_cap)
        windows = (n_cap + 16383) // 16384
        assert mp.magicpig_table_bytes(pt) == (256 + up(units * p.L * (nb + 1) * 4) + up(units * p.L * n_cap * 4)
                                               + up(units * p.L * windows * nb * 4))
        assert mp.magicpig_table_build_workspace_bytes(pt) == up(units * p.L * ((n_cap + 63) // 64 * 64) * 2)
    assert mp.magicpig_table_bytes(params(K=13)) == 0               # unsupported: no tables
    # Table "overhead of LSH": the (10,150) projector for d = 128 in bf16 is 384 KB
    assert 128 * p.K * p.L * 2 == 384000


@pytest.mark.parametrize("K,L,n_cap", [(10, 150, 200), (9, 120, 64), (8, 75, 130), (3, 33, 65), (1, 1, 1), (7, 65, 100)])
def test_code_layout_is_a_bijection_inside_the_buffer(K, L, n_cap):
    p = params(batch=2, n_q_heads=4, n_kv_heads=2, K=K, L=L, n_ctx=n_cap, n_cap=n_cap)
    idx = mp.key_code_gather_index(p)
    NW = mp.magicpig_code_words_per_key(p)
    assert idx.shape == (2, 2, n_cap, NW)
    flat = idx.ravel()
    assert len(np.unique(flat)) == flat.size
    assert flat.min() >= 0 and flat.max() < mp.magicpig_key_code_bytes(p) // 4
    rng = np.random.default_rng(0)
    for _ in range(50):      # the vectorised index agrees with the C function everywhere
        b, g, k, x = rng.integers(2), rng.integers(2), rng.integers(n_cap), rng.integers(NW)
        assert idx[b, g, k, x] == mp.magicpig_key_code_index(p, int(b), int(g), int(k), int(x))
    assert mp.magicpig_key_code_index(p, 0, 0, n_cap, 0) == ctypes.c_size_t(-1).value
    assert mp.magicpig_key_code_index(p, 0, 0, 0, NW) == ctypes.c_size_t(-1).value


@pytest.mark.parametrize("K,L", [(10, 150), (9, 120), (10, 170), (8, 75), (5, 70), (16, 33), (3, 64), (1, 1)])
def test_key_words_pack_and_unpack(K, L):
    rng = np.random.default_rng(2)
    Wd = (L + 31) // 32
    Lt = L - 32 * (Wd - 1)
    planes = rng.integers(0, 2 ** 32, size=(5, 3, K * Wd), dtype=np.uint64).astype(np.uint32)
    planes[..., K * (Wd - 1):] &= np.uint32((1 << Lt) - 1)       # tables >= L are 0 in key codes
    words = mp.key_words_from_planes(planes, K, L)
    assert words.shape[-1] == mp.magicpig_code_words_per_key(params(K=K, L=L))
    np.testing.assert_array_equal(mp.key_plane_words(words, K, L), planes)
    # bit b*Lt + beta of the tail string is bit b of table 32*(Wd-1) + beta
    xs = K * (Wd - 1)
    for b in range(K):
        for beta in (0, Lt - 1):
            pos = b * Lt + beta
            got = (words[..., xs + pos // 32] >> np.uint32(pos % 32)) & np.uint32(1)
            np.testing.assert_array_equal(got, (planes[..., xs + b] >> np.uint32(beta)) & np.uint32(1))


def test_table_codes_from_words_roundtrip():
    rng = np.random.default_rng(1)
    K, L = 5, 70
    Wd = 3
    bits = rng.integers(0, 2, size=(4, L, K))
    words = np.zeros((4, Wd * K), np.uint32)
    for t in range(L):
        for b in range(K):
            words[:, (t // 32) * K + b] |= (bits[:, t, b].astype(np.uint32) << np.uint32(t % 32))
    codes = mp.table_codes_from_words(words, K, L)
    expect = (bits * (1 << np.arange(K))).sum(axis=2)
    np.testing.assert_array_equal(codes, expect)


def _status(fn, *args):
    return fn(*args)


def test_argument_validation_without_a_gpu():
    lib = mp.lib()
    ws = (ctypes.c_char * 4096)()
    wsp = ctypes.addressof(ws)
    wsp += (-wsp) % 16
    fake = ctypes.c_void_p(wsp)
    big = 1 << 40

    def hash_query(p, q=fake, W=fake, codes=fake, wbytes=big):
        return lib.magicpig_hash_query(ctypes.byref(p), q, W, codes, fake, wbytes, None)

    assert hash_query(params(head_dim=64)) == -2
    assert hash_query(params(K=0)) == -2
    assert hash_query(params(K=17)) == -2
    assert hash_query(params(L=513)) == -2
    assert hash_query(params(dtype=7)) == -2
    assert hash_query(params(kv_dtype=5)) == -2
    assert hash_query(params(dtype="fp32", kv_dtype="fp8")) == -2   # e4m3 caches go with bf16 queries and projector
    assert hash_query(params(n_q_heads=6, n_kv_heads=4)) == -1
    assert hash_query(params(n_q_heads=24, n_kv_heads=8, batch=0)) == 0   # group size 3 is fine (batch 0: nothing to launch)
    assert hash_query(params(n_q_heads=72, n_kv_heads=8)) == -2      # group size 9
    assert hash_query(params(batch=4097, n_q_heads=32, n_kv_heads=8)) == -2   # more query vectors than one launch takes
    assert hash_query(params(n_ctx=100, n_cap=50)) == -1
    assert hash_query(params(n_local=(1 << 30) + 1)) == -1           # static-set sizes beyond 2^30
    assert hash_query(params(n_sink=-1)) == -1
    assert hash_query(params(), W=None) == -1
    assert hash_query(params(), q=ctypes.c_void_p(wsp + 2)) == -1     # misaligned
    p = params()
    many = 200                                                    # 8 KV heads x 200 keys: the matrix-core path, which needs scratch
    assert lib.magicpig_hash_keys(ctypes.byref(p), fake, None, fake, 0, many, fake, fake, 8, None) == -3
    assert lib.magicpig_hash_keys(ctypes.byref(p), fake, None, fake, 0, many, fake, None, 0, None) == -3
    assert lib.magicpig_hash_keys(ctypes.byref(p), fake, None, fake, 900, 200, fake, fake, big, None) == -1
    assert lib.magicpig_hash_keys(ctypes.byref(p), fake, None, fake, -1, 2, fake, fake, big, None) == -1
    bad = params(k_strides=(8 * 1000 * 128, 1000 * 128, 100))
    assert lib.magicpig_hash_keys(ctypes.byref(bad), fake, None, fake, 0, 1, fake, fake, big, None) == -1
    bad = params(k_strides=(8 * 1000 * 132, 1000 * 132, 132))
    assert lib.magicpig_hash_keys(ctypes.byref(bad), fake, None, fake, 0, 1, fake, fake, big, None) == -2
    assert lib.magicpig_sampled_attention(ctypes.byref(p), fake, fake, fake, None, fake, fake, None,
                                          None, None, None, 0, fake, big, None) == -1
    assert lib.magicpig_sampled_attention(ctypes.byref(p), fake, fake, fake, None, fake, fake, fake,
                                          None, fake, None, 4, fake, big, None) == -1
    assert lib.magicpig_sampled_attention(ctypes.byref(p), fake, fake, fake, None, fake, fake, fake,
                                          None, None, None, 0, fake, 16, None) == -3
    assert lib.magicpig_key_mean(ctypes.byref(p), fake, None, fake, big, None) == -1

    def decode_hash(pp, q=fake, first=0, count=1, kcodes=fake, qcodes=fake, wbytes=big):
        return lib.magicpig_hash_decode_step(ctypes.byref(pp), q, fake, None, fake, first, count, kcodes,
                                             qcodes, fake, wbytes, None)

    assert decode_hash(p, first=1000, count=1) == -1               # beyond the capacity
    assert decode_hash(p, qcodes=None) == -1
    assert decode_hash(p, kcodes=None) == -1
    assert decode_hash(p, q=None) == -1
    assert decode_hash(p, count=many, wbytes=8) == -3
    assert decode_hash(params(K=17)) == -2

    def attend_tables(pp, n_indexed, codes=fake, tables=fake):
        return lib.magicpig_sampled_attention_tables(ctypes.byref(pp), fake, fake, fake, None, tables, n_indexed,
                                                     codes, fake, fake, None, None, None, 0, fake, 16, None)

    n = p.n_ctx
    assert attend_tables(p, n - n % 64 - 64) == -3               # valid arguments get as far as the workspace check
    assert attend_tables(p, n) == -3
    assert attend_tables(p, n, codes=None) == -3                 # nothing behind the tables: no codes needed
    assert attend_tables(p, 0, codes=None) == -1                 # everything behind the tables: codes needed
    assert attend_tables(p, n + 64) == -1
    assert attend_tables(p, -64) == -1
    assert attend_tables(p, 100) == -1                           # neither everything nor whole blocks
    assert attend_tables(p, n, tables=None) == -1
    assert attend_tables(params(K=13), 64) == -2                 # tables unsupported beyond K = 12
    assert mp.magicpig_workspace_bytes(params(K=0)) == 0

    def attend_noalloc(pp, q=fake, out=fake, codes=fake):
        return lib.magicpig_sampled_attention_noalloc(ctypes.byref(pp), q, fake, fake, None, codes, fake, out, None)

    assert attend_noalloc(p, out=None) == -1
    assert attend_noalloc(p, codes=None) == -1
    assert attend_noalloc(params(K=17)) == -2
    # batch 8 x 64 heads at 131072 keys needs 35 MB of partial results: beyond the static array
    assert attend_noalloc(params(batch=8, n_q_heads=64, n_kv_heads=8, K=10, L=170, n_ctx=131072)) == -5
    assert b"static" in lib.magicpig_status_string(-5)
    assert lib.magicpig_status_string(-3) == b"workspace too small"
    assert lib.magicpig_status_string(0) == b"ok"


def test_header_is_plain_c_and_links_from_c(tmp_path):
    # the boundary is a C ABI: a C99 program includes the header (pedantic, warnings are errors),
    # links against the shared library and calls it without a GPU
    import subprocess
    exe = str(tmp_path / "use_from_c")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "c_abi", "use_from_c.c"), "-o", exe, mp.LIB_PATH,
                    "-Wl,-rpath," + os.path.dirname(mp.LIB_PATH)], check=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout.split()
    assert out[0] == "47" and int(out[1]) == mp.magicpig_workspace_bytes(params()) and "unsupported" in " ".join(out[2:])


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(mp, "_lib", None)
    monkeypatch.setattr(mp, "LIB_PATH", "/nonexistent/libmagicpig.so")
    with pytest.raises(mp.MagicpigError):
        mp.lib()
