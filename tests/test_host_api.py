"""Host-side checks that need no GPU: the C-ABI library loads, exports every declared symbol,
answers its closed-form size queries and rejects bad arguments before touching the GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest
import torch

import paper_2310_15929_amd as esp
from paper_2310_15929_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = esp.load_library()
    header = open(os.path.join(ROOT, "include", "esparse.h")).read()
    declared = set(re.findall(r"\b(esparse_[a-z_]+)\s*\(", header))
    declared -= {"esparse_ctx", "esparse_status", "esparse_dtype", "esparse_prune_opts"}
    assert declared == set(binding.EXPORTED)
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.esparse_version().startswith(b"esparse")


def test_size_queries_closed_form():
    for N, K in [(512, 512), (4096, 11008), (24, 320)]:
        vb, mb, nb = esp.compressed_size(N, K, 2, 4)
        assert vb == N * K and mb == N * ((K // 2 + 15) // 16) * 4
        Np, Kp = -(-N // 16) * 16, -(-K // 256) * 256
        assert nb == Np * Kp * 9 // 8
        vb8, mb8, nb8 = esp.compressed_size(N, K - K % 8, 4, 8)
        Kp8 = -(-(K - K % 8) // 256) * 256
        assert vb8 == N * (K - K % 8) and mb8 == N * (K - K % 8) // 8 and nb8 == Np * Kp8 * 9 // 8
    vb, mb, _ = esp.compressed_size(4096, 4096, 2, 4)
    assert (vb + mb) / (2 * 4096 * 4096) == 0.5625
    assert esp.dense_packed_size(24, 320) == 32 * 512 * 2
    assert esp.spmm_workspace(16, 512, 512) >= 16 * 512 * 2
    # the size for a named variant never exceeds the size that serves every variant, covers the staged activations,
    # and only variants that split K over workgroups ask for fp32 partial tiles
    for M, N, K in [(1, 4096, 4096), (33, 80, 2048), (128, 22016, 8192), (2048, 13824, 5120)]:
        every = esp.spmm_workspace(M, N, K)
        assert every == esp.spmm_workspace(M, N, K, -1)
        Mp = -(-M // 16) * 16
        for v in range(esp.num_variants()):
            one = esp.spmm_workspace(M, N, K, v)
            assert Mp * K * 2 <= one <= every, esp.variant_name(v)
            splits = "splitk" in esp.variant_name(v) or "stream" in esp.variant_name(v) or "_k" in esp.variant_name(v)
            if not splits:
                assert one < Mp * K * 2 * 2 + 4096, esp.variant_name(v)
    with pytest.raises(esp.EsparseError):
        esp.spmm_workspace(16, 512, 512, esp.num_variants())
    with pytest.raises(esp.EsparseError):
        esp.compressed_size(8, 8, 1, 4)


def test_argument_errors_need_no_gpu():
    ctx = esp.Context(0)
    W = torch.zeros(8, 16, dtype=torch.float16)
    Xc = torch.zeros(4, 16, dtype=torch.float16)

    def code(fn):
        with pytest.raises(esp.EsparseError) as e:
            fn()
        return e.value.code

    assert code(lambda: ctx.compress(W, None, None, 3, 4)) == -2
    assert code(lambda: ctx.compress(torch.zeros(8, 18, dtype=torch.float16), None, None, 2, 4)) == -1
    assert code(lambda: ctx.prune(Xc, W, esp.PruneOpts(block=24))) == -1          # 16 % 24
    assert code(lambda: ctx.prune(Xc, W, esp.PruneOpts(block=6))) == -1           # block % m
    assert code(lambda: ctx.prune(Xc, W, esp.PruneOpts(n_keep=1, m_group=4, block=8))) == -2
    assert code(lambda: ctx.prune(Xc, W, esp.PruneOpts(block=8, bins=0))) == -1
    assert code(lambda: ctx.prune(Xc, W, esp.PruneOpts(block=8, flags=esp.USE_GNS))) == -1
    assert code(lambda: ctx.prune(Xc, W, esp.PruneOpts(block=8, max_swaps=-1))) == -1
    lib = esp.load_library()
    assert lib.esparse_spmm(ctx._h, None, 4, None, None, 8, 16, 0, 1, 4, None, None, 0, -1) == -2   # no 1:4 product
    assert lib.esparse_spmm(ctx._h, None, 4, None, None, 8, 16, 0, 4, 8, None, None, 0, -1) == -1   # 4:8: null pointers
    assert lib.esparse_spmm(ctx._h, None, 4, None, None, 8, 16, 0, 2, 4, None, None, 0, -1) == -1
    assert b"null" in lib.esparse_last_error(ctx._h)
    assert lib.esparse_spmm(ctx._h, None, 0, None, None, 8, 16, 0, 2, 4, None, None, 0, -1) == 0   # M = 0
    assert lib.esparse_channel_stats(ctx._h, None, 4, 16, 0, 100, None, None) == -1
    assert lib.esparse_create(None, 0, None) == -1
    assert lib.esparse_output_error(ctx._h, None, None, 4, 4, 0, None, None) == -1      # null result pointers
    assert lib.esparse_spmm_group(ctx._h, 0, None, 4, None, None, 8, 16, 0, 2, 4, None, None, 0, -1) == -1   # count
    assert lib.esparse_spmm_group(ctx._h, 5, None, 4, None, None, 8, 16, 0, 2, 4, None, None, 0, -1) == -1
    assert lib.esparse_spmm_group(ctx._h, 2, None, 4, None, None, 8, 16, 0, 2, 4, None, None, 0, -1) == -1   # null arrays
    assert lib.esparse_spmm_group(ctx._h, 2, None, 4, None, None, 8, 16, 0, 3, 4, None, None, 0, -1) == -2   # no 3:4
    import ctypes as C
    nb = C.c_size_t(0)
    assert lib.esparse_spmm_group_workspace(3, 8, 512, 512, C.byref(nb)) == 0 and nb.value >= 65536 + 3 * 16 * 512 * 2
    assert lib.esparse_spmm_group_workspace(0, 8, 512, 512, C.byref(nb)) == -1
    assert lib.esparse_output_error(None, None, None, 4, 4, 0, None, None) == -1        # null context
    assert lib.esparse_tune_group(ctx._h, 0, 16, 512, 512, 0, 1, None, None) == -1       # count outside 1..4
    assert lib.esparse_tune_group(ctx._h, 5, 16, 512, 512, 0, 1, None, None) == -1
    assert lib.esparse_matrix_rate(ctx._h, 1, 0, 1, 0, None) == -1                       # null result pointer
    rate = C.c_double(0.0)
    assert lib.esparse_matrix_rate(ctx._h, 2, 0, 1, 0, C.byref(rate)) == -1              # sparse is 0 or 1
    assert lib.esparse_matrix_rate(ctx._h, 1, 7, 1, 0, C.byref(rate)) == -2              # no such dtype
    assert lib.esparse_matrix_rate(ctx._h, 1, 0, 1, 3, C.byref(rate)) == -1              # mix is 0, 1 or 2
    assert lib.esparse_matrix_rate(ctx._h, 0, 0, 1, 2, C.byref(rate)) == -2              # the stage mixes are 2:4 only
    # which kernel variants serve which weights is decided on the host, before any GPU call (the pointers are never used)
    vs = {esp.variant_name(v): v for v in range(esp.num_variants())}
    fake = C.c_void_p(1 << 20)

    def spmm_code(M, n, m, name):
        return lib.esparse_spmm(ctx._h, fake, M, fake, None, 512, 512, 0, n, m, fake, fake, 1 << 30, vs[name])

    assert spmm_code(256, 4, 8, "tile32_w8_t256") == -2       # the 32x32x32 kernel multiplies 2:4 weights only
    assert spmm_code(256, 2, 4, "tile48_w8_t128") == -2       # the tile48 kernels 4:8 weights only
    assert spmm_code(32, 4, 8, "tile48_w8_t128") == -2        # ... and 64 tokens or more
    assert spmm_code(64, 4, 8, "stream_w8_r1_d7") == -2       # 4:8 through the stream kernels: rings of four slots only
    assert spmm_code(256, 4, 8, "stream_w8_r1_d3") == -2      # ... and at most 128 tokens
    assert spmm_code(32, 4, 8, "ksplit_w8_r1_q") == -2        # one metadata load per four steps: at most 16 tokens
    assert spmm_code(256, 2, 4, "tile_w8_t256_h") == -2       # dense weights only
    assert b"variant" in lib.esparse_last_error(ctx._h)
    assert lib.esparse_read_rate(ctx._h, 1 << 20, None) == -1                             # null result pointer
    assert lib.esparse_read_rate(ctx._h, 16, C.byref(rate)) == -1                         # fewer than 4 KiB


def test_tune_table_text_roundtrip(tmp_path):
    ctx = esp.Context(0)
    p = tmp_path / "t.txt"
    p.write_text("# comment\n1 0 16 512 512 %s\n" % esp.variant_name(1))
    ctx.tune_load(str(p))
    q = tmp_path / "u.txt"
    ctx.tune_save(str(q))
    assert "1 0 16 512 512 " + esp.variant_name(1) in q.read_text()
    # a trailing count marks a choice for group launches; lines without it are for single products
    p.write_text("1 0 16 512 512 %s 3\n1 0 16 512 512 %s\n" % (esp.variant_name(4), esp.variant_name(1)))
    c2 = esp.Context(0)
    c2.tune_load(str(p))
    c2.tune_save(str(q))
    body = [l for l in q.read_text().splitlines() if not l.startswith("#")]
    assert sorted(body) == sorted(["1 0 16 512 512 %s 3" % esp.variant_name(4), "1 0 16 512 512 %s" % esp.variant_name(1)])


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libesparse.so")
    with pytest.raises(FileNotFoundError):
        binding.load_library()


def test_traffic_profile_rows_parse_and_name_existing_variants():
    """bench.py looks roofline.traffic up in profiles/product_kernels_hbm_traffic.txt by shape and kernel variant: every
    row must parse, name a variant the library has, and carry counter bytes of at least the algorithmic bytes."""
    names = {esp.variant_name(v) for v in range(esp.num_variants())}
    rows = [l for l in open(os.path.join(ROOT, "profiles", "product_kernels_hbm_traffic.txt")) if l.startswith("traffic ")]
    assert len(rows) >= 10
    seen = set()
    for line in rows:
        f = dict(kv.split("=", 1) for kv in line.split()[1:])
        assert f["variant"] in names, f["variant"]
        key = (f["members"], f["M"], f["N"], f["K"], f["variant"])
        assert key not in seen
        seen.add(key)
        moved = int(f["fetch_bytes"]) + int(f["write_bytes"])
        assert moved >= 0.98 * int(f["algorithmic_bytes"])
