"""CPU-side checks of the C ABI: the library loads, exports what the header declares, computes the
kept counts like the oracle and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import samkv_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "samkv.h")


@pytest.fixture(scope="module")
def S():
    lib = os.path.join(ROOT, "paper_2508_11661_amd", "lib", "libsamkv.so")
    if not os.path.exists(lib):
        from paper_2508_11661_amd import build
        build.build_library(verbose=False)
    from paper_2508_11661_amd import samkv
    return samkv


def test_library_exports_every_declared_symbol(S):
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(samkv_[a-z0-9_]+)\s*\(", text))
    assert declared == set(S.EXPORTS)
    for name in declared:
        assert hasattr(S._lib, name), name


def test_kept_count_matches_oracle_definition(S):
    rng = np.random.default_rng(0)
    cases = [(L, r) for L in (1, 2, 7, 20, 40, 100, 256, 1024, 2048, 4096, 65536)
             for r in (0.01, 0.05, 0.1, 0.15, 0.2, 0.25, 0.3, 0.5, 0.75, 1.0)]
    cases += [(int(rng.integers(1, 65537)), float(rng.uniform(0.001, 1.0))) for _ in range(2000)]
    for L, r in cases:
        assert S.samkv_kept_count(L, r) == O.kept_count(L, r), (L, r)
    assert [S.samkv_kept_count(L, 0.15) for L in (256, 1024, 2048, 4096)] == [39, 154, 308, 615]
    assert S.samkv_kept_count(0, 0.5) == 0 and S.samkv_kept_count(10, 0.0) == 0 and S.samkv_kept_count(10, 1.5) == 0


def test_top_p_and_mid_counts_match_oracle(S):
    rng = np.random.default_rng(1)
    for _ in range(50):
        n_layers, n_ctx = int(rng.integers(1, 6)), int(rng.integers(1, 9))
        mn = rng.standard_normal((n_layers, n_ctx)).astype(np.float32)
        mx = mn + np.abs(rng.standard_normal((n_layers, n_ctx))).astype(np.float32)
        anc = (mn + rng.uniform(-0.3, 1.3, size=(n_layers, n_ctx)) * (mx - mn)).astype(np.float32)
        got = S.samkv_top_p(anc.tolist(), mx.tolist(), mn.tolist())
        assert np.allclose(got, O.top_p(anc, mx, mn), rtol=1e-6, atol=1e-7)
    assert S.samkv_top_p([[4.0, 10.0, 0.0]], [[10.0, 10.0, 10.0]], [[0.0, 0.0, 0.0]]) == pytest.approx([0.6, 0.0, 0.0])
    for L, p, a, b in [(1000, 0.0, 64, 128), (1000, 1.0, 64, 128), (1000, 0.25, 64, 128), (100, 0.5, 64, 128),
                       (20, 0.1, 0, 0), (20, 0.0, 0, 0), (4096, 0.149, 64, 128), (7, 0.33, 1, 1)]:
        assert S.samkv_kept_count_mid(L, p, a, b) == O.kept_count_mid(L, p, a, b), (L, p, a, b)


def test_block_filter_count_matches_oracle(S):
    """Host arithmetic of the cross-document filter: tokens kept per head = what the oracle's rows hold."""
    rng = np.random.default_rng(5)
    for _ in range(40):
        n = int(rng.integers(1, 6))
        block = int(rng.choice([1, 4, 16, 64]))
        lens = [int(rng.integers(1, 40 * block)) for _ in range(n)]
        p = [float(x) for x in rng.choice([0.0, 0.1, 0.33, 0.5, 1.0], n)]
        n_init, n_local = int(rng.integers(0, 3)), int(rng.integers(1, 3))
        bs = [rng.standard_normal((1, -(-L // block))) for L in lens]
        want = O.block_filter(bs, lens, block, p, n_init, n_local).shape[1]
        c = _caches(S, n_ctx=n, lens=tuple(lens))
        pp = (ctypes.c_float * n)(*p)
        assert S._lib.samkv_block_filter_count(ctypes.byref(c), block, pp, n_init, n_local) == want, (lens, block, p)
    c = _caches(S, lens=(10, 8))
    assert S._lib.samkv_block_filter_count(ctypes.byref(c), 4, (ctypes.c_float * 2)(0.5, 0.5), 1, 0) == 0   # short last block


def test_workspace_bytes(S):
    assert S.samkv_workspace_bytes(10, 32, 8, 128, 32, 1540) > 0
    assert S.samkv_workspace_bytes(0, 32, 8, 128, 32, 1540) == 0


def _caches(S, n_ctx=2, hq=4, hkv=2, d=128, dtype=1, lens=(8, 8), k=True, v=True):
    fake = 0x1000  # never dereferenced: every call below must fail validation before any launch
    arr_len = (ctypes.c_int32 * n_ctx)(*lens[:n_ctx])
    arr_k = (ctypes.c_void_p * n_ctx)(*([fake] * n_ctx))
    c = S._Caches(n_ctx, hq, hkv, d, dtype, ctypes.cast(arr_len, ctypes.POINTER(ctypes.c_int32)),
                  ctypes.cast(arr_k, ctypes.POINTER(ctypes.c_void_p)) if k else None,
                  ctypes.cast(arr_k, ctypes.POINTER(ctypes.c_void_p)) if v else None)
    c._keep = (arr_len, arr_k)
    return c


def test_argument_errors_are_reported_before_any_launch(S):
    L = S._lib
    fake = ctypes.c_void_p(0x1000)
    ok = _caches(S)
    cu = (ctypes.c_int32 * 3)()
    # samkv_score
    assert L.samkv_score(None, fake, 4, None, 0, fake, fake, 1 << 20, None) == -1
    assert L.samkv_score(ctypes.byref(ok), None, 4, None, 0, fake, fake, 1 << 20, None) == -1
    assert L.samkv_score(ctypes.byref(ok), fake, 0, None, 0, fake, fake, 1 << 20, None) == -1
    assert L.samkv_score(ctypes.byref(ok), fake, 4, None, 0, fake, None, 0, None) == -3
    assert L.samkv_score(ctypes.byref(ok), fake, 4, None, 0, fake, fake, 16, None) == -3
    assert L.samkv_score(ctypes.byref(_caches(S, hq=3)), fake, 4, None, 0, fake, fake, 1 << 20, None) == -1
    assert L.samkv_score(ctypes.byref(_caches(S, d=96)), fake, 4, None, 0, fake, fake, 1 << 20, None) == -2
    assert L.samkv_score(ctypes.byref(_caches(S, dtype=7)), fake, 4, None, 0, fake, fake, 1 << 20, None) == -2
    assert L.samkv_score(ctypes.byref(_caches(S, lens=(8, 0))), fake, 4, None, 0, fake, fake, 1 << 20, None) == -1
    assert L.samkv_score(ctypes.byref(_caches(S, lens=(8, 70000))), fake, 4, None, 0, fake, fake, 1 << 20, None) == -2
    assert L.samkv_score(ctypes.byref(_caches(S, k=False)), fake, 4, None, 0, fake, fake, 1 << 20, None) == -1
    # samkv_score_select
    assert L.samkv_score_select(ctypes.byref(ok), fake, 4, None, 0, 0.5, 0, 0, fake, None, None, cu, fake, 1 << 20, None) == -1
    assert L.samkv_score_select(ctypes.byref(ok), fake, 4, None, 0, 0.0, 0, 0, fake, fake, None, cu, fake, 1 << 20, None) == -1
    assert L.samkv_score_select(ctypes.byref(ok), fake, 4, None, 0, 0.5, 0, 0, fake, fake, None, cu, None, 0, None) == -3
    assert L.samkv_score_select(ctypes.byref(_caches(S, lens=(8, 9000))), fake, 4, None, 0, 0.5, 0, 0, None, fake, None, cu,
                                fake, 1 << 20, None) == -1   # rows beyond the fused kernel need the score buffer
    # samkv_score_select_gather
    assert L.samkv_score_select_gather(ctypes.byref(ok), fake, 4, None, 0, 0.5, 0, 0, fake, fake, None, cu, None, fake, fake,
                                       1 << 20, None) == -1      # no k_c
    assert L.samkv_score_select_gather(ctypes.byref(ok), fake, 4, None, 0, 0.5, 0, 0, fake, fake, None, cu, fake, None, fake,
                                       1 << 20, None) == -1      # no v_c
    assert L.samkv_score_select_gather(ctypes.byref(ok), fake, 4, None, 0, 0.5, 0, 0, fake, None, None, cu, fake, fake, fake,
                                       1 << 20, None) == -1      # no idx
    assert L.samkv_score_select_gather(ctypes.byref(_caches(S, v=False)), fake, 4, None, 0, 0.5, 0, 0, fake, fake, None, cu,
                                       fake, fake, fake, 1 << 20, None) == -1   # V is read
    assert L.samkv_score_select_gather(ctypes.byref(ok), fake, 4, None, 0, 0.5, 0, 0, fake, fake, None, cu, fake, fake, None,
                                       0, None) == -3
    # samkv_topk_select
    assert L.samkv_topk_select(None, ctypes.byref(ok), 0.5, 0, 0, fake, None, cu, None, 0, None) == -1
    assert L.samkv_topk_select(fake, ctypes.byref(ok), 0.0, 0, 0, fake, None, cu, None, 0, None) == -1
    assert L.samkv_topk_select(fake, ctypes.byref(ok), 1.5, 0, 0, fake, None, cu, None, 0, None) == -1
    assert L.samkv_topk_select(fake, ctypes.byref(ok), float("nan"), 0, 0, fake, None, cu, None, 0, None) == -1
    assert L.samkv_topk_select(fake, ctypes.byref(ok), 0.5, 3, 2, fake, None, cu, None, 0, None) == -1   # 5 forced > k = 4
    assert L.samkv_topk_select(fake, ctypes.byref(ok), 0.5, -1, 0, fake, None, cu, None, 0, None) == -1
    # samkv_gather
    assert L.samkv_gather(ctypes.byref(_caches(S, v=False)), fake, 0.5, fake, fake, None) == -1
    assert L.samkv_gather(ctypes.byref(ok), None, 0.5, fake, fake, None) == -1
    assert L.samkv_gather(ctypes.byref(ok), fake, 2.0, fake, fake, None) == -1
    qp = (ctypes.c_void_p * 2)(0x1000, 0x1000)
    assert L.samkv_gather_q(ctypes.byref(ok), None, fake, 0.5, fake, None) == -1
    assert L.samkv_gather_q(ctypes.byref(ok), qp, None, 0.5, fake, None) == -1
    assert L.samkv_gather_q(ctypes.byref(ok), qp, fake, 0.0, fake, None) == -1
    assert L.samkv_gather_q(ctypes.byref(ok), (ctypes.c_void_p * 2)(0x1000, None), fake, 0.5, fake, None) == -1
    # block-granular selection
    pf = (ctypes.c_float * 2)(0.5, 0.5)
    ragged = _caches(S, lens=(10, 8))
    assert L.samkv_block_scores(None, ctypes.byref(ok), 4, fake, None) == -1
    assert L.samkv_block_scores(fake, ctypes.byref(ok), 0, fake, None) == -1
    assert L.samkv_block_scores(fake, ctypes.byref(ok), 5000, fake, None) == -1
    assert L.samkv_block_workspace_bytes(ctypes.byref(ok), 0) == 0
    assert L.samkv_block_workspace_bytes(ctypes.byref(ok), 4) >= 2 * 4 * 4
    assert L.samkv_block_select(fake, ctypes.byref(ok), 4, None, 1, 1, fake, None, cu, fake, 1 << 20, None) == -1
    assert L.samkv_block_select(fake, ctypes.byref(ok), 4, pf, -1, 1, fake, None, cu, fake, 1 << 20, None) == -1
    assert L.samkv_block_select(fake, ctypes.byref(ok), 4, pf, 1, 1, fake, None, cu, None, 0, None) == -3
    # a short last block that only some heads might keep: rejected (10 tokens in blocks of 4, no local block forced)
    assert L.samkv_block_select(fake, ctypes.byref(ragged), 4, pf, 1, 0, fake, None, cu, fake, 1 << 20, None) == -1
    assert L.samkv_block_select_filter(fake, ctypes.byref(ragged), 4, pf, 1, 0, fake, fake, 1 << 20, None) == -1
    assert L.samkv_block_select_filter(fake, ctypes.byref(ok), 4, pf, 1, 1, fake, None, 0, None) == -3
    assert L.samkv_block_select_filter(fake, ctypes.byref(ok), 4, pf, 1, 1, None, fake, 1 << 20, None) == -1
    assert L.samkv_gather_g(ctypes.byref(ok), None, 4, fake, fake, None) == -1
    assert L.samkv_gather_g(ctypes.byref(ok), fake, 0, fake, fake, None) == -1
    assert L.samkv_gather_q_g(ctypes.byref(ok), qp, fake, 4, None, None) == -1
    assert L.samkv_gather_q_v(ctypes.byref(ok), qp, fake, None, fake, None) == -1
    assert L.samkv_gather_q_v(ctypes.byref(ok), qp, fake, (ctypes.c_int32 * 3)(0, 9, 12), fake, None) == -1   # 9 > len 8
    assert L.samkv_gather_v(ctypes.byref(ok), fake, (ctypes.c_int32 * 3)(1, 2, 3), fake, fake, None) == -1
    # attention
    assert L.samkv_recompute_attn(None, fake, fake, 8, 4, 2, 128, 1, 0.1, fake, fake, None, 0, None) == -1
    assert L.samkv_recompute_attn(fake, fake, fake, 0, 4, 2, 128, 1, 0.1, fake, fake, None, 0, None) == -1
    assert L.samkv_recompute_attn(fake, fake, fake, 8, 4, 3, 128, 1, 0.1, fake, fake, None, 0, None) == -1
    assert L.samkv_recompute_attn(fake, fake, fake, 8, 4, 2, 100, 1, 0.1, fake, fake, None, 0, None) == -2
    assert L.samkv_recompute_attn(fake, fake, fake, 8, 4, 2, 128, 5, 0.1, fake, fake, None, 0, None) == -2
    assert L.samkv_recompute_attn(fake, fake, fake, 8, 4, 2, 128, 1, 0.0, fake, fake, None, 0, None) == -1
    assert L.samkv_query_attn(fake, 4, fake, fake, 4096, 4, 2, 128, 1, 0.1, fake, fake, None, 0, None) == -3
    # bf16 attention needs room for the half-precision copy of V; float32 causal attention needs none
    assert L.samkv_recompute_attn(fake, fake, fake, 8, 4, 2, 128, 1, 0.1, fake, fake, None, 0, None) == -3
    assert L.samkv_recompute_attn(fake, fake, fake, 8, 4, 2, 128, 1, 0.1, fake, fake, fake, 64, None) == -3
    assert L.samkv_recompute_attn(fake, fake, fake, 8, 4, 2, 128, 1, 0.1, fake, fake, ctypes.c_void_p(0x1010), 1 << 20, None) == -3
    # tensors are moved with 16-byte accesses: a pointer that is not 16-byte aligned is an argument error
    odd = ctypes.c_void_p(0x1008)
    assert L.samkv_recompute_attn(odd, fake, fake, 8, 4, 2, 128, 1, 0.1, fake, fake, fake, 1 << 20, None) == -1
    assert L.samkv_recompute_attn(fake, odd, fake, 8, 4, 2, 128, 1, 0.1, fake, fake, fake, 1 << 20, None) == -1
    assert L.samkv_recompute_attn(fake, fake, odd, 8, 4, 2, 128, 1, 0.1, fake, fake, fake, 1 << 20, None) == -1
    assert L.samkv_recompute_attn(fake, fake, fake, 8, 4, 2, 128, 1, 0.1, odd, fake, fake, 1 << 20, None) == -1
    assert L.samkv_recompute_attn(fake, fake, fake, 8, 4, 2, 128, 1, 0.1, fake, ctypes.c_void_p(0x1002), fake, 1 << 20, None) == -1
    assert L.samkv_query_attn(odd, 4, fake, fake, 64, 4, 2, 128, 1, 0.1, fake, fake, fake, 1 << 20, None) == -1
    assert L.samkv_score(ctypes.byref(ok), odd, 4, None, 0, fake, fake, 1 << 20, None) == -1
    assert L.samkv_score(ctypes.byref(ok), fake, 4, odd, 2, fake, fake, 1 << 20, None) == -1
    assert L.samkv_gather(ctypes.byref(ok), fake, 0.5, odd, fake, None) == -1
    assert L.samkv_gather(ctypes.byref(ok), fake, 0.5, fake, odd, None) == -1
    assert L.samkv_gather_q(ctypes.byref(ok), qp, fake, 0.5, odd, None) == -1
    assert L.samkv_gather_q(ctypes.byref(ok), (ctypes.c_void_p * 2)(0x1000, 0x1004), fake, 0.5, fake, None) == -1
    assert L.samkv_kv_update(fake, odd, fake, fake, 8, 2, 128, 1, 1, None) == -1
    misaligned = _caches(S)
    misaligned._keep[1][1] = 0x1008
    assert L.samkv_score(ctypes.byref(misaligned), fake, 4, None, 0, fake, fake, 1 << 20, None) == -1
    assert L.samkv_query_attn(fake, 0, fake, fake, 64, 4, 2, 128, 1, 0.1, fake, fake, None, 0, None) == -1
    pair = lambda *x: L.samkv_recompute_query_attn(*x)
    assert pair(fake, None, 4, fake, fake, 64, 4, 2, 128, 1, 0.1, fake, fake, fake, fake, fake, 1 << 30, None) == -1
    assert pair(fake, fake, 4, fake, fake, 64, 4, 2, 128, 1, 0.1, fake, fake, None, fake, fake, 1 << 30, None) == -1
    assert pair(fake, fake, 0, fake, fake, 64, 4, 2, 128, 1, 0.1, fake, fake, fake, fake, fake, 1 << 30, None) == -1
    assert pair(fake, fake, 4, fake, fake, 64, 4, 2, 128, 1, 0.1, fake, fake, fake, fake, None, 0, None) == -3
    assert pair(fake, fake, 4, fake, fake, 64, 4, 2, 96, 1, 0.1, fake, fake, fake, fake, fake, 1 << 30, None) == -2
    assert L.samkv_query_attn_self(fake, 4, fake, fake, 64, None, fake, 4, 2, 128, 1, 0.1, fake, fake, fake, 1 << 30, None) == -1
    assert L.samkv_query_attn_self(fake, 4, fake, fake, 64, fake, fake, 4, 2, 128, 1, 0.1, fake, fake, None, 0, None) == -3
    assert L.samkv_query_attn_self(fake, 4, fake, fake, 64, fake, fake, 4, 2, 128, 1, 0.1, fake, fake, fake, 64, None) == -3
    # samkv_kv_update
    assert L.samkv_kv_update(None, fake, fake, fake, 8, 2, 128, 1, 1, None) == -1
    assert L.samkv_kv_update(fake, fake, fake, fake, 0, 2, 128, 1, 1, None) == -1
    assert L.samkv_kv_update(fake, fake, fake, fake, 8, 2, 128, 1, 2, None) == -1
    assert L.samkv_kv_update(fake, fake, fake, fake, 8, 2, 96, 1, 1, None) == -2
    assert L.samkv_kv_update(fake, fake, fake, fake, 8, 2, 128, 3, 1, None) == -2
    # the measuring kernels
    assert L.samkv_peak_mfma_bf16(None, 4, 4, None) == -1
    assert L.samkv_peak_mfma_bf16_data(fake, 4, 4, 3, None) == -1     # unknown operand pattern
    assert L.samkv_peak_mfma_bf16_data(fake, 0, 4, 2, None) == -1
    assert L.samkv_peak_copy(fake, fake, 24, None) == -1               # not a multiple of 16
    assert S._lib.samkv_strerror(-3).decode().startswith("workspace")


def test_binding_refuses_to_run_without_library(tmp_path, monkeypatch):
    # the product path has no fallback: a missing library is an import error
    import importlib
    import paper_2508_11661_amd.samkv as mod
    monkeypatch.setattr(mod, "_LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        mod._load()
    importlib.reload(mod)
