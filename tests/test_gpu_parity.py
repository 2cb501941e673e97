"""GPU parity: every entry point of the C ABI against the fp64 oracle, element by element.

Each stage is fed the ORACLE's output of the previous stage, so no expected value and no oracle
input ever comes from the HIP path; one chained run per workload then checks the five calls
back to back."""
import math

import numpy as np
import pytest

from oracle import samkv_oracle as O
from paper_2508_11661_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def S():
    from paper_2508_11661_amd import samkv
    return samkv


def _ws(S, x, n_rows_q, m):
    import torch
    w = x.workload
    nbytes = S.samkv_workspace_bytes(len(x.k), w.n_q_heads, w.n_kv_heads, w.head_dim, n_rows_q, m)
    return torch.empty((nbytes,), dtype=torch.uint8, device="cuda")


def _stages(S, x, ratio, n_sink=0, n_local=0, use_bias=True, q_rec_seed_rows=None):
    """Runs every stage on the GPU from the oracle's previous stage and checks it."""
    import torch
    w = x.workload
    dt = w.dtype
    ref = H.oracle_front(x, ratio, n_sink, n_local, use_bias)
    m = int(ref.cu_k[-1])
    caches = H.upload_caches(x)
    q_tok = H.to_dev(x.q_tok, dt)
    q_loc = H.to_dev(x.q_loc, dt) if use_bias else None
    ws = _ws(S, x, w.n_q_tok, m)
    hkv, hq, d = w.n_kv_heads, w.n_q_heads, w.head_dim

    # ---- score
    scores = torch.full((hkv, caches.total_len), float("nan"), device="cuda")
    S.samkv_score(caches, q_tok, q_loc, scores, ws)
    sg = scores.cpu().numpy().astype(np.float64)
    bound = H.score_error_bound(x, ref)
    cu = np.concatenate([[0], np.cumsum(x.lens)])
    for i in range(len(x.k)):
        err = np.abs(sg[:, cu[i]:cu[i + 1]] - ref.scores[i])
        assert np.all(err <= bound[i]), f"score document {i}: max err {err.max():.3e}"

    # ---- select (on the GPU's own float32 scores; compared under the tie-margin rule)
    idx = torch.full((hkv, m), -1, dtype=torch.int32, device="cuda")
    cu_k_dev = torch.zeros((len(x.k) + 1,), dtype=torch.int32, device="cuda")
    cu_k = S.samkv_topk_select(scores, caches, ratio, n_sink, n_local, idx, cu_k_dev, ws)
    assert cu_k == ref.cu_k.tolist() and cu_k_dev.cpu().tolist() == cu_k
    in_margin, clean_heads = H.compare_kept_sets(idx.cpu().numpy(), ref, n_sink, n_local)

    # ---- select again on the oracle's scores rounded to float32: bit-exact against the oracle's
    #      selection of those same float32 values
    s32 = [s.astype(np.float32) for s in ref.scores]
    idx32, _ = O.select([s.astype(np.float64) for s in s32], ratio, n_sink, n_local)
    scores2 = torch.from_numpy(np.concatenate(s32, axis=1)).cuda()
    idx2 = torch.full((hkv, m), -1, dtype=torch.int32, device="cuda")
    S.samkv_topk_select(scores2, caches, ratio, n_sink, n_local, idx2, None, ws)
    assert np.array_equal(idx2.cpu().numpy(), idx32)

    # ---- gather from the oracle's kept sets: bit-exact
    idx_ref = torch.from_numpy(ref.idx).cuda()
    k_c = torch.zeros((hkv, m, d), dtype=H.torch_dtype(dt), device="cuda")
    v_c = torch.zeros_like(k_c)
    S.samkv_gather(caches, idx_ref, ratio, k_c, v_c)
    assert np.array_equal(k_c.float().cpu().numpy(), ref.k_c)
    assert np.array_equal(v_c.float().cpu().numpy(), ref.v_c)

    # ---- attention over the oracle's compacted cache
    scale = 1.0 / math.sqrt(d)
    q_rec_np = synth.make_q_rec(w, x.layer, m)
    q_rec = H.to_dev(q_rec_np, dt)
    kc_ref, vc_ref = H.to_dev(ref.k_c, dt), H.to_dev(ref.v_c, dt)
    out = torch.full((hq, m, d), float("nan"), device="cuda")
    lse = torch.full((hq, m), float("nan"), device="cuda")
    S.samkv_recompute_attn(q_rec, kc_ref, vc_ref, scale, out, lse, ws)
    o_ref, l_ref = O.attention(q_rec_np, ref.k_c, ref.v_c, scale, True)
    e_rec = H.check_attention(out.cpu().numpy(), lse.cpu().numpy(), o_ref, l_ref, dt, "recompute")

    out_q = torch.full((hq, w.n_q_tok, d), float("nan"), device="cuda")
    lse_q = torch.full((hq, w.n_q_tok), float("nan"), device="cuda")
    S.samkv_query_attn(q_tok, kc_ref, vc_ref, scale, out_q, lse_q, ws)
    oq_ref, lq_ref = O.attention(x.q_tok, ref.k_c, ref.v_c, scale, False)
    e_q = H.check_attention(out_q.cpu().numpy(), lse_q.cpu().numpy(), oq_ref, lq_ref, dt, "query")

    # ---- the five calls chained on the GPU: every head, through the GPU's own kept sets
    buf = S.alloc_layer_buffers(caches, w.n_q_tok, ratio)
    S.hot_path(caches, q_tok, q_loc, q_rec, ratio, scale, buf, n_sink, n_local)
    torch.cuda.synchronize()
    idx_chain = buf.idx.cpu().numpy()
    H.compare_kept_sets(idx_chain, ref, n_sink, n_local)
    H.check_chained(x, ref, idx_chain, buf.k_c.float().cpu().numpy(), buf.v_c.float().cpu().numpy(),
                    buf.rec_out.cpu().numpy(), buf.rec_lse.cpu().numpy(), buf.q_out.cpu().numpy(), buf.q_lse.cpu().numpy(),
                    q_rec_np, scale)
    # ---- the fused calls (score+select+gather, both attentions) and the five separate calls: the same bits, except
    #      for the bf16 query attention, which the pair call computes over all keys in one chunk and the separate call
    #      in several that it merges (both were just held against the oracle; here: within the bar of each other)
    buf2 = S.alloc_layer_buffers(caches, w.n_q_tok, ratio)
    S.hot_path(caches, q_tok, q_loc, q_rec, ratio, scale, buf2, n_sink, n_local, fused=False)
    torch.cuda.synchronize()
    for name in ("idx", "k_c", "v_c", "rec_out", "rec_lse", "q_out", "q_lse"):
        a, b = getattr(buf, name), getattr(buf2, name)
        if dt == "bf16" and name in ("q_out", "q_lse"):
            assert (a - b).abs().max().item() <= H.BF16_ABS, f"fused and separate calls differ in {name}"
        else:
            assert torch.equal(a, b), f"fused and separate calls differ in {name}"
    H.check_chained(x, ref, idx_chain, buf2.k_c.float().cpu().numpy(), buf2.v_c.float().cpu().numpy(),
                    buf2.rec_out.cpu().numpy(), buf2.rec_lse.cpu().numpy(), buf2.q_out.cpu().numpy(),
                    buf2.q_lse.cpu().numpy(), q_rec_np, scale, what="separate calls")
    return dict(in_margin=in_margin, clean=len(clean_heads), e_rec=e_rec, e_q=e_q, m=m)


def test_config1_tiny_f32(S):
    r = _stages(S, synth.make_layer(synth.WORKLOADS["tiny_f32"]), 0.15)
    assert r["m"] == 156


def test_config2_llama_layer_bf16(S):
    r = _stages(S, synth.make_layer(synth.WORKLOADS["llama3_8b_layer"]), 0.15)
    assert r["m"] == 1540


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 128), ("f32", 64)])
def test_ragged_documents_with_forced_positions(S, dtype, d):
    # lengths off every tile size; M = 90 + 24 + 308 + 154 = 576 kept rows; initial/local positions forced
    x = synth.make_small(11, dtype, [300, 77, 1025, 513], 8, 2, d, 5, 7)
    _stages(S, x, 0.3, n_sink=4, n_local=8)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_full_budget_is_dense_attention(S, dtype):
    # budget 100 %: every token kept, compacted cache = concatenation, query attention = dense attention
    x = synth.make_small(12, dtype, [130, 65, 200], 4, 4, 128, 9, 3)
    r = _stages(S, x, 1.0)
    assert r["m"] == 395 and r["in_margin"] == 0


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_single_document_and_no_local_cache(S, dtype):
    x = synth.make_small(13, dtype, [333], 4, 1, 64, 3, 2, dup=0.0)
    _stages(S, x, 0.2)
    x = synth.make_small(14, dtype, [100, 90], 2, 2, 128, 1, 1)
    _stages(S, x, 0.5, use_bias=False)


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64)])
def test_many_short_documents(S, dtype, d):
    # more than 64 documents: Eq. 1 runs as separate pooling / bias / fold launches instead of the single launch
    # that short inputs take; ragged lengths, a local Q cache of 5 rows
    lens = [40 + (7 * i) % 90 for i in range(70)]
    x = synth.make_small(17, dtype, lens, 8, 2, d, 6, 5)
    _stages(S, x, 0.25)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_degenerate_sizes(S, dtype):
    # documents of one and two tokens, compacted cache of a handful of rows
    x = synth.make_small(15, dtype, [1, 2, 1], 2, 1, 64, 1, 1, planted=0.0, dup=0.0)
    r = _stages(S, x, 0.15)
    assert r["m"] == 3
    x = synth.make_small(16, dtype, [1], 1, 1, 128, 2, 1, planted=0.0, dup=0.0)
    assert _stages(S, x, 1.0)["m"] == 1


@pytest.mark.parametrize("L", [1, 2, 63, 64, 65, 1000, 1024, 1025, 4096, 4097, 16384, 20000, 65536])
def test_select_alone_exact_with_ties(S, L):
    """Selection in isolation on float32 scores with many exact ties (quantised values): bit-exact."""
    import torch
    rng = np.random.default_rng(L)
    hkv = 2
    lens = [L, max(1, L // 3)]
    rows = [np.round(rng.standard_normal((hkv, n)) * 4.0).astype(np.float32) / 4.0 for n in lens]
    rows[0][0, : min(L, 50)] = 0.0           # a run of equal scores at the threshold region
    rows[0][1, :] = -1.5                       # a whole row of equal scores
    ratio = 0.15
    n_sink, n_local = (1, 2) if min(O.kept_count(n, ratio) for n in lens) >= 3 else (0, 0)
    want, cu = O.select([r.astype(np.float64) for r in rows], ratio, n_sink, n_local)

    # select reads no K/V: uninitialised caches of the right shape carry the lengths
    k = [torch.empty((hkv, n, 64), dtype=torch.bfloat16, device="cuda") for n in lens]
    caches = S.Caches(k, None, hkv)
    scores = torch.from_numpy(np.concatenate(rows, axis=1)).cuda()
    idx = torch.full((hkv, int(cu[-1])), -1, dtype=torch.int32, device="cuda")
    got_cu = S.samkv_topk_select(scores, caches, ratio, n_sink, n_local, idx, None, None)
    assert got_cu == cu.tolist()
    assert np.array_equal(idx.cpu().numpy(), want)
    # negative zero, infinities and denormals keep their numeric order
    special = np.array([[-0.0, 0.0, np.inf, -np.inf, 1e-40, -1e-40, 3.0, -3.0]], dtype=np.float32)
    k = [torch.empty((1, 8, 64), dtype=torch.bfloat16, device="cuda")]
    caches = S.Caches(k, None, 1)
    idx = torch.full((1, 4), -1, dtype=torch.int32, device="cuda")
    S.samkv_topk_select(torch.from_numpy(special).cuda(), caches, 0.5, 0, 0, idx, None, None)
    assert idx.cpu().numpy().tolist() == [[0, 2, 4, 6]]


def test_gather_clamps_out_of_range_indices(S):
    import torch
    x = synth.make_small(17, "bf16", [40, 50], 2, 2, 128, 2, 2)
    caches = H.upload_caches(x)
    ratio = 0.1
    m = sum(O.kept_count(n, ratio) for n in x.lens)
    idx = torch.tensor([[-5, 0, 10, 39, 0, 49, 1000, 7, 8]] * 2, dtype=torch.int32, device="cuda")
    assert idx.shape[1] == m
    k_c = torch.zeros((2, m, 128), dtype=torch.bfloat16, device="cuda")
    v_c = torch.zeros_like(k_c)
    S.samkv_gather(caches, idx, ratio, k_c, v_c)
    clamped = np.array([0, 0, 10, 39, 0, 49, 49, 7, 8])
    want = np.stack([np.concatenate([x.k[0][g, clamped[:4]], x.k[1][g, clamped[4:]]]) for g in range(2)])
    assert np.array_equal(k_c.float().cpu().numpy(), want)


def test_outputs_are_deterministic(S):
    import torch
    x = synth.make_layer(synth.WORKLOADS["llama3_8b_layer"])
    w = x.workload
    caches = H.upload_caches(x)
    q_tok, q_loc = H.to_dev(x.q_tok, w.dtype), H.to_dev(x.q_loc, w.dtype)
    m = sum(S.samkv_kept_count(n, 0.15) for n in x.lens)
    q_rec = H.to_dev(synth.make_q_rec(w, 0, m), w.dtype)
    runs = []
    for _ in range(2):
        buf = S.alloc_layer_buffers(caches, w.n_q_tok, 0.15)
        S.hot_path(caches, q_tok, q_loc, q_rec, 0.15, 1.0 / math.sqrt(w.head_dim), buf)
        torch.cuda.synchronize()
        runs.append([t.clone() for t in (buf.scores, buf.idx, buf.k_c, buf.rec_out, buf.q_out, buf.q_lse)])
    for a, b in zip(*runs):
        assert torch.equal(a, b)


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 128), ("f32", 64)])
def test_kv_update_overwrite_and_fusion(S, dtype, d):
    """Eq. 4 on the compacted cache.  float32 caches: relative 1e-5 of the row norm.  bf16 caches: the result is
    rounded to bf16 once, so it may sit one bf16 step (2^-8 relative) from the rounded oracle value."""
    import torch
    x = synth.make_small(31, dtype, [300, 77, 129], 4, 2, d, 3, 2)
    ref = H.oracle_front(x, 0.5)
    w = x.workload
    k_new = synth.make_recomputed_rows(w, 0, ref.k_c, x.sigma_k, 0)
    v_new = synth.make_recomputed_rows(w, 0, ref.v_c, x.sigma_v, 1)
    k_new[0, 5] = 0.0                      # a zero row: the cosine is undefined, the new row is taken
    for mode, fusion in ((S.SAMKV_OVERWRITE, False), (S.SAMKV_FUSION, True)):
        k_c, v_c = H.to_dev(ref.k_c, dtype), H.to_dev(ref.v_c, dtype)
        S.samkv_kv_update(k_c, v_c, H.to_dev(k_new, dtype), H.to_dev(v_new, dtype), mode)
        for got, old, new in ((k_c, ref.k_c, k_new), (v_c, ref.v_c, v_new)):
            want = O.kv_update(old, new, fusion)
            g = got.float().cpu().numpy().astype(np.float64)
            if not fusion:
                assert np.array_equal(g, want)
                continue
            row = np.linalg.norm(want, axis=2, keepdims=True)
            tol = 1e-5 * row + 1e-7 if dtype == "f32" else 2.0 ** -8 * np.abs(want) + 1e-5 * row + 1e-7
            assert np.all(np.abs(g - want) <= tol), f"max excess {(np.abs(g - want) - tol).max():.3e}"


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 128), ("f32", 64)])
def test_gather_q_cache_bit_exact(S, dtype, d):
    import torch
    x = synth.make_small(41, dtype, [300, 77, 1025, 5], 8, 2, d, 3, 2)
    ref = H.oracle_front(x, 0.3)
    q_np = synth.make_q_cache(x.workload, 0, x.lens)
    caches = H.upload_caches(x)
    q_dev = [H.to_dev(a, dtype) for a in q_np]
    m = int(ref.cu_k[-1])
    q_rec = torch.zeros((8, m, d), dtype=H.torch_dtype(dtype), device="cuda")
    S.samkv_gather_q(caches, q_dev, torch.from_numpy(ref.idx).cuda(), 0.3, q_rec)
    assert np.array_equal(q_rec.float().cpu().numpy(), O.gather_q(q_np, ref.idx, ref.cu_k))


def test_hot_path_under_hip_graph_capture_replays_identically(S):
    """The five calls copy nothing from the host and allocate nothing, so they can be captured into a HIP graph;
    every replay (with eager work and synchronisations in between) must reproduce the eager results bit for bit."""
    import torch
    x = synth.make_small(51, "bf16", [300, 200, 260], 8, 2, 128, 8, 16)
    w = x.workload
    caches = H.upload_caches(x)
    q_tok, q_loc = H.to_dev(x.q_tok, w.dtype), H.to_dev(x.q_loc, w.dtype)
    ratio, scale = 0.25, 1.0 / math.sqrt(w.head_dim)
    m = sum(S.samkv_kept_count(n, ratio) for n in x.lens)
    q_rec = H.to_dev(synth.make_q_rec(w, 0, m), w.dtype)
    buf = S.alloc_layer_buffers(caches, w.n_q_tok, ratio)
    S.hot_path(caches, q_tok, q_loc, q_rec, ratio, scale, buf)
    torch.cuda.synchronize()
    eager = [t.clone() for t in (buf.scores, buf.idx, buf.k_c, buf.v_c, buf.rec_out, buf.rec_lse, buf.q_out, buf.q_lse)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        S.hot_path(caches, q_tok, q_loc, q_rec, ratio, scale, buf)       # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        S.hot_path(caches, q_tok, q_loc, q_rec, ratio, scale, buf)
    for rep in range(3):
        for t in (buf.scores, buf.k_c, buf.v_c, buf.rec_out, buf.rec_lse, buf.q_out, buf.q_lse):
            t.fill_(float("nan"))                                         # eager work between replays
        buf.idx.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip((buf.scores, buf.idx, buf.k_c, buf.v_c, buf.rec_out, buf.rec_lse, buf.q_out, buf.q_lse), eager):
            assert torch.equal(got, want), f"replay {rep} differs from the eager run"


def test_select_with_per_document_top_p_and_explicit_gather(S):
    """Eq. 3's P_i per document on the middle segment, forced initial/local positions, a document that keeps only
    its forced positions and one that keeps nothing at all; gather with the explicit prefix sums."""
    import torch
    x = synth.make_small(61, "bf16", [700, 130, 64, 1500, 33], 8, 2, 128, 4, 8)
    n = len(x.k)
    scores32 = [s.astype(np.float32) for s in O.score(O.personalized_query(x.q_tok, x.q_loc, n), x.k)]
    caches = H.upload_caches(x)
    dev_scores = torch.from_numpy(np.concatenate(scores32, axis=1)).cuda()
    for p, n_sink, n_local in (([0.15, 0.5, 0.0, 0.07, 1.0], 8, 16), ([0.3, 0.0, 0.0, 0.2, 0.0], 0, 0)):
        want, cu = O.select_v([s.astype(np.float64) for s in scores32], p, n_sink, n_local)
        m = int(cu[-1])
        idx = torch.full((2, m), -1, dtype=torch.int32, device="cuda")
        cu_dev = torch.zeros((n + 1,), dtype=torch.int32, device="cuda")
        got_cu = S.samkv_topk_select_v(dev_scores, caches, p, n_sink, n_local, idx, cu_dev)
        assert got_cu == cu.tolist() == cu_dev.cpu().tolist()
        assert np.array_equal(idx.cpu().numpy(), want)
        k_c = torch.zeros((2, m, 128), dtype=torch.bfloat16, device="cuda")
        v_c = torch.zeros_like(k_c)
        S.samkv_gather_v(caches, idx, got_cu, k_c, v_c)
        k_ref, v_ref = O.gather(x.k, x.v, want, cu)
        assert np.array_equal(k_c.float().cpu().numpy(), k_ref) and np.array_equal(v_c.float().cpu().numpy(), v_ref)


def test_block_level_scores_selection_and_gather(S):
    """Sec. 3.2 at block granularity: block score = score of the mean key; initial / local blocks forced; the kept
    blocks come back as token positions that gather_v and gather_q_v take.  Ragged last blocks, a document shorter
    than one block, one made of forced blocks only, shares 0 and 1."""
    import torch
    lens = [700, 130, 64, 1500, 33, 4096 + 17]
    x = synth.make_small(71, "bf16", lens, 8, 2, 128, 4, 8)
    n = len(lens)
    q_hat = O.personalized_query(x.q_tok, x.q_loc, n)
    tok32 = [s.astype(np.float32) for s in O.score(q_hat, x.k)]
    caches = H.upload_caches(x)
    dev_scores = torch.from_numpy(np.concatenate(tok32, axis=1)).cuda()
    q_cache = synth.make_q_cache(x.workload, 0, x.lens)
    dev_q = [H.to_dev(q, "bf16") for q in q_cache]
    for block, n_init, n_local, p in ((64, 1, 2, [0.25, 0.5, 0.3, 0.1, 1.0, 0.05]), (16, 2, 1, [0.0, 1.0, 0.5, 0.2, 0.4, 0.15]),
                                      (64, 0, 1, [0.3, 0.0, 0.0, 0.2, 0.0, 0.1])):
        nbs = [-(-L // block) for L in lens]
        # (1) block scores: against the oracle's definition (mean key, fp64), and against the exact mean of the
        #     same float32 token scores (only the kernel's own summation error is left)
        b_ref = O.block_scores(q_hat, x.k, block)
        bs = torch.full((2, sum(nbs)), float("nan"), dtype=torch.float32, device="cuda")
        S.samkv_block_scores(dev_scores, caches, block, bs)
        got = bs.cpu().numpy().astype(np.float64)
        off = 0
        for i, L in enumerate(lens):
            smax = float(np.abs(tok32[i]).max())
            g_i = got[:, off:off + nbs[i]]
            assert np.abs(g_i - b_ref[i]).max() <= 2e-5 * smax + 1e-6, (block, i)
            exact = np.stack([tok32[i][:, t * block:(t + 1) * block].astype(np.float64).mean(axis=1) for t in range(nbs[i])], axis=1)
            assert np.abs(g_i - exact).max() <= block * 2.0 ** -24 * smax, (block, i)
            off += nbs[i]
        # (2) selection on the oracle's block scores rounded to float32: both sides decide on the same numbers
        b32 = [b.astype(np.float32) for b in b_ref]
        want, cu = O.block_select([b.astype(np.float64) for b in b32], lens, block, p, n_init, n_local)
        m = int(cu[-1])
        idx = torch.full((2, m), -1, dtype=torch.int32, device="cuda")
        cu_dev = torch.zeros((n + 1,), dtype=torch.int32, device="cuda")
        ws = torch.empty(S.samkv_block_workspace_bytes(caches, block), dtype=torch.uint8, device="cuda")
        got_cu = S.samkv_block_select(torch.from_numpy(np.concatenate(b32, axis=1)).cuda(), caches, block, p, n_init,
                                      n_local, idx, cu_dev, ws)
        assert got_cu == cu.tolist() == cu_dev.cpu().tolist()
        assert np.array_equal(idx.cpu().numpy(), want), (block, n_init, n_local)
        # (3) the token positions feed the explicit-count gathers
        k_c = torch.zeros((2, m, 128), dtype=torch.bfloat16, device="cuda")
        v_c = torch.zeros_like(k_c)
        S.samkv_gather_v(caches, idx, got_cu, k_c, v_c)
        k_want, v_want = O.gather(x.k, x.v, want, cu)
        assert np.array_equal(k_c.float().cpu().numpy(), k_want) and np.array_equal(v_c.float().cpu().numpy(), v_want)
        q_rec = torch.zeros((8, m, 128), dtype=torch.bfloat16, device="cuda")
        S.samkv_gather_q_v(caches, dev_q, idx, got_cu, q_rec)
        assert np.array_equal(q_rec.float().cpu().numpy(), O.gather_q(q_cache, want, cu))
        # (4) the whole chain on the device (token scores -> block scores -> selection): the kept block sets may
        #     differ from the oracle's only at blocks whose score is within the tie margin of the threshold
        idx2 = torch.full((2, m), -1, dtype=torch.int32, device="cuda")
        assert S.samkv_block_select(bs, caches, block, p, n_init, n_local, idx2, None, ws) == cu.tolist()
        got2 = idx2.cpu().numpy()
        for g in range(2):
            for i in range(n):
                a, b = set(got2[g, cu[i]:cu[i + 1]].tolist()), set(want[g, cu[i]:cu[i + 1]].tolist())
                if a == b:
                    continue
                kept_blocks = sorted({t // block for t in b})
                free = [t for t in kept_blocks if n_init <= t < nbs[i] - n_local]
                tau = min(b_ref[i][g, t] for t in free)
                for t in {t // block for t in a ^ b}:
                    assert abs(b_ref[i][g, t] - tau) <= H.TIE_MARGIN * max(1.0, abs(tau))


def test_select_full_length_row_of_equal_scores(S):
    """A maximum-length row whose scores are all equal: ties go to the lower positions, and a full budget keeps all
    65536 of them (the counts of the ordered compaction reach 2^16)."""
    import torch
    L = 65536
    k = torch.zeros((1, L, 64), dtype=torch.float32, device="cuda")
    caches = S.Caches([k], None, 1)
    sc = np.full((1, L), 0.25, np.float32)
    dev = torch.from_numpy(sc).cuda()
    for ratio, n_sink, n_local in ((1.0, 0, 0), (0.5, 0, 0), (0.25, 4, 100)):
        want, cu = O.select([sc.astype(np.float64)], ratio, n_sink, n_local)
        idx = torch.full((1, int(cu[-1])), -1, dtype=torch.int32, device="cuda")
        assert S.samkv_topk_select(dev, caches, ratio, n_sink, n_local, idx, None) == cu.tolist()
        assert np.array_equal(idx.cpu().numpy(), want)


def test_block_filter_across_documents_and_gather_by_global_positions(S):
    """Second filter of Sec. 3.2 (min-max reading, decisions in float32 on both sides): surviving blocks per KV head
    as global token positions, bit-exact; K/V and Q-cache gathers by global position, bit-exact."""
    import torch
    lens = [700, 130, 64, 1500, 33, 4096 + 17]
    x = synth.make_small(72, "bf16", lens, 8, 2, 128, 4, 8)
    q_hat = O.personalized_query(x.q_tok, x.q_loc, len(lens))
    caches = H.upload_caches(x)
    q_cache = synth.make_q_cache(x.workload, 0, x.lens)
    dev_q = [H.to_dev(q, "bf16") for q in q_cache]
    for block, n_init, n_local, p in ((64, 1, 2, [0.25, 0.5, 0.3, 0.1, 1.0, 0.05]), (16, 2, 1, [0.0, 1.0, 0.5, 0.2, 0.4, 0.15]),
                                      (16, 0, 1, [0.0, 0.0, 0.0, 0.0, 0.0, 0.0]), (8, 1, 1, [1.0] * 6)):
        b32 = [b.astype(np.float32) for b in O.block_scores(q_hat, x.k, block)]
        want = O.block_filter([b.astype(np.float64) for b in b32], lens, block, p, n_init, n_local)
        m = want.shape[1]
        assert S.samkv_block_filter_count(caches, block, p, n_init, n_local) == m
        gidx = torch.full((2, m), -1, dtype=torch.int32, device="cuda")
        ws = torch.empty(S.samkv_block_workspace_bytes(caches, block), dtype=torch.uint8, device="cuda")
        S.samkv_block_select_filter(torch.from_numpy(np.concatenate(b32, axis=1)).cuda(), caches, block, p, n_init,
                                    n_local, gidx, ws)
        assert np.array_equal(gidx.cpu().numpy(), want), (block, n_init, n_local)
        k_c = torch.zeros((2, m, 128), dtype=torch.bfloat16, device="cuda")
        v_c = torch.zeros_like(k_c)
        S.samkv_gather_g(caches, gidx, k_c, v_c)
        assert np.array_equal(k_c.float().cpu().numpy(), O.gather_global(x.k, want))
        assert np.array_equal(v_c.float().cpu().numpy(), O.gather_global(x.v, want))
        q_rec = torch.zeros((8, m, 128), dtype=torch.bfloat16, device="cuda")
        S.samkv_gather_q_g(caches, dev_q, gidx, q_rec)
        assert np.array_equal(q_rec.float().cpu().numpy(), O.gather_global(q_cache, want, group=4))


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("f32", 128), ("bf16", 64)])
def test_gather_by_global_positions_other_row_sizes(S, dtype, d):
    import torch
    x = synth.make_small(73, dtype, [300, 77, 1025, 5], 8, 2, d, 3, 2)
    rng = np.random.default_rng(73)
    total = sum(x.lens)
    gidx = np.sort(rng.choice(total, size=(2, 501), replace=True), axis=1).astype(np.int32)   # repeats are legal
    caches = H.upload_caches(x)
    k_c = torch.zeros((2, 501, d), dtype=H.torch_dtype(dtype), device="cuda")
    v_c = torch.zeros_like(k_c)
    S.samkv_gather_g(caches, torch.from_numpy(gidx).cuda(), k_c, v_c)
    assert np.array_equal(k_c.float().cpu().numpy(), O.gather_global(x.k, gidx))
    assert np.array_equal(v_c.float().cpu().numpy(), O.gather_global(x.v, gidx))


@pytest.mark.parametrize("dtype,d,lens,ratio,n_sink,n_local", [
    ("bf16", 128, [300, 77, 1025, 513], 0.3, 4, 8), ("bf16", 64, [1000, 1024, 5], 0.15, 0, 0),
    ("f32", 128, [4096, 4097, 130], 0.1, 2, 2), ("f32", 64, [8192, 63, 2500], 0.2, 0, 8),
    ("bf16", 128, [9000, 700], 0.05, 1, 1),        # longer than the fused kernel's rows: falls back to two launches
])
def test_fused_score_select_equals_the_two_calls(S, dtype, d, lens, ratio, n_sink, n_local):
    """One pass over K must keep exactly what samkv_score followed by samkv_topk_select keeps (bit-identical scores
    and positions), and that must agree with the oracle under the tie-margin rule."""
    import torch
    x = synth.make_small(81, dtype, lens, 8, 2, d, 6, 9)
    ref = H.oracle_front(x, ratio, n_sink, n_local)
    caches = H.upload_caches(x)
    q_tok, q_loc = H.to_dev(x.q_tok, dtype), H.to_dev(x.q_loc, dtype)
    m = int(ref.cu_k[-1])
    ws = _ws(S, x, x.workload.n_q_tok, m)
    sc_a = torch.full((2, caches.total_len), float("nan"), device="cuda")
    idx_a = torch.full((2, m), -1, dtype=torch.int32, device="cuda")
    S.samkv_score(caches, q_tok, q_loc, sc_a, ws)
    cu_a = S.samkv_topk_select(sc_a, caches, ratio, n_sink, n_local, idx_a, None, ws)
    sc_b = torch.full((2, caches.total_len), float("nan"), device="cuda")
    idx_b = torch.full((2, m), -1, dtype=torch.int32, device="cuda")
    cu_dev = torch.zeros((len(lens) + 1,), dtype=torch.int32, device="cuda")
    cu_b = S.samkv_score_select(caches, q_tok, q_loc, ratio, n_sink, n_local, sc_b, idx_b, cu_dev, ws)
    assert cu_a == cu_b == ref.cu_k.tolist() == cu_dev.cpu().tolist()
    assert torch.equal(sc_a, sc_b) and torch.equal(idx_a, idx_b)
    H.compare_kept_sets(idx_b.cpu().numpy(), ref, n_sink, n_local)
    if max(lens) <= 8192:                           # without a score buffer
        idx_c = torch.full((2, m), -1, dtype=torch.int32, device="cuda")
        S.samkv_score_select(caches, q_tok, q_loc, ratio, n_sink, n_local, None, idx_c, None, ws)
        assert torch.equal(idx_a, idx_c)
    else:
        with pytest.raises(S.SamKVError):
            S.samkv_score_select(caches, q_tok, q_loc, ratio, n_sink, n_local, None, idx_b, None, ws)


@pytest.mark.parametrize("dtype,d,lens,ratio,n_sink,n_local,hq,hkv", [
    ("bf16", 128, [300, 77, 1025, 513], 0.3, 4, 8, 8, 2), ("bf16", 64, [1000, 1024, 5], 0.15, 0, 0, 8, 2),
    ("f32", 128, [4096, 4097, 130], 0.1, 2, 2, 8, 2), ("f32", 64, [8192, 63, 2500], 0.2, 0, 8, 8, 2),
    ("bf16", 128, [9000, 700], 0.05, 1, 1, 8, 2),  # longer than the fused kernel's rows: falls back to three launches
    ("bf16", 64, [37 + (i % 5) for i in range(40)], 0.25, 1, 2, 64, 64),  # 2560 rows: compaction as its own kernel
])
def test_fused_score_select_gather_equals_the_separate_calls(S, dtype, d, lens, ratio, n_sink, n_local, hq, hkv):
    """score + select + gather in one call: positions and compacted rows bit-identical to the separate calls, and the
    compacted rows are exactly the source rows at the positions the call itself reports (checked on the host)."""
    import torch
    x = synth.make_small(83, dtype, lens, hq, hkv, d, 6, 9)
    ref = H.oracle_front(x, ratio, n_sink, n_local)
    caches = H.upload_caches(x)
    q_tok, q_loc = H.to_dev(x.q_tok, dtype), H.to_dev(x.q_loc, dtype)
    m = int(ref.cu_k[-1])
    ws = _ws(S, x, x.workload.n_q_tok, m)
    td = H.torch_dtype(dtype)
    sc_a = torch.full((hkv, caches.total_len), float("nan"), device="cuda")
    idx_a = torch.full((hkv, m), -1, dtype=torch.int32, device="cuda")
    k_a, v_a = torch.zeros((hkv, m, d), dtype=td, device="cuda"), torch.zeros((hkv, m, d), dtype=td, device="cuda")
    S.samkv_score_select(caches, q_tok, q_loc, ratio, n_sink, n_local, sc_a, idx_a, None, ws)
    S.samkv_gather_v(caches, idx_a, ref.cu_k.tolist(), k_a, v_a)
    sc_b = torch.full((hkv, caches.total_len), float("nan"), device="cuda")
    idx_b = torch.full((hkv, m), -1, dtype=torch.int32, device="cuda")
    k_b, v_b = torch.ones((hkv, m, d), dtype=td, device="cuda"), torch.ones((hkv, m, d), dtype=td, device="cuda")
    cu_b = S.samkv_score_select_gather(caches, q_tok, q_loc, ratio, n_sink, n_local, sc_b, idx_b, None, k_b, v_b, ws)
    assert cu_b == ref.cu_k.tolist()
    assert torch.equal(sc_a, sc_b) and torch.equal(idx_a, idx_b)
    assert torch.equal(k_a, k_b) and torch.equal(v_a, v_b)
    H.compare_kept_sets(idx_b.cpu().numpy(), ref, n_sink, n_local)
    idx_h = idx_b.cpu().numpy()
    kc, vc = k_b.float().cpu().numpy(), v_b.float().cpu().numpy()
    for i in range(len(lens)):
        for g in range(hkv):
            pos = idx_h[g, ref.cu_k[i]:ref.cu_k[i + 1]]
            assert np.array_equal(kc[g, ref.cu_k[i]:ref.cu_k[i + 1]], x.k[i][g][pos])
            assert np.array_equal(vc[g, ref.cu_k[i]:ref.cu_k[i + 1]], x.v[i][g][pos])
    if max(lens) <= 8192:                           # without a score buffer
        k_c, v_c = torch.zeros_like(k_b), torch.zeros_like(v_b)
        idx_c = torch.full((hkv, m), -1, dtype=torch.int32, device="cuda")
        S.samkv_score_select_gather(caches, q_tok, q_loc, ratio, n_sink, n_local, None, idx_c, None, k_c, v_c, ws)
        assert torch.equal(idx_a, idx_c) and torch.equal(k_a, k_c) and torch.equal(v_a, v_c)


def test_layers_stacked_as_heads(S):
    """Several layers in one call: every document's cache holds all layers as [(layer, KV head)][L][d] and the Q
    tensors likewise.  The library sees 3 x Hkv KV heads; each layer's slice must agree with the oracle run on that
    layer alone (query head h reads KV head h / G, which never leaves its layer)."""
    import torch
    lens, hq, hkv, d, ratio = [300, 77, 513], 4, 2, 128, 0.3
    xs = [synth.make_small(90 + l, "bf16", lens, hq, hkv, d, 5, 7) for l in range(3)]
    refs = [H.oracle_front(x, ratio) for x in xs]
    m = int(refs[0].cu_k[-1])
    cat = lambda arrs, axis=0: H.to_dev(np.concatenate(arrs, axis=axis), "bf16")
    k = [cat([x.k[i] for x in xs]) for i in range(len(lens))]
    v = [cat([x.v[i] for x in xs]) for i in range(len(lens))]
    caches = S.Caches(k, v, 3 * hq)
    q_tok = cat([x.q_tok for x in xs])
    q_loc = cat([x.q_loc for x in xs], axis=1)
    q_rec_np = [synth.make_q_rec(x.workload, l, m) for l, x in enumerate(xs)]
    q_rec = cat(q_rec_np)
    scale = 1.0 / math.sqrt(d)
    buf = S.alloc_layer_buffers(caches, xs[0].workload.n_q_tok, ratio)
    S.hot_path(caches, q_tok, q_loc, q_rec, ratio, scale, buf)
    torch.cuda.synchronize()
    sg, idx = buf.scores.cpu().numpy().astype(np.float64), buf.idx.cpu().numpy()
    cu = np.concatenate([[0], np.cumsum(lens)])
    G = hq // hkv
    for l, (x, ref) in enumerate(zip(xs, refs)):
        bound = H.score_error_bound(x, ref)
        for i in range(len(lens)):
            assert np.all(np.abs(sg[l * hkv:(l + 1) * hkv, cu[i]:cu[i + 1]] - ref.scores[i]) <= bound[i]), (l, i)
        kv, qh = slice(l * hkv, (l + 1) * hkv), slice(l * hq, (l + 1) * hq)
        H.compare_kept_sets(idx[kv], ref)
        H.check_chained(x, ref, idx[kv], buf.k_c[kv].float().cpu().numpy(), buf.v_c[kv].float().cpu().numpy(),
                        buf.rec_out[qh].cpu().numpy(), buf.rec_lse[qh].cpu().numpy(), buf.q_out[qh].cpu().numpy(),
                        buf.q_lse[qh].cpu().numpy(), q_rec_np[l], scale, f"layer {l}")


def test_measuring_kernels_run_and_leave_their_sink_alone(S):
    """The micro-kernels that bench.py quotes ceilings from: the copy copies, the others touch nothing."""
    import torch
    sink = torch.full((4,), 7.0, device="cuda")
    for pattern in (0, 1, 2):
        assert S.samkv_peak_mfma_bf16_data(sink, 8, 4, pattern) == 8 * 4 * 4 * 16 * 32768
    assert S.samkv_peak_mfma_bf16(sink, 8, 4) == 8 * 4 * 4 * 16 * 32768
    src = torch.arange(1 << 16, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    assert S.samkv_peak_copy(src, dst) == 2 * src.numel() * 4
    assert S.samkv_peak_read(src, sink) == src.numel() * 4
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    assert torch.equal(sink.cpu(), torch.full((4,), 7.0))
    with pytest.raises(S.SamKVError):
        S.samkv_peak_mfma_bf16_data(sink, 8, 4, 5)

