"""Pins of the fp64 oracle against things other than itself: hand-worked values, closed forms,
invariants, brute force and library routines.  CPU only."""
import itertools
import math

import numpy as np
import pytest

from oracle import samkv_oracle as O
from paper_2508_11661_amd import synth


def rng(seed):
    return np.random.default_rng(seed)


def paper_constants():
    """tests/golden/paper_constants.txt: the few numbers the paper prints, each with the place it prints it."""
    import os
    out = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = (x.strip() for x in line.split("="))
            out[k] = float(v)
    return out


# ------------------------------------------------------------------ Eq. 1 (personalized query)
def test_pooled_query_hand_values():
    # two tokens (1,2) and (3,6) -> mean (2,4)   [Sec. 3.1: mean pooling over the sequence dimension]
    q = np.array([[[1.0, 2.0], [3.0, 6.0]]])
    assert np.array_equal(O.pooled_query(q), [[2.0, 4.0]])


def test_eq1_single_document_has_no_bias():
    r = rng(0)
    q_tok = r.standard_normal((3, 5, 8))
    q_loc = r.standard_normal((1, 3, 4, 8))
    qh = O.personalized_query(q_tok, q_loc, 1)
    assert np.allclose(qh[0], q_tok.mean(axis=1), rtol=0, atol=1e-15)


def test_eq1_no_local_cache_means_generic_query():
    r = rng(1)
    q_tok = r.standard_normal((2, 7, 4))
    qh = O.personalized_query(q_tok, None, 3)
    for i in range(3):
        assert np.allclose(qh[i], q_tok.mean(axis=1), atol=1e-15)


def test_eq1_two_documents_by_hand_d2():
    # Q_que = (1, 0); local query of document 2 = (1, 1): cos = 1/sqrt(2)
    # Q^_1 = (1,0) + |cos| (1,1) / (2-1) = (1 + 0.70710678, 0.70710678)
    # local query of document 1 = (-1, 1): cos = -1/sqrt(2), weight is the absolute value
    # Q^_2 = (1,0) + 0.70710678 (-1, 1) = (0.29289322, 0.70710678)
    q_tok = np.array([[[1.0, 0.0]]])
    q_loc = np.array([[[[-1.0, 1.0]]], [[[1.0, 1.0]]]])
    qh = O.personalized_query(q_tok, q_loc, 2)
    c = 1.0 / math.sqrt(2.0)
    assert np.allclose(qh[0, 0], [1.0 + c, c], atol=1e-15)
    assert np.allclose(qh[1, 0], [1.0 - c, c], atol=1e-15)


def test_eq1_three_documents_normalised_by_d_minus_1():
    # Q_que = (2, 0).  local queries: doc0 (0, 3) [cos 0], doc1 (4, 0) [cos 1], doc2 (3, 4) [cos 0.6]
    # Q^_0 = (2,0) + (1*(4,0) + 0.6*(3,4)) / 2 = (2 + 2.9, 1.2)
    # Q^_1 = (2,0) + (0*(0,3) + 0.6*(3,4)) / 2 = (2.9, 1.2)
    # Q^_2 = (2,0) + (0*(0,3) + 1*(4,0)) / 2  = (4, 0)
    q_tok = np.array([[[2.0, 0.0]]])
    q_loc = np.array([[[[0.0, 3.0]]], [[[4.0, 0.0]]], [[[3.0, 4.0]]]])
    qh = O.personalized_query(q_tok, q_loc, 3)
    assert np.allclose(qh[:, 0], [[4.9, 1.2], [2.9, 1.2], [4.0, 0.0]], atol=1e-14)


def test_eq1_local_cache_rows_are_mean_pooled():
    # the local Q cache of a document is several rows; rows (2,0) and (0,2) pool to (1,1)
    q_tok = np.array([[[1.0, 0.0]]])
    q_loc = np.array([[[[5.0, 5.0], [5.0, 5.0]]], [[[2.0, 0.0], [0.0, 2.0]]]])
    qh = O.personalized_query(q_tok, q_loc, 2)
    c = 1.0 / math.sqrt(2.0)
    assert np.allclose(qh[0, 0], [1.0 + c, c], atol=1e-15)


def test_eq1_orthogonal_local_queries_leave_query_unchanged():
    r = rng(2)
    d = 16
    q_tok = r.standard_normal((2, 3, d))
    que = q_tok.mean(axis=1)
    q_loc = r.standard_normal((4, 2, 5, d))
    # remove from every row its component along Q_que: the pooled vector is then orthogonal too
    for h in range(2):
        u = que[h] / np.linalg.norm(que[h])
        q_loc[:, h] -= (q_loc[:, h] @ u)[..., None] * u
    qh = O.personalized_query(q_tok, q_loc, 4)
    assert np.allclose(qh, que[None], atol=1e-12)


@pytest.mark.parametrize("c", [0.5, 2.0, -0.25])
def test_eq1_collinear_local_queries_scale_the_query(c):
    r = rng(3)
    q_tok = r.standard_normal((3, 4, 8))
    que = q_tok.mean(axis=1)
    n = 5
    q_loc = np.broadcast_to((c * que)[None, :, None, :], (n, 3, 2, 8)).copy()
    qh = O.personalized_query(q_tok, q_loc, n)
    # |cos| = 1 for every other document: Q^ = Q_que + (1/(n-1)) * (n-1) * c Q_que
    assert np.allclose(qh, (1.0 + c) * que[None], atol=1e-12)


def test_eq1_invariant_to_order_of_other_documents():
    r = rng(4)
    q_tok = r.standard_normal((2, 3, 8))
    q_loc = r.standard_normal((4, 2, 3, 8))
    qh = O.personalized_query(q_tok, q_loc, 4)
    perm = [0, 3, 1, 2]
    qh_p = O.personalized_query(q_tok, q_loc[perm], 4)
    assert np.allclose(qh_p[0], qh[0], atol=1e-13)         # document 0 kept its place
    assert np.allclose(qh_p[1], qh[3], atol=1e-13)


def test_eq1_zero_norm_local_query_gets_zero_weight():
    q_tok = np.array([[[1.0, 2.0]]])
    q_loc = np.zeros((2, 1, 1, 2))
    qh = O.personalized_query(q_tok, q_loc, 2)
    assert np.array_equal(qh[0, 0], [1.0, 2.0]) and np.all(np.isfinite(qh))


def test_generated_local_queries_have_small_cosine():
    # Sec. 3.1 reports the range cos(Q_que, Q_loc) usually stays in; the synthetic caches land there
    bound = paper_constants()["cos_query_local_max"]
    x = synth.make_layer(synth.WORKLOADS["llama3_8b_layer"])
    que = O.pooled_query(x.q_tok)
    loc = O.local_query(x.q_loc)
    cos = [O.abs_cos(que[h], loc[j, h]) for j in range(loc.shape[0]) for h in range(que.shape[0])]
    assert np.median(cos) < bound and np.quantile(cos, 0.9) < 1.5 * bound


# ------------------------------------------------------------------ scoring
def test_score_matches_einsum_and_is_mean_over_group():
    r = rng(5)
    n, hq, hkv, d = 3, 6, 2, 8
    qh = r.standard_normal((n, hq, d))
    k = [r.standard_normal((hkv, L, d)) for L in (5, 9, 4)]
    s = O.score(qh, k)
    for i in range(n):
        ref = np.einsum("ghc,gtc->gt", qh[i].reshape(hkv, hq // hkv, d), k[i]) / (hq // hkv)
        assert np.allclose(s[i], ref, rtol=1e-13, atol=1e-13)


def test_score_hand_values():
    # one KV head, two query heads (1,0) and (0,1): score of key (3,5) = (3 + 5)/2 = 4
    qh = np.array([[[1.0, 0.0], [0.0, 1.0]]])
    k = [np.array([[[3.0, 5.0], [-2.0, 0.0]]])]
    assert np.array_equal(O.score(qh, k)[0], [[4.0, -1.0]])


def test_score_single_head_single_token_is_matvec():
    r = rng(6)
    k = [r.standard_normal((1, 11, 4))]
    q_tok = r.standard_normal((1, 1, 4))
    s = O.score(O.personalized_query(q_tok, None, 1), k)[0]
    assert np.allclose(s[0], k[0][0] @ q_tok[0, 0], atol=1e-14)


def test_score_linearity_in_the_bias_terms():
    # <Q^_i, K> = <Q_que, K> + 1/(D-1) sum_j w_j <Q_loc_j, K>: three dot products computed apart
    r = rng(7)
    n, hq, d = 3, 2, 8
    q_tok = r.standard_normal((hq, 4, d))
    q_loc = r.standard_normal((n, hq, 3, d))
    k = [r.standard_normal((hq, 6, d)) for _ in range(n)]
    s = O.score(O.personalized_query(q_tok, q_loc, n), k)
    que, loc = q_tok.mean(axis=1), q_loc.mean(axis=2)
    for i in range(n):
        for h in range(hq):
            expect = k[i][h] @ que[h]
            for j in range(n):
                if j != i:
                    w = abs(que[h] @ loc[j, h]) / (np.linalg.norm(que[h]) * np.linalg.norm(loc[j, h]))
                    expect = expect + w * (k[i][h] @ loc[j, h]) / (n - 1)
            assert np.allclose(s[i][h], expect, atol=1e-12)


def test_collinear_bias_keeps_the_same_set():
    x = synth.make_small(3, "f32", [64, 80], 4, 2, 16, 5, 4)
    que = O.pooled_query(x.q_tok)
    q_loc = np.broadcast_to((0.7 * que)[None, :, None, :], (2, 4, 4, 16)).copy()
    a, _ = O.select(O.score(O.personalized_query(x.q_tok, None, 2), x.k), 0.25)
    b, _ = O.select(O.score(O.personalized_query(x.q_tok, q_loc, 2), x.k), 0.25)
    assert np.array_equal(a, b)


# ------------------------------------------------------------------ selection
def test_kept_count_values_of_the_configurations():
    assert [O.kept_count(L, 0.15) for L in (256, 1024, 2048, 4096)] == [39, 154, 308, 615]
    assert [O.kept_count(2048, r) for r in (0.05, 0.10, 0.15, 0.25)] == [103, 205, 308, 512]
    assert O.kept_count(100, 1.0) == 100 and O.kept_count(1, 0.01) == 1 and O.kept_count(7, 0.5) == 4
    assert O.kept_count(20, 0.1) == 2 and O.kept_count(40, 0.05) == 2      # exact products do not round up


def test_select_row_brute_force_all_subsets_tiny():
    r = rng(8)
    for trial in range(20):
        L = int(r.integers(3, 9))
        k = int(r.integers(1, L + 1))
        s = r.standard_normal(L)
        best = max(itertools.combinations(range(L), k), key=lambda c: sum(s[list(c)]))
        assert list(O.select_row(s, k)) == sorted(best)


def test_select_row_properties_and_ties():
    r = rng(9)
    s = r.standard_normal(300)
    k = 45
    idx = O.select_row(s, k)
    assert len(idx) == k and len(set(idx.tolist())) == k
    assert np.all(np.diff(idx) > 0) and idx.min() >= 0 and idx.max() < 300
    dropped = np.setdiff1d(np.arange(300), idx)
    assert s[idx].min() >= s[dropped].max()
    # ties go to the lower position
    t = np.array([1.0, 5.0, 5.0, 5.0, 0.0, 5.0])
    assert list(O.select_row(t, 2)) == [1, 2]
    assert list(O.select_row(t, 3)) == [1, 2, 3]
    assert list(O.select_row(np.zeros(6), 4)) == [0, 1, 2, 3]
    # hand example: scores (0.1, 0.9, 0.3, 0.8, 0.2), keep 2 -> positions 1 and 3
    assert list(O.select_row(np.array([0.1, 0.9, 0.3, 0.8, 0.2]), 2)) == [1, 3]


def test_select_row_forced_initial_and_local_positions():
    # Sec. 3.2: initial and local positions are kept without sparsification
    s = np.array([-9.0, -8.0, 1.0, 7.0, 3.0, 6.0, -7.0, -6.0])
    assert list(O.select_row(s, 5, n_sink=2, n_local=2)) == [0, 1, 3, 6, 7]
    assert list(O.select_row(s, 4, n_sink=2, n_local=2)) == [0, 1, 6, 7]
    # forced positions with a high score are not counted twice
    s2 = np.array([9.0, 0.0, 1.0, 2.0, 8.0])
    assert list(O.select_row(s2, 3, n_sink=1, n_local=1)) == [0, 3, 4]


def test_select_sizes_order_and_full_budget_identity():
    r = rng(10)
    lens = [17, 40, 9]
    scores = [r.standard_normal((3, L)) for L in lens]
    idx, cu = O.select(scores, 0.15)
    assert list(cu) == [0, 3, 9, 11]            # ceil(2.55), ceil(6.0), ceil(1.35)
    assert idx.shape == (3, 11)
    for i, L in enumerate(lens):
        for g in range(3):
            seg = idx[g, cu[i]:cu[i + 1]]
            assert np.all(np.diff(seg) > 0) and seg.min() >= 0 and seg.max() < L
            order = np.argsort(-scores[i][g], kind="stable")[: len(seg)]
            assert sorted(order.tolist()) == seg.tolist()
    idx1, cu1 = O.select(scores, 1.0)
    assert list(cu1) == [0, 17, 57, 66]
    for g in range(3):
        assert idx1[g].tolist() == sum((list(range(L)) for L in lens), [])


def test_select_maps_under_permutation_of_tokens():
    r = rng(11)
    s = r.standard_normal(50)
    perm = r.permutation(50)
    a = O.select_row(s, 9)
    b = O.select_row(s[perm], 9)
    assert sorted(perm[b].tolist()) == a.tolist()


def test_planted_tokens_are_recalled():
    # statistical sanity of the synthetic workload, not parity: +2 sigma planted keys, 10 % planted, 15 % kept
    x = synth.make_layer(synth.WORKLOADS["tiny_f32"])
    s = O.score(O.personalized_query(x.q_tok, None, len(x.k)), x.k)
    idx, cu = O.select(s, 0.15)
    hits = total = 0
    for i in range(len(x.k)):
        for g in range(idx.shape[0]):
            hits += np.isin(x.planted_pos[i], idx[g, cu[i]:cu[i + 1]]).sum()
            total += len(x.planted_pos[i])
    assert 0.5 < hits / total <= 1.0


# ------------------------------------------------------------------ compaction
def test_gather_equals_fancy_indexing_and_full_budget_is_concatenation():
    r = rng(12)
    lens = [6, 11, 3]
    k = [r.standard_normal((2, L, 4)).astype(np.float32) for L in lens]
    v = [r.standard_normal((2, L, 4)).astype(np.float32) for L in lens]
    idx, cu = O.select([r.standard_normal((2, L)) for L in lens], 0.4)
    k_c, v_c = O.gather(k, v, idx, cu)
    for i in range(3):
        for g in range(2):
            sl = slice(cu[i], cu[i + 1])
            assert k_c[g, sl].tobytes() == k[i][g][idx[g, sl]].tobytes()
            assert v_c[g, sl].tobytes() == v[i][g][idx[g, sl]].tobytes()
    idx1, cu1 = O.select([r.standard_normal((2, L)) for L in lens], 1.0)
    k_c, v_c = O.gather(k, v, idx1, cu1)
    assert k_c.tobytes() == np.concatenate(k, axis=1).tobytes()
    assert v_c.tobytes() == np.concatenate(v, axis=1).tobytes()


def test_gather_q_uses_the_kv_heads_positions():
    r = rng(19)
    lens = [7, 5]
    q = [r.standard_normal((4, L, 3)).astype(np.float32) for L in lens]       # 4 query heads, 2 KV heads
    idx, cu = O.select([r.standard_normal((2, L)) for L in lens], 0.5)
    out = O.gather_q(q, idx, cu)
    assert out.shape == (4, int(cu[-1]), 3)
    for i in range(2):
        sl = slice(cu[i], cu[i + 1])
        for h in range(4):
            assert out[h, sl].tobytes() == q[i][h][idx[h // 2, sl]].tobytes()


# ------------------------------------------------------------------ attention
def _sdpa(q, k, v, scale, causal):
    import torch
    import torch.nn.functional as F
    hq, hkv = q.shape[0], k.shape[0]
    kk = torch.from_numpy(np.repeat(k, hq // hkv, axis=0))[None]
    vv = torch.from_numpy(np.repeat(v, hq // hkv, axis=0))[None]
    o = F.scaled_dot_product_attention(torch.from_numpy(q)[None], kk, vv, is_causal=causal, scale=scale)
    return o[0].numpy()


@pytest.mark.parametrize("causal", [False, True])
def test_attention_matches_library_sdpa_fp64(causal):
    r = rng(13)
    hq, hkv, M, d = 6, 2, 37, 16
    k = r.standard_normal((hkv, M, d))
    v = r.standard_normal((hkv, M, d))
    q = r.standard_normal((hq, M if causal else 5, d)) * 2.0
    scale = 1.0 / math.sqrt(d)
    o, lse = O.attention(q, k, v, scale, causal)
    assert np.allclose(o, _sdpa(q, k, v, scale, causal), rtol=1e-12, atol=1e-12)


def test_attention_hand_values():
    # one query, two keys with logits 0 and ln 3 -> weights 1/4, 3/4; values 4 and 8 -> 7; lse = ln 4
    q = np.array([[[1.0]]])
    k = np.array([[[0.0], [math.log(3.0)]]])
    v = np.array([[[4.0], [8.0]]])
    o, lse = O.attention(q, k, v, 1.0, False)
    assert abs(o[0, 0, 0] - 7.0) < 1e-14 and abs(lse[0, 0] - math.log(4.0)) < 1e-14
    # the scale multiplies the logits: scale 2 -> logits 0, ln 9 -> weights 0.1, 0.9 -> 7.6
    o, lse = O.attention(q, k, v, 2.0, False)
    assert abs(o[0, 0, 0] - 7.6) < 1e-14 and abs(lse[0, 0] - math.log(10.0)) < 1e-14


@pytest.mark.parametrize("causal", [False, True])
def test_attention_invariants(causal):
    r = rng(14)
    hq, hkv, M, d = 4, 2, 23, 8
    k = r.standard_normal((hkv, M, d))
    v = r.standard_normal((hkv, M, d))
    q = r.standard_normal((hq, M, d))
    scale = 0.3
    o, lse = O.attention(q, k, v, scale, causal)
    # softmax rows sum to one: rebuild the weights from LSE
    for h in range(hq):
        for p in range(M):
            last = p + 1 if causal else M
            w = np.exp(scale * (k[h // 2, :last] @ q[h, p]) - lse[h, p])
            assert abs(w.sum() - 1.0) < 1e-12
            assert np.allclose(w @ v[h // 2, :last], o[h, p], atol=1e-12)
    # V == 1 -> O == 1
    o1, _ = O.attention(q, k, np.ones_like(v), scale, causal)
    assert np.allclose(o1, 1.0, atol=1e-14)
    # Q == 0 -> uniform weights: (prefix) mean of V, LSE = log(count)
    o0, l0 = O.attention(np.zeros_like(q), k, v, scale, causal)
    for p in range(M):
        last = p + 1 if causal else M
        assert np.allclose(o0[0, p], v[0, :last].mean(axis=0), atol=1e-13)
        assert abs(l0[0, p] - math.log(last)) < 1e-13
    # outputs stay inside the range of the values they average
    assert np.all(o <= v.max(axis=1)[np.repeat(np.arange(hkv), 2)][:, None, :] + 1e-12)
    assert np.all(o >= v.min(axis=1)[np.repeat(np.arange(hkv), 2)][:, None, :] - 1e-12)


def test_recompute_is_causal_across_documents_and_includes_self():
    r = rng(15)
    hq, hkv, M, d = 2, 1, 12, 4
    k = r.standard_normal((hkv, M, d))
    v = r.standard_normal((hkv, M, d))
    q = r.standard_normal((hq, M, d))
    o, _ = O.attention(q, k, v, 0.5, True)
    assert np.allclose(o[:, 0], v[0, 0][None], atol=1e-14)          # row 0 sees only itself
    k2, v2 = k.copy(), v.copy()
    k2[:, 7:] += 3.0
    v2[:, 7:] -= 5.0
    o2, _ = O.attention(q, k2, v2, 0.5, True)
    assert np.array_equal(o2[:, :7], o[:, :7])                       # later keys never reach earlier rows
    assert not np.allclose(o2[:, 7], o[:, 7])                        # but a row does see its own key
    # a row in the second "document" (positions 6..11) does see the first one
    k3 = k.copy()
    k3[:, 2] += 4.0
    o3, _ = O.attention(q, k3, v, 0.5, True)
    assert not np.allclose(o3[:, 9], o[:, 9])


def test_query_attention_invariant_to_cache_order_and_single_key():
    r = rng(16)
    k = r.standard_normal((2, 9, 4))
    v = r.standard_normal((2, 9, 4))
    q = r.standard_normal((4, 3, 4))
    o, lse = O.attention(q, k, v, 0.5, False)
    perm = r.permutation(9)
    o2, lse2 = O.attention(q, k[:, perm], v[:, perm], 0.5, False)
    assert np.allclose(o, o2, atol=1e-13) and np.allclose(lse, lse2, atol=1e-13)
    o1, l1 = O.attention(q, k[:, :1], v[:, :1], 0.5, False)
    assert np.allclose(o1, np.repeat(v[:, :1], 2, axis=0), atol=1e-15)
    assert np.allclose(l1[0], 0.5 * (q[0] @ k[0, 0]), atol=1e-14)


def test_attention_row_subset_matches_full():
    r = rng(17)
    k = r.standard_normal((1, 20, 4))
    v = r.standard_normal((1, 20, 4))
    q = r.standard_normal((2, 20, 4))
    o, lse = O.attention(q, k, v, 0.5, True)
    os_, ls = O.attention(q, k, v, 0.5, True, rows=[0, 7, 19])
    assert np.array_equal(os_, o[:, [0, 7, 19]]) and np.array_equal(ls, lse[:, [0, 7, 19]])


def test_full_budget_pipeline_is_dense_attention_over_concatenated_caches():
    # budget 100 %: every token kept, compacted cache = concatenation, query attention = the
    # "Reuse" baseline of the Evaluation section (dense attention over the concatenated caches)
    x = synth.make_small(5, "f32", [9, 14, 6], 4, 2, 8, 3, 2)
    n = len(x.k)
    s = O.score(O.personalized_query(x.q_tok, x.q_loc, n), x.k)
    idx, cu = O.select(s, 1.0)
    k_c, v_c = O.gather(x.k, x.v, idx, cu)
    scale = 1.0 / math.sqrt(8)
    o, _ = O.attention(x.q_tok, k_c, v_c, scale, False)
    kk = np.concatenate(x.k, axis=1).astype(np.float64)
    vv = np.concatenate(x.v, axis=1).astype(np.float64)
    assert np.allclose(o, _sdpa(x.q_tok.astype(np.float64), kk, vv, scale, False), atol=1e-12)
    q_rec = rng(18).standard_normal((4, 29, 8))
    o, _ = O.attention(q_rec, k_c, v_c, scale, True)
    assert np.allclose(o, _sdpa(q_rec, kk, vv, scale, True), atol=1e-12)


# ------------------------------------------------------------------ cache update (Eq. 4)
def test_kv_update_hand_values_and_closed_forms():
    # old (1,0), new (1,1): theta = 1/sqrt(2); result = theta (1,1) + (1-theta) (1,0) = (1, theta)
    th = 1.0 / math.sqrt(2.0)
    out = O.kv_update(np.array([[[1.0, 0.0]]]), np.array([[[1.0, 1.0]]]), True)
    assert np.allclose(out, [[[1.0, th]]], atol=1e-15)
    r = rng(20)
    old = r.standard_normal((2, 5, 8))
    new = r.standard_normal((2, 5, 8))
    assert np.array_equal(O.kv_update(old, new, False), new)                      # overwrite
    assert np.allclose(O.kv_update(old, old, True), old, atol=1e-14)              # new == old: theta = 1, unchanged
    assert np.allclose(O.kv_update(old, 2.5 * old, True), 2.5 * old, atol=1e-13)  # parallel: theta = 1, new wins
    assert np.allclose(O.kv_update(old, -old, True), 3.0 * old, atol=1e-13)       # theta = -1: -new + 2 old = 3 old
    perp = new - (np.einsum("gmc,gmc->gm", new, old) / np.einsum("gmc,gmc->gm", old, old))[..., None] * old
    assert np.allclose(O.kv_update(old, perp, True), old, atol=1e-12)             # orthogonal: theta = 0, old stays
    # the cosine is per cached token and head: changing one row leaves every other row's result alone
    new2 = new.copy()
    new2[1, 3] *= -4.0
    a, b = O.kv_update(old, new, True), O.kv_update(old, new2, True)
    mask = np.ones((2, 5), bool)
    mask[1, 3] = False
    assert np.array_equal(a[mask], b[mask]) and not np.allclose(a[1, 3], b[1, 3])
    # zero rows: theta = 1, the new row is taken
    z = np.zeros((1, 1, 4))
    assert np.array_equal(O.kv_update(z, np.ones((1, 1, 4)), True), np.ones((1, 1, 4)))
    assert np.array_equal(O.kv_update(np.ones((1, 1, 4)), z, True), z)


def test_generated_recomputed_rows_have_cosine_near_the_reported_value():
    x = synth.make_layer(synth.WORKLOADS["llama3_8b_layer"])
    old = np.concatenate(x.k, axis=1)[:, :500]
    new = synth.make_recomputed_rows(x.workload, 0, old, x.sigma_k, 0)
    cos = np.einsum("gmc,gmc->gm", new, old) / (np.linalg.norm(new, axis=2) * np.linalg.norm(old, axis=2))
    assert abs(np.median(cos) - paper_constants()["fusion_cos_typical"]) < 0.05     # the fusion weight Sec. 3.3 reports


# ------------------------------------------------------------------ query prefill with its own K/V
def test_attention_with_self_matches_masked_library_sdpa_and_hand_values():
    import torch
    import torch.nn.functional as F
    r = rng(21)
    hq, hkv, M, lq, d = 4, 2, 11, 5, 8
    k_c, v_c = r.standard_normal((hkv, M, d)), r.standard_normal((hkv, M, d))
    k_s, v_s = r.standard_normal((hkv, lq, d)), r.standard_normal((hkv, lq, d))
    q = r.standard_normal((hq, lq, d))
    o, lse = O.attention_with_self(q, k_c, v_c, k_s, v_s, 0.4)
    kk = torch.from_numpy(np.repeat(np.concatenate([k_c, k_s], axis=1), 2, axis=0))[None]
    vv = torch.from_numpy(np.repeat(np.concatenate([v_c, v_s], axis=1), 2, axis=0))[None]
    mask = torch.ones(lq, M + lq, dtype=torch.bool)
    mask[:, M:] = torch.tril(torch.ones(lq, lq, dtype=torch.bool))
    ref = F.scaled_dot_product_attention(torch.from_numpy(q)[None], kk, vv, attn_mask=mask, scale=0.4)[0].numpy()
    assert np.allclose(o, ref, atol=1e-12)
    # token 0 with an empty... one cached key (logit 0) and its own key (logit ln 3): weights 1/4, 3/4
    o, lse = O.attention_with_self(np.array([[[1.0]]]), np.array([[[0.0]]]), np.array([[[4.0]]]),
                                   np.array([[[math.log(3.0)]]]), np.array([[[8.0]]]), 1.0)
    assert abs(o[0, 0, 0] - 7.0) < 1e-14 and abs(lse[0, 0] - math.log(4.0)) < 1e-14
    # merging the two partial attentions by log-sum-exp gives the same result (the identity the kernels use)
    oc, lc = O.attention(q, k_c, v_c, 0.4, False)
    os_, ls = O.attention(q, k_s, v_s, 0.4, True)
    o, lse = O.attention_with_self(q, k_c, v_c, k_s, v_s, 0.4)
    tot = np.logaddexp(lc, ls)
    assert np.allclose(lse, tot, atol=1e-12)
    assert np.allclose(o, np.exp(lc - tot)[..., None] * oc + np.exp(ls - tot)[..., None] * os_, atol=1e-12)


# ------------------------------------------------------------------ dynamic Top-P (Eq. 2, Eq. 3)
def test_top_p_hand_values_and_edge_cases():
    # one layer, five documents: (anc, max, min)
    #   (4, 10, 0)  -> (10 - 4) / (10 - 0) = 0.6
    #   (10, 10, 0) -> anchor equals max: inside (min, max], numerator 0 -> 0
    #   (0, 10, 0)  -> anchor equals min: outside the half-open interval -> 0
    #   (12, 10, 0) -> anchor above max -> 0
    #   (5, 5, 5)   -> empty interval -> 0
    anc = np.array([[4.0, 10.0, 0.0, 12.0, 5.0]])
    mx = np.array([[10.0, 10.0, 10.0, 10.0, 5.0]])
    mn = np.array([[0.0, 0.0, 0.0, 0.0, 5.0]])
    assert np.allclose(O.top_p(anc, mx, mn), [0.6, 0.0, 0.0, 0.0, 0.0], atol=1e-15)
    # Eq. 3: mean over layers; 0.6 and 0.2 -> 0.4; a layer that falls in the "otherwise" branch counts as 0
    anc = np.array([[4.0], [8.0], [11.0]])
    mx = np.array([[10.0], [10.0], [10.0]])
    mn = np.array([[0.0], [0.0], [0.0]])
    assert np.allclose(O.top_p(anc[:2], mx[:2], mn[:2]), [0.4], atol=1e-15)
    assert np.allclose(O.top_p(anc, mx, mn), [0.8 / 3.0], atol=1e-15)
    # the direction the paper argues for: P grows with s_max, shrinks with s_anc and with s_min
    base = O.top_p([[4.0]], [[10.0]], [[0.0]])[0]
    assert O.top_p([[4.0]], [[12.0]], [[0.0]])[0] > base
    assert O.top_p([[5.0]], [[10.0]], [[0.0]])[0] < base
    assert O.top_p([[4.0]], [[10.0]], [[1.0]])[0] > base - 1.0 and O.top_p([[4.0]], [[10.0]], [[-5.0]])[0] < base


def test_kept_count_mid_and_select_v():
    assert O.kept_count_mid(1000, 0.0, 64, 128) == 192
    assert O.kept_count_mid(1000, 1.0, 64, 128) == 1000
    assert O.kept_count_mid(1000, 0.25, 64, 128) == 192 + 202          # ceil(0.25 * 808)
    assert O.kept_count_mid(100, 0.5, 64, 128) == 100                  # forced positions cover the document
    assert O.kept_count_mid(20, 0.1, 0, 0) == 2 and O.kept_count_mid(20, 0.0, 0, 0) == 0
    r = rng(22)
    scores = [r.standard_normal((2, L)) for L in (30, 12, 50)]
    idx, cu = O.select_v(scores, [0.2, 0.0, 0.5], n_sink=2, n_local=3)
    assert list(cu) == [0, 5 + 5, 10 + 5, 15 + 5 + 23]                 # forced 5 each + ceil(0.2*25)=5, 0, ceil(0.5*45)=23
    for g in range(2):
        seg = idx[g, :10]
        assert set([0, 1, 27, 28, 29]) <= set(seg.tolist())
        mid = [p for p in seg if 2 <= p < 27]
        best = np.argsort(-scores[0][g, 2:27], kind="stable")[:5] + 2
        assert sorted(mid) == sorted(best.tolist())
        assert idx[g, 10:15].tolist() == [0, 1, 9, 10, 11]             # a document with P = 0 keeps only the forced ones


# ------------------------------------------------------------------ block-level retrieval (Sec. 3.2)
def test_block_scores_hand_values_and_linearity():
    # one head, d = 1, keys 1..5 in blocks of 2 -> representatives 1.5, 3.5, 5; Q^ = 2 -> scores 3, 7, 10
    k = [np.arange(1.0, 6.0).reshape(1, 5, 1)]
    assert np.array_equal(O.block_scores(np.full((1, 1, 1), 2.0), k, 2)[0], [[3.0, 7.0, 10.0]])
    # the inner product is linear: the score of the mean key is the mean of the token scores (ragged last block,
    # grouped heads); O.score on the tokens is an independent path to the same number
    r = rng(90)
    lens, hq, hkv, d, block = (37, 64, 5), 4, 2, 8, 16
    ks = [r.standard_normal((hkv, L, d)) for L in lens]
    q_hat = r.standard_normal((3, hq, d))
    tok = O.score(q_hat, ks)
    for i, b in enumerate(O.block_scores(q_hat, ks, block)):
        assert b.shape == (hkv, -(-lens[i] // block))
        for n in range(b.shape[1]):
            want = tok[i][:, n * block:(n + 1) * block].mean(axis=1)
            assert np.allclose(b[:, n], want, rtol=1e-12, atol=1e-12)


def test_block_select_hand_values_and_token_granularity_special_case():
    # 10 tokens in blocks of 3: blocks 0..3, the last holds token 9 only.  First and last block forced, half of the
    # two middle blocks -> one more, the better of blocks 1 (score 1) and 2 (score 5).
    b = [np.array([[0.0, 1.0, 5.0, -3.0], [9.0, 2.0, 1.0, 9.0]])]
    idx, cu_k = O.block_select(b, [10], 3, [0.5], 1, 1)
    assert cu_k.tolist() == [0, 7]
    assert idx.tolist() == [[0, 1, 2, 6, 7, 8, 9], [0, 1, 2, 3, 4, 5, 9]]
    # p = 0 keeps only the forced blocks, p = 1 everything
    assert O.block_select(b, [10], 3, [0.0], 1, 1)[0].tolist() == [[0, 1, 2, 9]] * 2
    assert O.block_select(b, [10], 3, [1.0], 1, 1)[0].tolist() == [list(range(10))] * 2
    # blocks of one token are the token-level selection
    r = rng(91)
    sc = [r.standard_normal((3, L)) for L in (17, 40)]
    a = O.block_select(sc, [17, 40], 1, [0.3, 0.6], 2, 3)
    w = O.select_v(sc, [0.3, 0.6], 2, 3)
    assert np.array_equal(a[0], w[0]) and np.array_equal(a[1], w[1])
    # heads that would keep different token counts are refused (short last block neither forced nor dropped by all)
    with pytest.raises(AssertionError):
        O.block_select([np.array([[0.0, 1.0, 5.0, -3.0], [9.0, 2.0, 1.0, 9.0]])], [10], 3, [0.5], 1, 0)


def test_block_filter_hand_values_and_reductions():
    # Two documents, blocks of 2 tokens, first and last block forced, every middle block retrieved (p = 1).
    #   document 0: 5 blocks, scores 9 1 5 3 9 -> candidates 1, 2, 3 with min-max normalised scores 0, 1, 0.5
    #   document 1: 4 blocks, scores 0 10 20 0 -> candidates 1, 2 with normalised scores 0, 1
    # 5 candidates over 2 documents -> 3 survive: block 2 of each document (1.0) and block 3 of document 0 (0.5).
    b = [np.array([[9.0, 1, 5, 3, 9]]), np.array([[0.0, 10, 20, 0]])]
    got = O.block_filter(b, [10, 8], 2, [1.0, 1.0], 1, 1)
    assert got.tolist() == [[0, 1, 4, 5, 6, 7, 8, 9, 10, 11, 14, 15, 16, 17]]
    # the scale of a document's scores does not matter (that is what the normalisation is for) ...
    b2 = [b[0] * 1000.0 - 7.0, b[1] * 0.001 + 3.0]
    assert np.array_equal(O.block_filter(b2, [10, 8], 2, [1.0, 1.0], 1, 1), got)
    # ... a single document keeps everything it retrieved (C / 1 = C): the filter reduces to block_select
    r = rng(92)
    bs = [r.standard_normal((3, 12))]
    idx, cu = O.block_select(bs, [12 * 8 - 3], 8, [0.4], 1, 2)
    assert np.array_equal(O.block_filter(bs, [12 * 8 - 3], 8, [0.4], 1, 2), idx)
    # ... and with several documents: forced blocks always survive, the survivors are a subset of what the
    # per-document selection retrieved, and their number is forced + ceil(C / N) blocks
    lens, block = [200, 64, 333, 1000], 16
    bs = [r.standard_normal((2, -(-L // block))) for L in lens]
    p = [0.5, 0.3, 0.0, 0.2]
    idx, cu = O.block_select(bs, lens, block, p, 1, 2)
    got = O.block_filter(bs, lens, block, p, 1, 2)
    cu_len = np.concatenate([[0], np.cumsum(lens)])
    n_cand = sum(O.kept_count_mid(-(-L // block), pi, 1, 2) - 3 for L, pi in zip(lens, p))
    forced_tokens = sum(16 + (L - (-(-L // block) - 2) * block) for L in lens)
    assert got.shape[1] == forced_tokens + -(-n_cand // 4) * block
    for g in range(2):
        retrieved = set()
        for i in range(4):
            retrieved |= {int(cu_len[i] + t) for t in idx[g, cu[i]:cu[i + 1]]}
            forced = set(range(cu_len[i], cu_len[i] + 16)) | set(range(cu_len[i] + (-(-lens[i] // block) - 2) * block, cu_len[i + 1]))
            assert forced <= set(got[g].tolist())
        assert set(got[g].tolist()) <= retrieved
        assert np.all(np.diff(got[g]) > 0)


def test_gather_global_matches_per_document_gather():
    r = rng(93)
    lens = [9, 4, 17]
    k = [r.standard_normal((2, L, 4)) for L in lens]
    v = [r.standard_normal((2, L, 4)) for L in lens]
    idx, cu = O.select([r.standard_normal((2, L)) for L in lens], 0.5)
    cu_len = np.concatenate([[0], np.cumsum(lens)])
    gidx = idx.copy()
    for i in range(3):
        gidx[:, cu[i]:cu[i + 1]] += cu_len[i]
    k_c, v_c = O.gather(k, v, idx, cu)
    assert np.array_equal(O.gather_global(k, gidx), k_c) and np.array_equal(O.gather_global(v, gidx), v_c)
    q = [r.standard_normal((6, L, 4)) for L in lens]
    assert np.array_equal(O.gather_global(q, gidx, group=3), O.gather_q(q, idx, cu))


# ------------------------------------------------------------------ the constants the paper prints
def test_paper_constants_meet_oracle_defaults_and_workloads():
    c = paper_constants()
    # Setup: 64-token blocks, 1 initial and 2 local blocks always kept -> the oracle's defaults force exactly those
    block, ni, nl = int(c["block_size"]), int(c["initial_blocks"]), int(c["local_blocks"])
    L = 20 * block + 7                                   # 21 blocks, the last one 7 tokens long
    idx, cu = O.block_select([np.zeros((1, 21))], [L], block, [0.0])
    assert cu.tolist() == [0, ni * block + (nl - 1) * block + 7]
    assert idx[0].tolist() == list(range(block)) + list(range(19 * block, L))
    # Table 1: the budget of the named workloads (15 %) is the paper's sequence ratio to within a point, and every
    # kept token is recomputed, which is what its recomputation ratio says to within a point
    for w in synth.WORKLOADS.values():
        if 0.15 in w.ratios:
            kept = sum(O.kept_count(n, 0.15) for n in w.lens) / sum(w.lens) * 100
            assert abs(kept - c["sequence_ratio_percent"]) < 1.0 and abs(kept - c["recompute_ratio_percent"]) < 1.0
