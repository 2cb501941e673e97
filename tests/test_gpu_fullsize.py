"""GPU parity at the full sizes of the named workloads, through the same calls and buffers that
bench.py times.  Scores, kept sets and the compacted cache are compared in full; attention rows are
sampled (first row, last row, rows at document boundaries, seeded random rows), each sampled row
computed by the oracle on its own."""
import math

import numpy as np
import pytest

from oracle import samkv_oracle as O
from paper_2508_11661_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _sample_rows(cu_k, m, n_random, seed):
    rng = np.random.default_rng(seed)
    rows = {0, m - 1}
    for b in cu_k[1:-1]:
        rows.update((int(b) - 1, int(b)))
    rows.update(int(r) for r in rng.integers(0, m, size=n_random))
    return np.array(sorted(rows))


def _full_size(name, layer, ratio, n_rows_rec, n_rows_q):
    import torch
    from paper_2508_11661_amd import samkv as S
    w = synth.WORKLOADS[name]
    x = synth.make_layer(w, layer)
    ref = H.oracle_front(x, ratio)
    m = int(ref.cu_k[-1])
    caches = H.upload_caches(x)
    q_tok, q_loc = H.to_dev(x.q_tok, w.dtype), H.to_dev(x.q_loc, w.dtype)
    q_rec_np = synth.make_q_rec(w, layer, m)
    q_rec = H.to_dev(q_rec_np, w.dtype)
    scale = 1.0 / math.sqrt(w.head_dim)
    buf = S.alloc_layer_buffers(caches, w.n_q_tok, ratio)
    S.hot_path(caches, q_tok, q_loc, q_rec, ratio, scale, buf)
    torch.cuda.synchronize()
    assert buf.cu_k == ref.cu_k.tolist()

    # scores, everywhere
    sg = buf.scores.cpu().numpy().astype(np.float64)
    bound = H.score_error_bound(x, ref)
    cu = np.concatenate([[0], np.cumsum(x.lens)])
    for i in range(len(x.k)):
        assert np.all(np.abs(sg[:, cu[i]:cu[i + 1]] - ref.scores[i]) <= bound[i]), f"score, document {i}"
    # kept sets, everywhere (tie-margin rule); compacted cache of the heads that match exactly
    in_margin, clean = H.compare_kept_sets(buf.idx.cpu().numpy(), ref)
    assert len(clean) >= max(1, w.n_kv_heads // 2), f"only {len(clean)} KV heads reproduce the oracle's kept set"
    kc, vc = buf.k_c.float().cpu().numpy(), buf.v_c.float().cpu().numpy()
    for g in clean:
        assert np.array_equal(kc[g], ref.k_c[g]) and np.array_equal(vc[g], ref.v_c[g]), f"gather, KV head {g}"
    heads = [h for h in range(w.n_q_heads) if h // w.group in clean]

    # recompute attention on sampled rows, query attention on sampled (or all) rows
    rows = _sample_rows(ref.cu_k, m, n_rows_rec, seed=layer)
    o_ref, l_ref = O.attention(q_rec_np[heads], ref.k_c[clean], ref.v_c[clean], scale, True, rows=rows)
    got_o = buf.rec_out[heads][:, torch.from_numpy(rows).cuda()].cpu().numpy()
    got_l = buf.rec_lse[heads][:, torch.from_numpy(rows).cuda()].cpu().numpy()
    e_rec = H.check_attention(got_o, got_l, o_ref, l_ref, w.dtype, f"{name} recompute")
    q_rows = np.arange(w.n_q_tok) if n_rows_q >= w.n_q_tok else np.unique(
        np.concatenate([[0, w.n_q_tok - 1], np.random.default_rng(7).integers(0, w.n_q_tok, size=n_rows_q)]))
    o_ref, l_ref = O.attention(x.q_tok[heads], ref.k_c[clean], ref.v_c[clean], scale, False, rows=q_rows)
    got_o = buf.q_out[heads][:, torch.from_numpy(q_rows).cuda()].cpu().numpy()
    got_l = buf.q_lse[heads][:, torch.from_numpy(q_rows).cuda()].cpu().numpy()
    e_q = H.check_attention(got_o, got_l, o_ref, l_ref, w.dtype, f"{name} query")
    # the selection exactly as bench.py launches it (no score buffer), and the two separate calls: same bits
    idx2 = torch.full_like(buf.idx, -1)
    S.samkv_score_select(caches, q_tok, q_loc, ratio, 0, 0, None, idx2, None, buf.ws)
    assert torch.equal(idx2, buf.idx)
    sc3, idx3 = torch.empty_like(buf.scores), torch.full_like(buf.idx, -1)
    S.samkv_score(caches, q_tok, q_loc, sc3, buf.ws)
    S.samkv_topk_select(sc3, caches, ratio, 0, 0, idx3, None, buf.ws)
    assert torch.equal(sc3, buf.scores) and torch.equal(idx3, buf.idx)
    print(f"{name} layer {layer} ratio {ratio}: M={m}, rows differing inside the tie margin={in_margin}, "
          f"KV heads exact={len(clean)}/{w.n_kv_heads}, max |err| recompute={e_rec:.2e} query={e_q:.2e}")
    return m


@pytest.mark.parametrize("layer", [0, 31])
def test_config3_llama_32layers_one_layer(layer):
    assert _full_size("llama3_8b_32layers", layer, 0.15, 24, 64) == 6160


@pytest.mark.parametrize("ratio,m", [(0.05, 4120), (0.25, 20480)])
def test_config4_mistral_sweep(ratio, m):
    assert _full_size("mistral_7b_sweep", 0, ratio, 16, 24) == m


def test_config5_large_cache_stress():
    assert _full_size("large_cache_stress", 0, 0.15, 8, 8) == 39360
