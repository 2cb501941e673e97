"""Attention entry points on shapes chosen to reach every kernel variant and every prologue/tail case:
one, two, three and four key tiles, ragged last tiles, many heads with few rows (the 8-wave asynchronous
kernel is picked by row-tile count), key chunks with a merge, both head dims and both dtypes."""
import math

import numpy as np
import pytest

from oracle import samkv_oracle as O
from paper_2508_11661_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _data(seed, dtype, hq, hkv, rows, m, d):
    rng = np.random.default_rng(seed)
    q = synth.round_to_dtype(rng.standard_normal((hq, rows, d), dtype=np.float32) * 1.5, dtype)
    k = synth.round_to_dtype(rng.standard_normal((hkv, m, d), dtype=np.float32) * 1.5, dtype)
    v = synth.round_to_dtype(rng.standard_normal((hkv, m, d), dtype=np.float32) * 2.0, dtype)
    return q, k, v


def _rows(m, n, seed):
    if m <= n:
        return None
    rng = np.random.default_rng(seed)
    fixed = [0, 1, 31, 32, 63, 64, 65, 127, 128, 255, 256, 257, m - 2, m - 1]
    return np.unique(np.clip(np.concatenate([fixed, rng.integers(0, m, size=n)]), 0, m - 1))


@pytest.mark.parametrize("dtype,d,hq,hkv,m", [
    ("bf16", 128, 1024, 8, 1), ("bf16", 128, 1024, 8, 63), ("bf16", 128, 1024, 8, 64), ("bf16", 128, 1024, 8, 65),
    ("bf16", 128, 1024, 8, 129), ("bf16", 128, 1024, 8, 200), ("bf16", 128, 512, 8, 300), ("bf16", 128, 64, 8, 4200),
    ("bf16", 128, 128, 16, 2049), ("bf16", 64, 64, 8, 4200), ("bf16", 64, 8, 2, 700), ("bf16", 128, 8, 8, 700),
    ("f32", 128, 4, 2, 150), ("f32", 64, 8, 1, 97),
    # few workgroups and more than 256 rows: the variant whose two key groups split every 128-key step
    ("bf16", 128, 32, 8, 1540), ("bf16", 128, 4, 2, 257), ("bf16", 128, 4, 4, 321), ("bf16", 64, 16, 4, 449),
    ("bf16", 128, 2, 1, 385), ("bf16", 64, 2, 2, 2048),
    # enough row tiles for the asynchronous-load kernel, whose workgroups hold the 2, 4 or 8 query heads of a KV head:
    # two heads per KV head, and a KV head count that is not a multiple of eight
    ("bf16", 128, 48, 24, 2300), ("bf16", 128, 40, 10, 2600),
])
def test_recompute_attention_shapes(dtype, d, hq, hkv, m):
    import torch
    from paper_2508_11661_amd import samkv as S
    q, k, v = _data(m + hq, dtype, hq, hkv, m, m, d)
    scale = 1.0 / math.sqrt(d)
    out = torch.full((hq, m, d), float("nan"), device="cuda")
    lse = torch.full((hq, m), float("nan"), device="cuda")
    ws = torch.empty((S.samkv_workspace_bytes(1, hq, hkv, d, 1, m),), dtype=torch.uint8, device="cuda")
    S.samkv_recompute_attn(H.to_dev(q, dtype), H.to_dev(k, dtype), H.to_dev(v, dtype), scale, out, lse, ws)
    rows = _rows(m, 12 if hq * m > 20000 else m, seed=m)
    heads = list(range(hq)) if hq <= 64 else sorted({0, 1, hq // 2, hq - 1} | set(range(0, hq, max(1, hq // 24))))
    G = hq // hkv
    kv = sorted({h // G for h in heads})
    remap = {g: n for n, g in enumerate(kv)}
    o_ref = np.empty((len(heads), m if rows is None else len(rows), d))
    l_ref = np.empty((len(heads), m if rows is None else len(rows)))
    for n, h in enumerate(heads):          # one query head at a time against its own KV head
        o, l = O.attention(q[h:h + 1], k[h // G:h // G + 1], v[h // G:h // G + 1], scale, True, rows=rows)
        o_ref[n], l_ref[n] = o[0], l[0]
    sel = slice(None) if rows is None else torch.from_numpy(rows).cuda()
    got_o = out[heads][:, sel].cpu().numpy()
    got_l = lse[heads][:, sel].cpu().numpy()
    H.check_attention(got_o, got_l, o_ref, l_ref, dtype, f"recompute {dtype} d={d} hq={hq} m={m}")
    assert torch.isfinite(out).all() and torch.isfinite(lse).all()


@pytest.mark.parametrize("dtype,d,hq,hkv,lq,m", [
    ("bf16", 128, 32, 2, 64, 1), ("bf16", 128, 32, 2, 64, 64), ("bf16", 128, 32, 2, 64, 65), ("bf16", 128, 32, 2, 64, 130),
    ("bf16", 128, 32, 2, 64, 1000), ("bf16", 128, 32, 2, 64, 3001), ("bf16", 128, 64, 8, 256, 5000),
    ("bf16", 128, 8, 8, 3, 777), ("bf16", 64, 16, 2, 130, 999), ("f32", 128, 4, 2, 5, 333), ("f32", 64, 8, 8, 40, 2100),
])
def test_query_attention_shapes(dtype, d, hq, hkv, lq, m):
    import torch
    from paper_2508_11661_amd import samkv as S
    q, k, v = _data(m + lq, dtype, hq, hkv, lq, m, d)
    scale = 1.0 / math.sqrt(d)
    out = torch.full((hq, lq, d), float("nan"), device="cuda")
    lse = torch.full((hq, lq), float("nan"), device="cuda")
    ws = torch.empty((S.samkv_workspace_bytes(1, hq, hkv, d, lq, m),), dtype=torch.uint8, device="cuda")
    S.samkv_query_attn(H.to_dev(q, dtype), H.to_dev(k, dtype), H.to_dev(v, dtype), scale, out, lse, ws)
    rows = _rows(lq, 24 if hq * lq * m > 3e7 else lq, seed=m)
    rows = None if rows is None else rows[rows < lq]
    o_ref, l_ref = O.attention(q, k, v, scale, False, rows=rows)
    sel = slice(None) if rows is None else torch.from_numpy(rows).cuda()
    H.check_attention(out[:, sel].cpu().numpy(), lse[:, sel].cpu().numpy(), o_ref, l_ref, dtype,
                      f"query {dtype} d={d} hq={hq} lq={lq} m={m}")
    assert torch.isfinite(out).all() and torch.isfinite(lse).all()


@pytest.mark.parametrize("dtype,d,hq,hkv,lq,m", [
    ("bf16", 128, 32, 8, 32, 1540), ("bf16", 128, 8, 2, 1, 100), ("bf16", 64, 8, 8, 70, 333), ("bf16", 128, 64, 8, 256, 3000),
    ("f32", 64, 8, 2, 16, 156), ("f32", 128, 4, 4, 33, 65),
])
def test_query_attention_with_self_tail(dtype, d, hq, hkv, lq, m):
    import torch
    from paper_2508_11661_amd import samkv as S
    q, k, v = _data(7 * m + lq, dtype, hq, hkv, lq, m, d)
    _, ks, vs = _data(11 * m + lq, dtype, hq, hkv, lq, lq, d)
    scale = 1.0 / math.sqrt(d)
    out = torch.full((hq, lq, d), float("nan"), device="cuda")
    lse = torch.full((hq, lq), float("nan"), device="cuda")
    ws = torch.empty((S.samkv_workspace_bytes(1, hq, hkv, d, lq, m),), dtype=torch.uint8, device="cuda")
    S.samkv_query_attn_self(H.to_dev(q, dtype), H.to_dev(k, dtype), H.to_dev(v, dtype), H.to_dev(ks, dtype),
                            H.to_dev(vs, dtype), scale, out, lse, ws)
    heads = list(range(hq)) if hq * lq <= 4096 else [0, 1, hq // 2, hq - 1]
    G = hq // hkv
    o_ref = np.empty((len(heads), lq, d))
    l_ref = np.empty((len(heads), lq))
    for n, h in enumerate(heads):
        g = h // G
        o, l = O.attention_with_self(q[h:h + 1], k[g:g + 1], v[g:g + 1], ks[g:g + 1], vs[g:g + 1], scale)
        o_ref[n], l_ref[n] = o[0], l[0]
    H.check_attention(out[heads].cpu().numpy(), lse[heads].cpu().numpy(), o_ref, l_ref, dtype, "query+self")
    assert torch.isfinite(out).all()


@pytest.mark.parametrize("dtype,d,hq,hkv,lq,m", [
    # one launch for both attentions, in every workgroup shape the causal problem can select (the query attention
    # takes the same shape and walks all keys in one chunk): 128 rows x two key groups, four waves, the asynchronous
    # kernel with KV heads in groups of 8 / in three such groups / not a multiple of 8, eight waves at d = 64
    ("bf16", 128, 32, 8, 32, 1540), ("bf16", 128, 8, 2, 5, 200), ("bf16", 128, 4, 4, 1, 1),
    ("bf16", 128, 64, 8, 256, 4200), ("bf16", 128, 48, 24, 7, 2300), ("bf16", 128, 40, 10, 33, 2600),
    ("bf16", 64, 64, 8, 130, 4200), ("bf16", 64, 16, 4, 64, 449), ("bf16", 64, 8, 2, 3, 100),
    ("bf16", 128, 32, 8, 300, 700),      # more query rows than one workgroup holds, short cache
    ("f32", 64, 8, 2, 16, 156),          # float32: the call runs the two kernels one after the other
])
def test_both_attentions_in_one_call(dtype, d, hq, hkv, lq, m):
    """samkv_recompute_query_attn against the two separate calls and the oracle: the recompute attention runs the same
    arithmetic in the same order (same bits); the query attention walks the keys in one chunk instead of several
    (same definition, different rounding), so it is held against the oracle and must stay within the bar of the
    separate call's result as well."""
    import torch
    from paper_2508_11661_amd import samkv as S
    q, k, v = _data(3 * m + hq, dtype, hq, hkv, m, m, d)
    qt = synth.round_to_dtype(np.random.default_rng(5 * m + lq).standard_normal((hq, lq, d), dtype=np.float32) * 1.5, dtype)
    scale = 1.0 / math.sqrt(d)
    dev = [H.to_dev(x, dtype) for x in (q, qt, k, v)]
    nan = lambda *shape: torch.full(shape, float("nan"), device="cuda")
    ro, rl, qo, ql = nan(hq, m, d), nan(hq, m), nan(hq, lq, d), nan(hq, lq)
    ro2, rl2, qo2, ql2 = nan(hq, m, d), nan(hq, m), nan(hq, lq, d), nan(hq, lq)
    ws = torch.empty((S.samkv_workspace_bytes(1, hq, hkv, d, lq, m),), dtype=torch.uint8, device="cuda")
    S.samkv_recompute_query_attn(dev[0], dev[1], dev[2], dev[3], scale, ro, rl, qo, ql, ws)
    S.samkv_recompute_attn(dev[0], dev[2], dev[3], scale, ro2, rl2, ws)
    S.samkv_query_attn(dev[1], dev[2], dev[3], scale, qo2, ql2, ws)
    torch.cuda.synchronize()
    assert torch.equal(ro, ro2) and torch.equal(rl, rl2), "recompute attention: pair call and separate call differ"
    if dtype == "f32":
        assert torch.equal(qo, qo2) and torch.equal(ql, ql2)
    else:
        assert (qo - qo2).abs().max().item() <= H.BF16_ABS and (ql - ql2).abs().max().item() <= H.BF16_ABS
    rows = _rows(lq, 24 if hq * lq * m > 3e7 else lq, seed=m)
    rows = None if rows is None else rows[rows < lq]
    o_ref, l_ref = O.attention(qt, k, v, scale, False, rows=rows)
    sel = slice(None) if rows is None else torch.from_numpy(rows).cuda()
    H.check_attention(qo[:, sel].cpu().numpy(), ql[:, sel].cpu().numpy(), o_ref, l_ref, dtype,
                      f"query in the pair call {dtype} d={d} hq={hq} lq={lq} m={m}")
    assert torch.isfinite(qo).all() and torch.isfinite(ql).all() and torch.isfinite(ro).all()


@pytest.mark.parametrize("log2_scale", [-40, -20, 0, 7, 30, 100])
@pytest.mark.parametrize("causal", [True, False])
def test_bf16_attention_value_magnitudes(log2_scale, causal):
    """The bf16 kernels multiply the weights with a half-precision copy of V that is scaled per KV head by a power of
    two: outputs must follow V's magnitude exactly (values far outside the half-precision range included), heads
    with very different magnitudes must not disturb each other, an all-zero head gives zeros, and a few values 2^20
    below the head's maximum still count."""
    import torch
    from paper_2508_11661_amd import samkv as S
    hq, hkv, m, d, rows = 8, 4, 300, 128, 300 if causal else 40
    q, k, v = _data(900 + log2_scale, "bf16", hq, hkv, rows, m, d)
    mag = np.array([2.0 ** log2_scale, 1.0, 2.0 ** -log2_scale, 0.0], np.float32)      # per KV head; exact in bf16
    v = v * mag[:, None, None]
    v[1, ::3] *= np.float32(2.0 ** -20)           # rows far below the head's maximum
    scale = 1.0 / math.sqrt(d)
    out = torch.full((hq, rows, d), float("nan"), device="cuda")
    lse = torch.full((hq, rows), float("nan"), device="cuda")
    ws = torch.empty((S.samkv_workspace_bytes(1, hq, hkv, d, rows, m),), dtype=torch.uint8, device="cuda")
    args = (H.to_dev(q, "bf16"), H.to_dev(k, "bf16"), H.to_dev(v, "bf16"), scale, out, lse, ws)
    S.samkv_recompute_attn(*args) if causal else S.samkv_query_attn(*args)
    o_ref, l_ref = O.attention(q, k, v, scale, causal)
    got_o, got_l = out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got_o)) and np.abs(got_l - l_ref).max() <= H.BF16_ABS
    G = hq // hkv
    for h in range(hq):
        s = float(mag[h // G])
        err = np.abs(got_o[h] - o_ref[h]).max()
        assert err <= H.BF16_ABS * s, f"head {h} (values x {s:g}): error {err:.3e}"
