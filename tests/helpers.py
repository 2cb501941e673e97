"""Shared pieces of the GPU parity tests: upload helpers, oracle pipeline, comparison rules."""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional

import numpy as np

from oracle import samkv_oracle as O
from paper_2508_11661_amd import synth

# tolerances (written here once, used by every parity test)
F32_REL = 1e-4        # attention outputs, float32 path: relative error
BF16_ABS = 2e-2       # attention outputs, bf16 path: absolute error
TIE_MARGIN = 1e-3     # kept sets may differ only at scores within this margin of the k-th score


def torch_dtype(name: str):
    import torch
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def to_dev(a: np.ndarray, dtype: str):
    """float32 array whose values are exact in `dtype` -> device tensor of that dtype."""
    from paper_2508_11661_amd import samkv
    return samkv.upload(a, dtype)


@dataclass
class OracleRun:
    q_hat: np.ndarray
    scores: List[np.ndarray]      # per document [Hkv, L_i]
    idx: np.ndarray               # [Hkv, M]
    cu_k: np.ndarray
    k_c: np.ndarray
    v_c: np.ndarray


def oracle_front(x: synth.LayerInputs, ratio: float, n_sink: int = 0, n_local: int = 0,
                 use_bias: bool = True) -> OracleRun:
    """score -> select -> gather with the fp64 oracle."""
    n = len(x.k)
    q_hat = O.personalized_query(x.q_tok, x.q_loc if use_bias else None, n)
    scores = O.score(q_hat, x.k)
    idx, cu_k = O.select(scores, ratio, n_sink, n_local)
    k_c, v_c = O.gather(x.k, x.v, idx, cu_k)
    return OracleRun(q_hat, scores, idx, cu_k, k_c, v_c)


def score_error_bound(x: synth.LayerInputs, ref: OracleRun) -> List[np.ndarray]:
    """Per-score bound on float32 accumulation error: 2e-5 * |q~| * |K row| + 1e-6 (Cauchy-Schwarz on
    d * eps32 * sum |q_c k_c|, d <= 128, plus the float32 rounding of the query vector itself)."""
    hq = ref.q_hat.shape[1]
    out = []
    for i, k in enumerate(x.k):
        hkv = k.shape[0]
        qt = ref.q_hat[i].reshape(hkv, hq // hkv, -1).mean(axis=1)
        qn = np.linalg.norm(qt, axis=1)[:, None]
        kn = np.linalg.norm(k.astype(np.float64), axis=2)
        out.append(2e-5 * qn * kn + 1e-6)
    return out


def compare_kept_sets(idx_gpu: np.ndarray, ref: OracleRun, n_sink: int = 0, n_local: int = 0):
    """Kept sets must equal the oracle's except at positions whose oracle score lies within
    TIE_MARGIN * max(1, |tau|) of tau, the oracle's k-th largest score of the row.
    Returns (number of rows that differ inside the margin, list of KV heads whose sets are identical)."""
    hkv = idx_gpu.shape[0]
    assert idx_gpu.shape == ref.idx.shape
    in_margin_rows = 0
    clean_heads = []
    for g in range(hkv):
        clean = True
        for i, s in enumerate(ref.scores):
            a, b = int(ref.cu_k[i]), int(ref.cu_k[i + 1])
            got, want = idx_gpu[g, a:b], ref.idx[g, a:b]
            L = s.shape[1]
            assert np.all(np.diff(got) > 0), "positions must be strictly ascending"
            assert got.min() >= 0 and got.max() < L
            if np.array_equal(got, want):
                continue
            clean = False
            forced = set(range(n_sink)) | set(range(L - n_local, L))
            free = [p for p in want if p not in forced]
            tau = min(s[g, p] for p in free)
            margin = TIE_MARGIN * max(1.0, abs(tau))
            for p in set(got.tolist()) ^ set(want.tolist()):
                assert abs(s[g, p] - tau) <= margin, (
                    f"head {g} document {i}: position {p} (score {s[g, p]}) differs outside the tie margin of {tau}")
            in_margin_rows += 1
        if clean:
            clean_heads.append(g)
    return in_margin_rows, clean_heads


def check_attention(out_gpu: np.ndarray, lse_gpu: np.ndarray, out_ref: np.ndarray, lse_ref: np.ndarray,
                    dtype: str, what: str = "") -> float:
    """Attention parity rule.  float32: per (head, row) max-norm relative error <= 1e-4, and
    element-wise |err| <= 1e-4 * max(|O*|, rms of that output row) (an element much smaller than its
    row carries the row's rounding error, not its own).  bf16: absolute error <= 2e-2.  Same bars for LSE."""
    out_gpu = out_gpu.astype(np.float64)
    lse_gpu = lse_gpu.astype(np.float64)
    assert np.all(np.isfinite(out_gpu)) and np.all(np.isfinite(lse_gpu)), f"{what}: non-finite output"
    err = np.abs(out_gpu - out_ref)
    if dtype == "f32":
        row_ref = np.maximum(np.abs(out_ref).max(axis=-1), 1e-6)
        rel = err.max(axis=-1) / row_ref
        assert rel.max() <= F32_REL, f"{what}: row-relative error {rel.max():.3e} > {F32_REL}"
        row_rms = np.sqrt((out_ref ** 2).mean(axis=-1, keepdims=True))
        elem = err / np.maximum(np.maximum(np.abs(out_ref), row_rms), 1e-6)
        assert elem.max() <= F32_REL, f"{what}: element-wise relative error {elem.max():.3e}"
        lerr = np.abs(lse_gpu - lse_ref) / np.maximum(1.0, np.abs(lse_ref))
        assert lerr.max() <= F32_REL, f"{what}: LSE error {lerr.max():.3e}"
        return float(rel.max())
    assert err.max() <= BF16_ABS, f"{what}: absolute error {err.max():.3e} > {BF16_ABS}"
    lerr = np.abs(lse_gpu - lse_ref)
    assert lerr.max() <= BF16_ABS, f"{what}: LSE absolute error {lerr.max():.3e}"
    return float(err.max())


def upload_caches(x: synth.LayerInputs):
    from paper_2508_11661_amd import samkv
    dt = x.workload.dtype
    k = [to_dev(a, dt) for a in x.k]
    v = [to_dev(a, dt) for a in x.v]
    return samkv.Caches(k, v, x.workload.n_q_heads)


def check_chained(x: synth.LayerInputs, ref: OracleRun, idx_gpu: np.ndarray, k_c: np.ndarray, v_c: np.ndarray,
                  rec_out: np.ndarray, rec_lse: np.ndarray, q_out: np.ndarray, q_lse: np.ndarray, q_rec: np.ndarray,
                  scale: float, what: str = ""):
    """Results of the calls chained on the GPU, every head.  The kept sets have been compared under the tie-margin
    rule; from there on the oracle continues with the GPU's OWN kept set (identical to the oracle's wherever no score
    sat inside the margin), so a near-tie can neither hide a head nor cascade: the compacted cache must hold
    bit-exact copies of the rows at the kept positions, and both attentions over it must meet the attention bar.
    Returns (max error recompute, max error query)."""
    dt = x.workload.dtype
    k_own, v_own = O.gather(x.k, x.v, idx_gpu, ref.cu_k)
    assert np.array_equal(k_c, k_own) and np.array_equal(v_c, v_own), f"{what}: compacted cache"
    o_ref, l_ref = O.attention(q_rec, k_own, v_own, scale, True)
    e_rec = check_attention(rec_out, rec_lse, o_ref, l_ref, dt, f"{what} chained recompute")
    o_ref, l_ref = O.attention(x.q_tok, k_own, v_own, scale, False)
    e_q = check_attention(q_out, q_lse, o_ref, l_ref, dt, f"{what} chained query")
    return e_rec, e_q
