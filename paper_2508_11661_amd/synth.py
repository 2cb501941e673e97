"""Seeded synthetic multi-document caches, shaped like the paper's RAG workloads.

This module only *draws inputs*: per-document K/V caches, the user query's Q
states, each document's local Q cache and the Q states of the kept tokens.  It
holds none of the method's arithmetic (no pooling of the method, no Eq. 1, no
scoring, no selection, no attention) and imports neither the CPU oracle nor the
HIP binding; both consume the arrays produced here.

The paper evaluates on LongBench multi-document QA prompts (Evaluation, Setup).
Those datasets and the model weights are not available, so the caches below
stand in for them by shape and by value distribution only: Gaussian keys and
values with per-channel scales spread log-uniformly over [0.5, 4] (a few
dominant "outlier" channels, as real K caches have), a seeded fraction of
positions whose keys are pushed towards the query direction so that a relevant
set exists to be found, and key/value rows duplicated between documents so that
the inter-document consensus of Sec. 3.1 has something to act on.

Every array is float32 whose values are exactly representable in the workload's
storage dtype (float32 itself, or bfloat16 after one round-to-nearest-even on
the host), so the GPU path and the fp64 oracle read identical numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

BASE_SEED = 0x5A4D4B56


@dataclass(frozen=True)
class Workload:
    """One named configuration (shapes and distribution knobs)."""

    name: str
    cfg_id: int
    dtype: str                 # "f32" or "bf16": storage type of K, V and all Q tensors
    n_layers: int
    n_ctx: int                 # D in the paper: number of retrieved documents
    ctx_len: int               # tokens per document
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_q_tok: int               # user-query tokens
    ratios: Tuple[float, ...]  # budget ratios the workload is run at
    planted: float             # fraction of positions shifted towards the query
    dup: float                 # fraction of positions overwritten by rows of other documents
    w_loc: int                 # rows of each document's local Q cache
    planted_beta: Optional[Tuple[float, float]] = None  # per-document fraction ~ Beta(a, b)
    layer_outliers: bool = False

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def lens(self) -> List[int]:
        return [self.ctx_len] * self.n_ctx


WORKLOADS: Dict[str, Workload] = {
    w.name: w
    for w in (
        Workload("tiny_f32", 1, "f32", 1, 4, 256, 8, 2, 64, 16, (0.15,), 0.10, 0.0, 16),
        Workload("llama3_8b_layer", 2, "bf16", 1, 10, 1024, 32, 8, 128, 32, (0.15,), 0.08, 0.05, 128),
        Workload("llama3_8b_32layers", 3, "bf16", 32, 20, 2048, 32, 8, 128, 64, (0.15,), 0.08, 0.05, 128,
                 layer_outliers=True),
        Workload("mistral_7b_sweep", 4, "bf16", 1, 40, 2048, 32, 8, 128, 128, (0.05, 0.10, 0.15, 0.25),
                 0.08, 0.05, 128),
        Workload("large_cache_stress", 5, "bf16", 1, 64, 4096, 64, 8, 128, 256, (0.15,), 0.08, 0.05, 128,
                 planted_beta=(0.5, 5.0)),
    )
}
BY_ID = {w.cfg_id: w for w in WORKLOADS.values()}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return round_to_bf16(x)
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError(dtype)


def _rng(w: Workload, layer: int, tensor: int, sub: int = 0) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([BASE_SEED + w.cfg_id, layer, tensor, sub]))


# tensor ids for the seed streams
_T_SCALE, _T_DIR, _T_Q, _T_K, _T_V, _T_PLANT, _T_DUP, _T_QLOC, _T_QREC = range(9)


@dataclass
class LayerInputs:
    """Inputs of one layer of one workload (all float32, dtype-exact values)."""

    workload: Workload
    layer: int
    lens: List[int]
    k: List[np.ndarray]            # per document [Hkv, L_i, d]
    v: List[np.ndarray]            # per document [Hkv, L_i, d]
    q_tok: np.ndarray              # [Hq, Lq, d]
    q_loc: np.ndarray              # [N, Hq, Wloc, d]
    planted_pos: List[np.ndarray]  # per document: sorted positions whose keys were shifted
    dup_pos: List[np.ndarray]      # per document: positions overwritten by another document's rows
    dup_src: List[np.ndarray]      # per document: [n_dup, 2] = (source document, source position)
    sigma_k: np.ndarray = field(repr=False, default=None)  # [Hkv, d]
    sigma_v: np.ndarray = field(repr=False, default=None)  # [Hkv, d]


def _channel_scales(w: Workload, layer: int) -> Tuple[np.ndarray, np.ndarray]:
    rng = _rng(w, layer, _T_SCALE)
    lo, hi = np.log(0.5), np.log(4.0)
    sk = np.exp(rng.uniform(lo, hi, size=(w.n_kv_heads, w.head_dim)))
    sv = np.exp(rng.uniform(lo, hi, size=(w.n_kv_heads, w.head_dim)))
    if w.layer_outliers:
        # Deeper layers get stronger outlier channels, in K (and in Q, which shares K's scales) and in V,
        # each tensor with its own four seeded channels per KV head.
        for g in range(w.n_kv_heads):
            ch = rng.choice(w.head_dim, size=4, replace=False)
            sk[g, ch] *= 1.0 + layer / 8.0
        for g in range(w.n_kv_heads):
            ch = rng.choice(w.head_dim, size=4, replace=False)
            sv[g, ch] *= 1.0 + layer / 8.0
    return sk, sv


def _query_directions(w: Workload, layer: int) -> np.ndarray:
    """Unit direction per query head; heads of one KV group share a common component."""
    rng = _rng(w, layer, _T_DIR)
    base = rng.standard_normal((w.n_kv_heads, w.head_dim))
    own = rng.standard_normal((w.n_q_heads, w.head_dim))
    u = np.repeat(base, w.group, axis=0) + 0.5 * own
    return u / np.linalg.norm(u, axis=1, keepdims=True)


def make_layer(w: Workload, layer: int = 0, lens: Optional[List[int]] = None) -> LayerInputs:
    """Draw the caches and query tensors of one layer.  `lens` overrides the document lengths."""
    lens = list(w.lens if lens is None else lens)
    n_ctx, hkv, hq, d, g = len(lens), w.n_kv_heads, w.n_q_heads, w.head_dim, w.group
    sk, sv = _channel_scales(w, layer)
    u = _query_directions(w, layer)

    # noise-free query direction per query head and its KV-group average
    qbar_h = np.sqrt(d) * np.repeat(sk, g, axis=0) * u               # [Hq, d]
    qbar_g = qbar_h.reshape(hkv, g, d).mean(axis=1)                   # [Hkv, d]
    sigma_s = np.sqrt(((qbar_g * sk) ** 2).sum(axis=1))               # background score spread per group
    shift = (2.0 * sigma_s / (qbar_g ** 2).sum(axis=1))[:, None] * qbar_g   # raises <qbar_g, K> by 2 sigma_s

    rq = _rng(w, layer, _T_Q)
    z = rq.standard_normal((hq, w.n_q_tok, d), dtype=np.float32)
    q_tok = (np.repeat(sk, g, axis=0)[:, None, :] * (np.sqrt(d) * u[:, None, :] + z)).astype(np.float32)

    ks: List[np.ndarray] = []
    vs: List[np.ndarray] = []
    planted_pos: List[np.ndarray] = []
    rp = _rng(w, layer, _T_PLANT)
    sk32, sv32 = sk.astype(np.float32), sv.astype(np.float32)
    for i, L in enumerate(lens):
        kz = _rng(w, layer, _T_K, i).standard_normal((hkv, L, d), dtype=np.float32)
        kz *= sk32[:, None, :]
        vz = _rng(w, layer, _T_V, i).standard_normal((hkv, L, d), dtype=np.float32)
        vz *= sv32[:, None, :]
        frac = w.planted if w.planted_beta is None else float(rp.beta(*w.planted_beta))
        n_pl = min(L, int(round(frac * L)))
        pos = np.sort(rp.choice(L, size=n_pl, replace=False)) if n_pl else np.zeros(0, np.int64)
        if n_pl:
            kz[:, pos, :] += shift.astype(np.float32)[:, None, :]
        ks.append(kz)
        vs.append(vz)
        planted_pos.append(pos)

    # cross-document duplicates: rows of other documents (as drawn above) overwrite a few positions
    dup_pos: List[np.ndarray] = [np.zeros(0, np.int64) for _ in lens]
    dup_src: List[np.ndarray] = [np.zeros((0, 2), np.int64) for _ in lens]
    if w.dup > 0.0 and n_ctx > 1:
        rd = _rng(w, layer, _T_DUP)
        staged = []
        for i, L in enumerate(lens):
            n_dup = int(round(w.dup * L))
            if n_dup == 0:
                continue
            dst = np.sort(rd.choice(L, size=n_dup, replace=False))
            others = np.array([j for j in range(n_ctx) if j != i])
            # distinct (document, position) sources, so no row appears twice inside document i
            flat_sizes = np.array([lens[j] for j in others])
            flat = rd.choice(int(flat_sizes.sum()), size=n_dup, replace=False)
            bounds = np.concatenate([[0], np.cumsum(flat_sizes)])
            which = np.searchsorted(bounds, flat, side="right") - 1
            src = np.stack([others[which], flat - bounds[which]], axis=1)
            rows_k = np.stack([ks[j][:, p, :] for j, p in src], axis=1)   # copies of the original rows
            rows_v = np.stack([vs[j][:, p, :] for j, p in src], axis=1)
            staged.append((i, dst, src, rows_k, rows_v))
        for i, dst, src, rows_k, rows_v in staged:
            ks[i][:, dst, :] = rows_k
            vs[i][:, dst, :] = rows_v
            dup_pos[i], dup_src[i] = dst, src

    # local Q cache of each document: a direction tied to the rows it shares with others, plus noise
    rl = _rng(w, layer, _T_QLOC)
    q_loc = np.empty((n_ctx, hq, w.w_loc, d), dtype=np.float32)
    qn = np.linalg.norm(qbar_h, axis=1)                                 # [Hq]
    all_src = np.concatenate(dup_src, axis=0)
    for j in range(n_ctx):
        shared = all_src[all_src[:, 0] == j, 1]
        if shared.size:
            dirs = np.stack([ks[j][gg, shared, :].astype(np.float64).mean(axis=0) for gg in range(hkv)])
        else:
            dirs = rl.standard_normal((hkv, d))
        dirs = dirs / np.maximum(np.linalg.norm(dirs, axis=1, keepdims=True), 1e-30)
        centre = 0.5 * qn[:, None] * np.repeat(dirs, g, axis=0)        # [Hq, d]
        noise = rl.standard_normal((hq, w.w_loc, d), dtype=np.float32)
        q_loc[j] = centre[:, None, :].astype(np.float32) + np.repeat(sk32, g, axis=0)[:, None, :] * noise

    dt = w.dtype
    return LayerInputs(
        workload=w, layer=layer, lens=lens,
        k=[round_to_dtype(a, dt) for a in ks], v=[round_to_dtype(a, dt) for a in vs],
        q_tok=round_to_dtype(q_tok, dt), q_loc=round_to_dtype(q_loc, dt),
        planted_pos=planted_pos, dup_pos=dup_pos, dup_src=dup_src, sigma_k=sk, sigma_v=sv,
    )


def make_q_rec(w: Workload, layer: int, n_rows: int) -> np.ndarray:
    """Q states of the kept tokens, [Hq, n_rows, d]; same channel scales as K (a stored Q cache)."""
    sk, _ = _channel_scales(w, layer)
    z = _rng(w, layer, _T_QREC).standard_normal((w.n_q_heads, n_rows, w.head_dim), dtype=np.float32)
    z *= np.repeat(sk, w.group, axis=0).astype(np.float32)[:, None, :]
    return round_to_dtype(z, w.dtype)


def stack_layers(w: Workload, layers: List[LayerInputs], q_recs: List[np.ndarray]):
    """Layers of a multi-layer workload laid out for ONE call per entry point: every document's cache holds all
    layers as [(layer, KV head)][L][d], the Q tensors likewise [(layer, query head)][...].  Query head h of the stack
    reads KV head h / G, which stays inside its layer, so the library needs to know nothing about layers.
    Returns (k list, v list, q_tok, q_loc, q_rec), all float32 arrays with dtype-exact values."""
    n_ctx = len(layers[0].k)
    k = [np.concatenate([x.k[i] for x in layers], axis=0) for i in range(n_ctx)]
    v = [np.concatenate([x.v[i] for x in layers], axis=0) for i in range(n_ctx)]
    q_tok = np.concatenate([x.q_tok for x in layers], axis=0)
    q_loc = np.concatenate([x.q_loc for x in layers], axis=1)
    q_rec = np.concatenate(q_recs, axis=0)
    return k, v, q_tok, q_loc, q_rec


def make_q_cache(w: Workload, layer: int, lens: List[int]) -> List[np.ndarray]:
    """Stored per-document Q caches, [Hq, L_i, d] each, with K's channel scales."""
    sk, _ = _channel_scales(w, layer)
    scale = np.repeat(sk, w.group, axis=0).astype(np.float32)[:, None, :]
    out = []
    for i, L in enumerate(lens):
        z = np.random.default_rng(np.random.SeedSequence([BASE_SEED + w.cfg_id, layer, 200, i])).standard_normal(
            (w.n_q_heads, L, w.head_dim), dtype=np.float32)
        out.append(round_to_dtype(z * scale, w.dtype))
    return out


def make_recomputed_rows(w: Workload, layer: int, old: np.ndarray, sigma: np.ndarray, tensor: int) -> np.ndarray:
    """Stand-in for the K (tensor=0) or V (tensor=1) rows a model would recompute for the kept tokens:
    the old rows [Hkv, M, d] plus channel-scaled noise of relative size 0.45, which puts the cosine between
    new and old rows near the 0.9 the paper reports for its fusion weight (Sec. 3.3)."""
    rng = np.random.default_rng(np.random.SeedSequence([BASE_SEED + w.cfg_id, layer, 100 + tensor]))
    z = rng.standard_normal(old.shape, dtype=np.float32)
    new = old.astype(np.float32) + 0.45 * sigma.astype(np.float32)[:, None, :] * z
    return round_to_dtype(new, w.dtype)


def make_small(seed: int, dtype: str, lens: List[int], n_q_heads: int, n_kv_heads: int, head_dim: int,
               n_q_tok: int, w_loc: int, planted: float = 0.1, dup: float = 0.05) -> LayerInputs:
    """Ad-hoc small workload for tests (ragged document lengths, odd sizes)."""
    w = Workload(f"adhoc{seed}", 1000 + seed, dtype, 1, len(lens), max(lens), n_q_heads, n_kv_heads,
                 head_dim, n_q_tok, (0.15,), planted, dup, w_loc)
    return make_layer(w, 0, lens)
