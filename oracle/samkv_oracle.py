"""Plain fp64 CPU oracle of the SamKV hot path.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path may import this module: it exists so that tests,
the smoke check and the benchmark's CPU-baseline leg can compare the HIP
kernels against an independent, slow, obviously-correct statement of what the
paper computes.  It shares no code with the HIP library or its binding.

Every function works in numpy float64, one step of the method per function, in
the order and notation of the paper:

  pooled_query         Sec. 3.1 "Generate generic query vector": Q_que by mean pooling
  local_query          Sec. 3.1 "Add personalized bias": a document's local Q cache as one vector
  personalized_query   Eq. 1: Q^_doc-i = Q_que + 1/(D-1) * sum_{j != i} |cos(Q_que, Q_doc-j_loc)| Q_doc-j_loc
  score                Sec. 3.2 / Table 2: inner product <Q^_doc-i, K>
  top_p                Sec. 3.2, Eq. 2 and Eq. 3: dynamic share per document from anchor / max / min block scores
  kept_count           budget ratio -> number of kept tokens per document and head
  select_row / select  Sec. 3.2: keep the top-scoring share of each document (initial/local kept first)
  block_scores / block_select   Sec. 3.2 block-level retrieval: mean-key block representatives, forced blocks
  block_filter         Sec. 3.2 second filter across documents (normalisation is a reading: parity unpinned)
  gather_global        compaction by positions in the concatenation of all documents
  gather, gather_q     Sec. 3.2: concatenate the kept K/V (and stored Q) of all documents in their original order
  kv_update            Sec. 3.3, Eq. 4: overwrite or cosine-weighted fusion of recomputed K/V rows
  attention            Sec. 3.3 recomputation (causal over the compacted cache) and the final
                       incremental prefill of the user query (no mask): softmax(q k^T * scale) v
  attention_with_self  the same prefill with the query tokens' own K/V appended causally

Readings taken where the paper is silent (listed once more in the design notes):
the local Q cache becomes a vector by the same mean pooling as Q_que; under
grouped-query attention the score of a KV head is the mean over its query
heads; scores are raw inner products (no 1/sqrt(d), no softmax); ties in the
selection go to the lower position; with one document the bias term vanishes;
a cosine with a zero-norm argument counts as 0.

Parity status: every function here is pinned by tests/test_oracle_pins.py
(closed forms, hand-worked cases, brute force, library routines), except block_filter:
parity unpinned (the paper does not define its normalisation; the mechanics around the
reading are pinned, the reading itself cannot be).  The quality
of the whole pipeline (the paper's F1 tables) needs datasets and weights and is
parity unpinned.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------- Eq. 1
def pooled_query(q_tok: np.ndarray) -> np.ndarray:
    """Q_que[h, :] = mean over the query's tokens of Q[h, t, :].   q_tok [Hq, Lq, d] -> [Hq, d]."""
    q_tok = np.asarray(q_tok, F64)
    return q_tok.sum(axis=1) / q_tok.shape[1]


def local_query(q_loc: np.ndarray) -> np.ndarray:
    """Q_doc-j_loc as one vector per head: mean over the rows of the local Q cache.

    q_loc [N, Hq, Wloc, d] -> [N, Hq, d]."""
    q_loc = np.asarray(q_loc, F64)
    return q_loc.sum(axis=2) / q_loc.shape[2]


def abs_cos(a: np.ndarray, b: np.ndarray) -> float:
    """|cos(a, b)| over the channels of one head; 0 when either norm is (numerically) zero."""
    na = math.sqrt(float(np.dot(a, a)))
    nb = math.sqrt(float(np.dot(b, b)))
    if na < 1e-20 or nb < 1e-20:
        return 0.0
    return abs(float(np.dot(a, b)) / (na * nb))


def personalized_query(q_tok: np.ndarray, q_loc: Optional[np.ndarray], n_ctx: int) -> np.ndarray:
    """Eq. 1 for every document i and query head h.  Returns Q^ [N, Hq, d]."""
    q_que = pooled_query(q_tok)                       # [Hq, d]
    hq, d = q_que.shape
    q_hat = np.empty((n_ctx, hq, d), F64)
    if q_loc is None or n_ctx == 1:
        q_hat[:] = q_que[None]
        return q_hat
    loc = local_query(q_loc)                          # [N, Hq, d]
    assert loc.shape == (n_ctx, hq, d)
    for i in range(n_ctx):
        for h in range(hq):
            bias = np.zeros(d, F64)
            for j in range(n_ctx):
                if j == i:
                    continue
                bias += abs_cos(q_que[h], loc[j, h]) * loc[j, h]
            q_hat[i, h] = q_que[h] + bias / (n_ctx - 1)
    return q_hat


# --------------------------------------------------------------------------- scoring
def score(q_hat: np.ndarray, k: Sequence[np.ndarray]) -> List[np.ndarray]:
    """s[i][g, t] = (1/G) * sum_{h in group g} <Q^_i[h], K_i[g, t, :]>.

    q_hat [N, Hq, d]; k[i] [Hkv, L_i, d].  Returns one [Hkv, L_i] array per document."""
    n_ctx, hq, d = q_hat.shape
    out = []
    for i in range(n_ctx):
        ki = np.asarray(k[i], F64)
        hkv, L, _ = ki.shape
        G = hq // hkv
        s = np.zeros((hkv, L), F64)
        for g in range(hkv):
            for h in range(g * G, (g + 1) * G):
                s[g] += ki[g] @ q_hat[i, h]
            s[g] /= G
        out.append(s)
    return out


# --------------------------------------------------------------------------- selection
def kept_count(length: int, ratio: float) -> int:
    """Tokens kept per document and KV head: ceil(ratio * length), at least 1, at most length.

    The ratio is taken at float32 precision (what crosses the C boundary); the product is shrunk
    by 2^-22 (four float32 ulps) so that a budget that is integral in exact arithmetic, such as
    0.1 * 20, is not pushed up by the float32 rounding of the ratio."""
    r = float(np.float32(ratio))
    return int(min(length, max(1, math.ceil(r * length * (1.0 - 2.0 ** -22)))))


def top_p(s_anc: np.ndarray, s_max: np.ndarray, s_min: np.ndarray) -> np.ndarray:
    """Dynamic Top-P of Sec. 3.2.  Inputs [n_layers, n_ctx]: per stable layer and document the scores of the
    anchor block, of the most-attended and of the least-attended middle block.

    Eq. 2: P^(n)_i = (s_max - s_anc) / (s_max - s_min) if s_anc lies in (s_min, s_max], otherwise 0.
    Eq. 3: P_i = mean of P^(n)_i over the layers.  Returns [n_ctx]."""
    s_anc, s_max, s_min = (np.asarray(a, F64) for a in (s_anc, s_max, s_min))
    n_layers, n_ctx = s_anc.shape
    p = np.zeros(n_ctx, F64)
    for i in range(n_ctx):
        for n in range(n_layers):
            if s_min[n, i] < s_anc[n, i] <= s_max[n, i]:
                p[i] += (s_max[n, i] - s_anc[n, i]) / (s_max[n, i] - s_min[n, i])
        p[i] /= n_layers
    return p


def kept_count_mid(length: int, p: float, n_sink: int, n_local: int) -> int:
    """Kept tokens when the n_sink initial and n_local last positions are kept in full and the middle segment is
    sparsified to the share p (Sec. 3.2): forced + ceil(p * middle), with the float32 guard of kept_count."""
    forced = n_sink + n_local
    if forced >= length:
        return length
    mid = length - forced
    k = math.ceil(float(np.float32(p)) * mid * (1.0 - 2.0 ** -22))
    return forced + int(min(mid, max(0, k)))


def select_v(scores: Sequence[np.ndarray], p: Sequence[float], n_sink: int = 0, n_local: int = 0
             ) -> Tuple[np.ndarray, np.ndarray]:
    """As select, with one middle-segment share per document (the P_i of Eq. 3)."""
    hkv = scores[0].shape[0]
    ks = [kept_count_mid(s.shape[1], pi, n_sink, n_local) for s, pi in zip(scores, p)]
    cu_k = np.concatenate([[0], np.cumsum(ks)]).astype(np.int32)
    idx = np.empty((hkv, int(cu_k[-1])), np.int32)
    for i, s in enumerate(scores):
        if ks[i] == 0:
            continue
        L = s.shape[1]
        for g in range(hkv):
            idx[g, cu_k[i]:cu_k[i + 1]] = select_row(np.asarray(s[g], F64), ks[i], min(n_sink, L), min(n_local, max(0, L - n_sink)))
    return idx, cu_k


def select_row(scores: np.ndarray, k: int, n_sink: int = 0, n_local: int = 0) -> np.ndarray:
    """Positions of the k kept tokens of one (document, KV head) row, ascending.

    The first n_sink and last n_local positions are kept unconditionally (they count towards k);
    the rest of the budget goes to the largest scores, equal scores to the lower position."""
    L = scores.shape[0]
    assert 0 < k <= L and n_sink + n_local <= k
    forced = set(range(n_sink)) | set(range(L - n_local, L))
    order = sorted((p for p in range(L) if p not in forced), key=lambda p: (-scores[p], p))
    kept = sorted(forced | set(order[: k - len(forced)]))
    return np.asarray(kept, np.int32)


def select(scores: Sequence[np.ndarray], ratio: float, n_sink: int = 0, n_local: int = 0
           ) -> Tuple[np.ndarray, np.ndarray]:
    """Selection for every document and KV head.

    Returns idx [Hkv, M] (document-local positions, documents in order, ascending inside each)
    and cu_k [N+1] with M = cu_k[-1]."""
    hkv = scores[0].shape[0]
    ks = [kept_count(s.shape[1], ratio) for s in scores]
    cu_k = np.concatenate([[0], np.cumsum(ks)]).astype(np.int32)
    idx = np.empty((hkv, int(cu_k[-1])), np.int32)
    for i, s in enumerate(scores):
        for g in range(hkv):
            idx[g, cu_k[i]:cu_k[i + 1]] = select_row(np.asarray(s[g], F64), ks[i], n_sink, n_local)
    return idx, cu_k


def block_scores(q_hat: np.ndarray, k: Sequence[np.ndarray], block: int) -> List[np.ndarray]:
    """Block-level retrieval of Sec. 3.2: a block of `block` consecutive tokens is represented by the mean of its
    keys and scored like a token, b[i][g, n] = (1/G) * sum_{h in group g} <Q^_i[h], mean_t K_i[g, t, :]>, t over
    block n (the last block of a document may be short).  Returns one [Hkv, ceil(L_i / block)] array per document."""
    reps = []
    for ki in k:
        ki = np.asarray(ki, F64)
        hkv, L, d = ki.shape
        nb = -(-L // block)
        rep = np.zeros((hkv, nb, d), F64)
        for n in range(nb):
            rep[:, n, :] = ki[:, n * block:min(L, (n + 1) * block), :].mean(axis=1)
        reps.append(rep)
    return score(q_hat, reps)


def block_select(bscores: Sequence[np.ndarray], lens: Sequence[int], block: int, p: Sequence[float],
                 n_init_blocks: int = 1, n_local_blocks: int = 2) -> Tuple[np.ndarray, np.ndarray]:
    """Selection at block granularity (Sec. 3.2; Setup: the initial block and the last two are always kept).

    Per document and KV head the forced blocks are kept, and of the middle blocks the share p[i] with the largest
    block scores; the kept blocks are returned as the positions of their tokens: idx [Hkv, M] and cu_k [N+1]
    counting tokens.  Requires that every head keeps the same number of tokens (true when the short last block
    is forced, or when no block is short)."""
    hkv = bscores[0].shape[0]
    rows: List[List[np.ndarray]] = [[] for _ in range(hkv)]
    cu_k = [0]
    for i, (b, L) in enumerate(zip(bscores, lens)):
        nb = b.shape[1]
        assert nb == -(-L // block)
        kb = kept_count_mid(nb, p[i], n_init_blocks, n_local_blocks)
        n_tok = None
        for g in range(hkv):
            if kb == 0:
                toks = np.zeros(0, np.int32)
            else:
                ni = min(n_init_blocks, nb)
                blocks = select_row(np.asarray(b[g], F64), kb, ni, min(n_local_blocks, nb - ni))
                toks = np.concatenate([np.arange(n * block, min(L, (n + 1) * block)) for n in blocks]).astype(np.int32)
            assert n_tok is None or n_tok == toks.shape[0], "heads keep different numbers of tokens"
            n_tok = toks.shape[0]
            rows[g].append(toks)
        cu_k.append(cu_k[-1] + n_tok)
    idx = np.stack([np.concatenate(r) for r in rows]).astype(np.int32)
    return idx, np.asarray(cu_k, np.int32)


def block_filter(bscores: Sequence[np.ndarray], lens: Sequence[int], block: int, p: Sequence[float],
                 n_init_blocks: int = 1, n_local_blocks: int = 2) -> np.ndarray:
    """Second filter of Sec. 3.2 on top of block_select.  PARITY UNPINNED as far as the normalisation goes: the
    paper says the retrieved blocks' inner products are normalised across documents before they are compared, and
    that as many blocks survive as the total block count divided by the number of documents, but gives no formula.
    Reading implemented (the library documents the same one):
      * candidates: per KV head, the middle (non-forced) blocks that the per-document Top-P_i selection retrieved;
      * normalisation: min-max per document and head over its candidates, (s - min) / (max - min), evaluated in
        float32 (the decision is taken in the precision the kernel works in), 1 when max == min;
      * survivors: the ceil(C / N) candidates with the largest normalised score, C = number of candidates (the
        same for every head), ties to the earlier document and then the lower block;
      * forced blocks survive unconditionally.
    Returns the GLOBAL token positions (offset of the document in the concatenation + position) of the surviving
    blocks, ascending, one row per KV head: [Hkv, M]."""
    f32 = np.float32
    hkv, n_ctx = bscores[0].shape[0], len(lens)
    cu_len = np.concatenate([[0], np.cumsum(lens)])
    rows = []
    for g in range(hkv):
        forced_blocks, cands = [], []          # (document, block) and (normalised score, document, block)
        for i, (b, L) in enumerate(zip(bscores, lens)):
            nb = b.shape[1]
            kb = kept_count_mid(nb, p[i], n_init_blocks, n_local_blocks)
            if kb == 0:
                continue
            ni = min(n_init_blocks, nb)
            nl = min(n_local_blocks, nb - ni)
            kept = select_row(np.asarray(b[g], F64), kb, ni, nl)
            mid = [int(n) for n in kept if ni <= n < nb - nl]
            forced_blocks += [(i, int(n)) for n in kept if not (ni <= n < nb - nl)]
            if mid:
                sc = np.asarray([b[g, n] for n in mid]).astype(f32)
                mn, mx = sc.min(), sc.max()
                rng_ = f32(mx - mn)
                for n, s in zip(mid, sc):
                    cands.append((float(f32(s - mn) / rng_) if rng_ > 0 else 1.0, i, n))
        keep = -(-len(cands) // n_ctx)
        best = sorted(cands, key=lambda c: (-c[0], c[1], c[2]))[:keep]
        blocks = sorted(forced_blocks + [(i, n) for _, i, n in best])
        toks = [np.arange(cu_len[i] + n * block, cu_len[i] + min(lens[i], (n + 1) * block)) for i, n in blocks]
        rows.append(np.concatenate(toks).astype(np.int32))
    assert len({r.shape[0] for r in rows}) == 1, "heads keep different numbers of tokens"
    return np.stack(rows)


def gather_global(x: Sequence[np.ndarray], gidx: np.ndarray, group: int = 1) -> np.ndarray:
    """Compaction by global token positions: out[h, m, :] = x_i[h, gidx[h // group, m] - cu_len[i], :] with i the
    document that holds the position.  x[i] [H, L_i, d]; returns [H, M, d]."""
    lens = [a.shape[1] for a in x]
    cu_len = np.concatenate([[0], np.cumsum(lens)])
    H, _, d = x[0].shape
    out = np.empty((H, gidx.shape[1], d), x[0].dtype)
    for h in range(H):
        for m, gp in enumerate(gidx[h // group]):
            i = int(np.searchsorted(cu_len, gp, side="right")) - 1
            out[h, m] = x[i][h, gp - cu_len[i]]
    return out


# --------------------------------------------------------------------------- compaction
def gather(k: Sequence[np.ndarray], v: Sequence[np.ndarray], idx: np.ndarray, cu_k: np.ndarray
           ) -> Tuple[np.ndarray, np.ndarray]:
    """K_c[g, cu_k[i] + m, :] = K_i[g, idx[g, cu_k[i] + m], :], same for V.  Returns [Hkv, M, d] each."""
    hkv, M = idx.shape
    d = k[0].shape[2]
    k_c = np.empty((hkv, M, d), k[0].dtype)
    v_c = np.empty((hkv, M, d), v[0].dtype)
    for i in range(len(k)):
        for g in range(hkv):
            for m in range(int(cu_k[i]), int(cu_k[i + 1])):
                k_c[g, m, :] = k[i][g, idx[g, m], :]
                v_c[g, m, :] = v[i][g, idx[g, m], :]
    return k_c, v_c


def gather_q(q: Sequence[np.ndarray], idx: np.ndarray, cu_k: np.ndarray) -> np.ndarray:
    """Same compaction for the stored per-document Q caches: q[i] [Hq, L_i, d] -> [Hq, M, d], query head h
    taking the kept positions of its KV head h // (Hq / Hkv)."""
    hq, _, d = q[0].shape
    hkv, M = idx.shape
    G = hq // hkv
    out = np.empty((hq, M, d), q[0].dtype)
    for i in range(len(q)):
        for h in range(hq):
            for m in range(int(cu_k[i]), int(cu_k[i + 1])):
                out[h, m, :] = q[i][h, idx[h // G, m], :]
    return out


# --------------------------------------------------------------------------- cache update (Eq. 4)
def kv_update(old: np.ndarray, new: np.ndarray, fusion: bool) -> np.ndarray:
    """Cache update after recomputation, for K or for V alike.  old, new [Hkv, M, d] -> [Hkv, M, d] float64.

    Overwrite: the recomputed rows replace the old ones.  Fusion (Eq. 4): theta = cos(new, old),
    result = theta * new + (1 - theta) * old, with the cosine taken per cached token and KV head
    (the paper leaves its granularity open); theta = 1 when either row has (numerically) zero norm."""
    old = np.asarray(old, F64)
    new = np.asarray(new, F64)
    if not fusion:
        return new.copy()
    out = np.empty_like(old)
    for g in range(old.shape[0]):
        for m in range(old.shape[1]):
            a, b = new[g, m], old[g, m]
            na, nb = math.sqrt(float(a @ a)), math.sqrt(float(b @ b))
            theta = 1.0 if (na < 1e-20 or nb < 1e-20) else float(a @ b) / (na * nb)
            out[g, m] = theta * a + (1.0 - theta) * b
    return out


# --------------------------------------------------------------------------- attention
def attention(q: np.ndarray, k_c: np.ndarray, v_c: np.ndarray, scale: float, causal: bool,
              rows: Optional[Sequence[int]] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Softmax attention of query rows over the compacted cache.

    q [Hq, R, d]; k_c, v_c [Hkv, M, d]; query head h reads KV head h // (Hq / Hkv).
    causal=True is the recomputation of the kept tokens: row p (R == M) sees keys 0..p, itself
    included, across document boundaries.  causal=False is the user query's prefill over the cache.
    `rows` restricts the computation to those row numbers (outputs then have len(rows) rows).
    Returns O [Hq, R', d] and LSE [Hq, R'] = log sum_j exp(scale * q.k_j)."""
    q = np.asarray(q, F64)
    k_c = np.asarray(k_c, F64)
    v_c = np.asarray(v_c, F64)
    hq, R, d = q.shape
    hkv, M, _ = k_c.shape
    G = hq // hkv
    if causal:
        assert R == M
    sel = list(range(R)) if rows is None else [int(r) for r in rows]
    out = np.empty((hq, len(sel), d), F64)
    lse = np.empty((hq, len(sel)), F64)
    for h in range(hq):
        g = h // G
        for n, p in enumerate(sel):
            last = p + 1 if causal else M
            s = (k_c[g, :last] @ q[h, p]) * scale
            m = s.max()
            e = np.exp(s - m)
            z = e.sum()
            out[h, n] = (e / z) @ v_c[g, :last]
            lse[h, n] = m + math.log(z)
    return out, lse


def attention_with_self(q: np.ndarray, k_c: np.ndarray, v_c: np.ndarray, k_self: np.ndarray, v_self: np.ndarray,
                        scale: float) -> Tuple[np.ndarray, np.ndarray]:
    """Incremental prefill of the user query after the compacted cache (Sec. 3.3, last paragraph): query
    token t attends to every cached token and to query tokens 0..t, itself included.

    q [Hq, Lq, d]; k_c, v_c [Hkv, M, d]; k_self, v_self [Hkv, Lq, d].  Returns O [Hq, Lq, d], LSE [Hq, Lq]."""
    q = np.asarray(q, F64)
    hq, lq, d = q.shape
    hkv = k_c.shape[0]
    G = hq // hkv
    out = np.empty((hq, lq, d), F64)
    lse = np.empty((hq, lq), F64)
    for h in range(hq):
        g = h // G
        for t in range(lq):
            keys = np.concatenate([np.asarray(k_c[g], F64), np.asarray(k_self[g, : t + 1], F64)], axis=0)
            vals = np.concatenate([np.asarray(v_c[g], F64), np.asarray(v_self[g, : t + 1], F64)], axis=0)
            s = (keys @ q[h, t]) * scale
            m = s.max()
            e = np.exp(s - m)
            z = e.sum()
            out[h, t] = (e / z) @ vals
            lse[h, t] = m + math.log(z)
    return out, lse
